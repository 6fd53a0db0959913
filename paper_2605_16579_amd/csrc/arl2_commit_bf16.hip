// Post-denoise state commit on bf16 MFMA (gfx950):
//   S <- gate * S + sum_i k'_i^T v_i,   k'_i = k_i / sqrt(|k_i|^2 + eps)     paper Eq. (3), Eq. (4)
//
// The contraction runs over tokens, so both operands are needed token-major per feature:
// every workgroup transposes 64-token tiles of K and V through LDS.  To keep the fp32 state
// accurate the raw bf16 K (exact) is one operand and the row-scaled values r_i * v_i, split
// into bf16 hi + lo parts, are the other (two MFMAs per tile step, error ~2^-17).
//
// Tokens are split over `nsplit` workgroups per (stream, head); each writes a D x D fp32
// partial to the workspace.  A second kernel adds the partials in split order and applies the
// gate to the old state, so the result is bit-identical from run to run.
#include "arl2_device.h"

namespace arl2 {
namespace {

constexpr int BT = 64;    // tokens per tile
constexpr int NT = 256;

template <int D>
struct CommitCfg {
    static constexpr int DB = D / 32;
    static constexpr int CPR = D / 8;
    static constexpr int ROW = 2 * BT + 8;              // LDS bytes per transposed row (64 tokens + pad)
    static constexpr int MAT = D * ROW;                 // one transposed D x 64 matrix
    static constexpr int NEB = DB * DB / 4;             // e-blocks per wave
};

template <int D>
__global__ __launch_bounds__(NT, 1) void commit_partial_kernel(CommitArgs a)
{
    using C = CommitCfg<D>;
    __shared__ __attribute__((aligned(16))) unsigned char smem[3 * C::MAT];
    unsigned char *smKt = smem, *smVh = smem + C::MAT, *smVl = smem + 2 * C::MAT;

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, c = lane & 31, hh = lane >> 5;
    const int split = blockIdx.x % a.nsplit;
    const int bh = blockIdx.x / a.nsplit;
    const int h = bh % a.H, b = bh / a.H;
    const int L = a.L, H = a.H;
    const size_t tok_stride = (size_t)H * D;
    const bf16_t *kg = (const bf16_t *)a.k + ((size_t)b * L * H + h) * D;
    const bf16_t *vg = (const bf16_t *)a.v + ((size_t)b * L * H + h) * D;

    const int ntiles = (L + BT - 1) / BT;
    const int t_begin = (int)((long long)split * ntiles / a.nsplit);
    const int t_end = (int)((long long)(split + 1) * ntiles / a.nsplit);

    const int dg = tid % C::CPR, u = tid / C::CPR;      // 8-feature group, 4-token group
    const bool active = u < BT / 4;

    const int dblk = wave % C::DB;
    const int eb0 = (wave / C::DB) * C::NEB;
    f32x16 acc[C::NEB];
#pragma unroll
    for (int n = 0; n < C::NEB; ++n)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[n][r] = 0.f;

    for (int tile = t_begin; tile < t_end; ++tile) {
        const int tok0 = tile * BT;
        u32x4 kr[4], vr[4];
        if (active) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int tok = tok0 + 4 * u + e;
                u32x4 x = {0, 0, 0, 0}, y = {0, 0, 0, 0};
                if (tok < L) {
                    x = *(const u32x4 *)(kg + (size_t)tok * tok_stride + 8 * dg);
                    y = *(const u32x4 *)(vg + (size_t)tok * tok_stride + 8 * dg);
                }
                kr[e] = x;
                vr[e] = y;
            }
        }
        // 1 / sqrt(|k_tok|^2 + eps): partial sums over this thread's 8 features, then over the
        // CPR consecutive lanes that share the token rows
        float rn[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float ss = 0.f;
            if (active) {
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    const float lo = __uint_as_float(kr[e][w] << 16);
                    const float hi = __uint_as_float(kr[e][w] & 0xffff0000u);
                    ss = fmaf(lo, lo, ss);
                    ss = fmaf(hi, hi, ss);
                }
            }
#pragma unroll
            for (int off = 1; off < C::CPR; off <<= 1) ss += __shfl_xor(ss, off, kWave);
            rn[e] = 1.0f / sqrtf(ss + a.l2_eps);
        }

        __syncthreads();            // previous tile fully consumed
        if (active) {
#pragma unroll
            for (int m = 0; m < 8; ++m) {
                const int w = m >> 1;
                const uint32_t sel = (m & 1) ? 0x07060302u : 0x05040100u;
                u32x2 o;
                o[0] = __builtin_amdgcn_perm(kr[1][w], kr[0][w], sel);
                o[1] = __builtin_amdgcn_perm(kr[3][w], kr[2][w], sel);
                *(u32x2 *)(smKt + (8 * dg + m) * C::ROW + 8 * u) = o;
                bf16x4 vh, vl;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t word = vr[e][w];
                    const float val = (m & 1) ? __uint_as_float(word & 0xffff0000u) : __uint_as_float(word << 16);
                    const float sv = val * rn[e];
                    const bf16_t hi = to_bf16(sv);
                    vh[e] = hi;
                    vl[e] = to_bf16(sv - (float)hi);
                }
                *(bf16x4 *)(smVh + (8 * dg + m) * C::ROW + 8 * u) = vh;
                *(bf16x4 *)(smVl + (8 * dg + m) * C::ROW + 8 * u) = vl;
            }
        }
        __syncthreads();

#pragma unroll
        for (int t = 0; t < BT / 16; ++t) {
            const int off = 32 * t + 16 * hh;
            union { u32x2 u2[2]; bf16x8 v; } ka;
            const unsigned char *kp = smKt + (32 * dblk + c) * C::ROW + off;
            ka.u2[0] = *(const u32x2 *)kp;
            ka.u2[1] = *(const u32x2 *)(kp + 8);
#pragma unroll
            for (int n = 0; n < C::NEB; ++n) {
                union { u32x2 u2[2]; bf16x8 v; } bh_, bl_;
                const unsigned char *hp = smVh + (32 * (eb0 + n) + c) * C::ROW + off;
                const unsigned char *lp = smVl + (32 * (eb0 + n) + c) * C::ROW + off;
                bh_.u2[0] = *(const u32x2 *)hp;
                bh_.u2[1] = *(const u32x2 *)(hp + 8);
                bl_.u2[0] = *(const u32x2 *)lp;
                bl_.u2[1] = *(const u32x2 *)(lp + 8);
                acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka.v, bh_.v, acc[n], 0, 0, 0);
                acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka.v, bl_.v, acc[n], 0, 0, 0);
            }
        }
    }

    // partial[bh][split][d][e]
    float *part = (float *)a.workspace + ((size_t)bh * a.nsplit + split) * D * D;
#pragma unroll
    for (int n = 0; n < C::NEB; ++n)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int d = 32 * dblk + 8 * (r >> 2) + 4 * hh + (r & 3);
            const int e = 32 * (eb0 + n) + c;
            part[(size_t)d * D + e] = acc[n][r];
        }
}

// S[bh] = gate[bh] * S[bh] + sum_{split ascending} partial[bh][split]
__global__ __launch_bounds__(NT) void commit_reduce_kernel(CommitArgs a, int vec_per_head)
{
    const int bh = blockIdx.x / (vec_per_head / NT);
    const int vi = (blockIdx.x % (vec_per_head / NT)) * NT + threadIdx.x;
    const size_t head_elems = (size_t)vec_per_head * 4;
    const f32x4 *part = (const f32x4 *)((const float *)a.workspace + (size_t)bh * a.nsplit * head_elems);
    f32x4 sum = part[vi];
    for (int s = 1; s < a.nsplit; ++s) sum += part[(size_t)s * vec_per_head + vi];
    const float gate = a.gate[bh];
    f32x4 *Sg = (f32x4 *)(a.S + (size_t)bh * head_elems);
    const f32x4 old = Sg[vi];
    f32x4 res;
#pragma unroll
    for (int j = 0; j < 4; ++j) res[j] = fmaf(gate, old[j], sum[j]);
    Sg[vi] = res;
}

}  // namespace

int commit_nsplit(int B, int H, int L)
{
    const int ntiles = (L + BT - 1) / BT;
    long long bh = (long long)B * H;
    long long want = (256 + bh - 1) / bh;      // aim at about one workgroup per compute unit
    if (want < 1) want = 1;
    if (want > ntiles) want = ntiles;
    if (want > 32) want = 32;
    return (int)want;
}

hipError_t launch_commit_bf16(const CommitArgs &a, hipStream_t stream)
{
    const long long nwg = (long long)a.B * a.H * a.nsplit;
    if (nwg <= 0 || nwg > 0x7fffffffLL) return hipErrorInvalidValue;
    if (a.D == 128)
        hipLaunchKernelGGL(commit_partial_kernel<128>, dim3((unsigned)nwg), dim3(NT), 0, stream, a);
    else if (a.D == 64)
        hipLaunchKernelGGL(commit_partial_kernel<64>, dim3((unsigned)nwg), dim3(NT), 0, stream, a);
    else
        return hipErrorInvalidValue;
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int vec_per_head = a.D * a.D / 4;        // multiple of 256 for D in {64, 128}
    const long long rwg = (long long)a.B * a.H * (vec_per_head / NT);
    hipLaunchKernelGGL(commit_reduce_kernel, dim3((unsigned)rwg), dim3(NT), 0, stream, a, vec_per_head);
    return hipGetLastError();
}

}  // namespace arl2
