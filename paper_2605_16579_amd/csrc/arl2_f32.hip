// fp32-throughout variants of the two operations (for fp32 inputs; small problem sizes).
// Plain fp32 FMA arithmetic, two-pass softmax (row maximum first, then exp and sums), no
// reduced-precision step anywhere.  Same definitions as the bf16 kernels:
//   out = softmax(q k^T * sm_scale) v + g * L2Norm(q) S             paper Eq. (2), (3), (5), (6)
//   S  <- gate * S + sum_i L2Norm(k_i)^T v_i                        paper Eq. (3), Eq. (4)
#include "arl2_device.h"

namespace arl2 {
namespace {

constexpr int NT = 256;
constexpr int GROUP = 16;                 // lanes cooperating on one query row
constexpr int ROWS = NT / GROUP;          // query rows per workgroup

__device__ __forceinline__ float group_sum(float x)
{
#pragma unroll
    for (int off = 1; off < GROUP; off <<= 1) x += __shfl_xor(x, off, kWave);
    return x;
}

// 16 lanes own one query row; each lane keeps EPL = D/16 consecutive features.
template <int D>
__global__ __launch_bounds__(NT) void fwd_f32_kernel(FwdArgs a)
{
    constexpr int EPL = D / GROUP;
    const int tid = threadIdx.x;
    const int sub = tid % GROUP, rloc = tid / GROUP;
    const int h = blockIdx.y, b = blockIdx.z;
    const int H = a.H, Lq = a.Lq, Lkv = a.Lkv;
    const int row = blockIdx.x * ROWS + rloc;
    const bool valid = row < Lq;
    const int rowc = valid ? row : 0;
    const size_t ts = (size_t)H * D;

    const float *qg = (const float *)a.q + (((size_t)b * Lq + rowc) * H + h) * D + sub * EPL;
    const float *kg = (const float *)a.k + ((size_t)b * Lkv * H + h) * D + sub * EPL;
    const float *vg = (const float *)a.v + ((size_t)b * Lkv * H + h) * D + sub * EPL;

    float qr[EPL];
#pragma unroll
    for (int i = 0; i < EPL; ++i) qr[i] = qg[i];

    // pass 1: row maximum of the scaled logits
    float m = -INFINITY;
    for (int j = 0; j < Lkv; ++j) {
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < EPL; ++i) s = fmaf(qr[i], kg[(size_t)j * ts + i], s);
        s = group_sum(s) * a.sm_scale;
        m = fmaxf(m, s);
    }
    // pass 2: weights, normaliser, weighted values
    float l = 0.f;
    float o[EPL];
#pragma unroll
    for (int i = 0; i < EPL; ++i) o[i] = 0.f;
    for (int j = 0; j < Lkv; ++j) {
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < EPL; ++i) s = fmaf(qr[i], kg[(size_t)j * ts + i], s);
        s = group_sum(s) * a.sm_scale;
        const float p = expf(s - m);
        l += p;
#pragma unroll
        for (int i = 0; i < EPL; ++i) o[i] = fmaf(p, vg[(size_t)j * ts + i], o[i]);
    }
#pragma unroll
    for (int i = 0; i < EPL; ++i) o[i] /= l;

    if (a.S != nullptr) {
        if (a.q_lin != nullptr) {     // the linear branch's own query (Eq. (3)) replaces q from here on
            const float *ql = (const float *)a.q_lin + (((size_t)b * Lq + rowc) * H + h) * D + sub * EPL;
#pragma unroll
            for (int i = 0; i < EPL; ++i) qr[i] = ql[i];
        }
        float ss = 0.f;
#pragma unroll
        for (int i = 0; i < EPL; ++i) ss = fmaf(qr[i], qr[i], ss);
        ss = group_sum(ss);
        const float nq = sqrtf(ss + a.l2_eps);
        const float *Sg = a.S + ((size_t)b * H + h) * D * D + sub * EPL;
        float oi[EPL];
#pragma unroll
        for (int i = 0; i < EPL; ++i) oi[i] = 0.f;
        const int gbase = (tid & (kWave - 1)) & ~(GROUP - 1);
#pragma unroll
        for (int src = 0; src < GROUP; ++src) {
#pragma unroll
            for (int i = 0; i < EPL; ++i) {
                const float qd = __shfl(qr[i], gbase + src, kWave) / nq;   // feature d = src*EPL + i
                const int d = src * EPL + i;
#pragma unroll
                for (int e = 0; e < EPL; ++e) oi[e] = fmaf(qd, Sg[(size_t)d * D + e], oi[e]);
            }
        }
        const size_t gi = a.g_per_token ? (size_t)b * Lq + rowc : ((size_t)b * Lq + rowc) * H + h;
#pragma unroll
        for (int i = 0; i < EPL; ++i) {
            float g = 1.0f;                  // headwise or per-token gate, or one gate per output feature
            if (a.g != nullptr) {
                const size_t ge = a.g_per_element ? gi * D + sub * EPL + i : gi;
                g = a.g_is_bf16 ? (float)((const bf16_t *)a.g)[ge] : ((const float *)a.g)[ge];
            }
            o[i] = fmaf(g, oi[i], o[i]);
        }
    }
    if (valid) {
        float *og = (float *)a.out + (((size_t)b * Lq + row) * H + h) * D + sub * EPL;
#pragma unroll
        for (int i = 0; i < EPL; ++i) og[i] = o[i];
    }
}

// workspace[b][i][h] = 1 / sqrt(|k_i|^2 + eps)
__global__ __launch_bounds__(NT) void knorm_f32_kernel(CommitArgs a)
{
    const size_t n = (size_t)a.B * a.L * a.H;
    const size_t idx = (size_t)blockIdx.x * NT + threadIdx.x;
    if (idx >= n) return;
    const float *kp = (const float *)a.k + idx * a.D;
    float ss = 0.f;
    for (int d = 0; d < a.D; ++d) ss = fmaf(kp[d], kp[d], ss);
    ((float *)a.workspace)[idx] = 1.0f / sqrtf(ss + a.l2_eps);
}

// grid (D, H, B), D threads: thread e owns S[d = blockIdx.x][e]; tokens added in ascending order
__global__ void commit_f32_kernel(CommitArgs a)
{
    const int d = blockIdx.x, h = blockIdx.y, b = blockIdx.z, e = threadIdx.x;
    const int D = a.D, H = a.H, L = a.L;
    const size_t ts = (size_t)H * D;
    const float *kg = (const float *)a.k + ((size_t)b * L * H + h) * D;
    const float *vg = (const float *)a.v + ((size_t)b * L * H + h) * D;
    const float *rn = (const float *)a.workspace + (size_t)b * L * H + h;
    float acc = 0.f;
    for (int i = 0; i < L; ++i) {
        const float kn = kg[(size_t)i * ts + d] * rn[(size_t)i * H];
        acc = fmaf(kn, vg[(size_t)i * ts + e], acc);
    }
    float *Sp = a.S + (((size_t)b * H + h) * D + d) * D + e;
    *Sp = fmaf(a.gate[(size_t)b * H + h], *Sp, acc);
}

}  // namespace

hipError_t launch_fwd_f32(const FwdArgs &a, hipStream_t stream)
{
    const dim3 grid((a.Lq + ROWS - 1) / ROWS, a.H, a.B), block(NT);
    if (a.H > 65535 || a.B > 65535) return hipErrorInvalidValue;
    if (a.D == 64) return launch_kernel(fwd_f32_kernel<64>, grid, block, stream, a);
    if (a.D == 128) return launch_kernel(fwd_f32_kernel<128>, grid, block, stream, a);
    return hipErrorInvalidValue;
}

hipError_t launch_commit_f32(const CommitArgs &a, hipStream_t stream)
{
    if (a.H > 65535 || a.B > 65535) return hipErrorInvalidValue;
    const size_t n = (size_t)a.B * a.L * a.H;
    const hipError_t e = launch_kernel(knorm_f32_kernel, dim3((unsigned)((n + NT - 1) / NT)), dim3(NT), stream, a);
    if (e != hipSuccess) return e;
    return launch_kernel(commit_f32_kernel, dim3(a.D, a.H, a.B), dim3(a.D), stream, a);
}

}  // namespace arl2
