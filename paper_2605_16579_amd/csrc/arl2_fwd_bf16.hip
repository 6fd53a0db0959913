// Read-only denoising pass on bf16 MFMA (gfx950):
//   out = softmax(q k^T * sm_scale) v + g * L2Norm(q) S            paper Eq. (2), (3), (5), (6)
//
// One workgroup (4 wavefronts) owns 128 query rows of one (stream, head); each wavefront owns
// 32 of them.  Everything is computed transposed so that no operand ever has to be re-laid
// out between the two GEMMs:
//
//   S^T[kv][q]  = K[kv][:] . Q[q][:]      A = K tile rows from LDS,  B = Q fragments in registers
//   O^T[d][q]  += V^T[d][kv] . P^T[kv][q] A = V^T tile rows from LDS, B = exp'd S^T accumulators
//
// With v_mfma_f32_32x32x16_bf16 a lane holds one query column (lane % 32) of the S^T
// accumulator, so the softmax row statistics are in-lane reductions plus one exchange
// between the two half-waves.  The accumulator registers of S^T are exactly a B operand of
// the second GEMM for a permuted key order; V^T is written to LDS in that same permuted
// order (key index bits 2 and 3 swapped inside each group of 16 keys).
//
// Epilogue (fused linear readout): O_inter^T[e][q] = S^T[e][d] . Q^T[d][q] with the fp32
// state split into bf16 hi + lo parts staged through the (now free) K/V LDS, the raw bf16 q
// fragments as B operand, and the L2 norm of q applied as an fp32 per-column scale.
#include "arl2_device.h"

namespace arl2 {
namespace {

constexpr int BM = 128;   // query rows per workgroup
constexpr int BN = 64;    // keys per tile
constexpr int NT = 256;   // threads per workgroup

template <int D>
struct FwdCfg {
    static constexpr int KS = D / 16;            // k-steps of the QK^T contraction
    static constexpr int DB = D / 32;            // 32-row blocks of O^T
    static constexpr int CPR = D / 8;            // 16-byte chunks per row
    static constexpr int KROW = 2 * D + 16;      // LDS bytes per K row (padded: conflict-free b128 reads)
    static constexpr int VROW = 2 * BN + 8;      // LDS bytes per V^T row (padded: conflict-free b64 reads)
    static constexpr int K_BYTES = BN * KROW;
    static constexpr int V_BYTES = D * VROW;
    static constexpr int KV_BYTES = K_BYTES + V_BYTES;
    static constexpr int ST_BYTES = D * KROW;    // state staging [e][d]
    static constexpr int OUT_BYTES = BM * KROW;  // output staging [q][e]
    static constexpr int SMEM = (KV_BYTES > ST_BYTES ? (KV_BYTES > OUT_BYTES ? KV_BYTES : OUT_BYTES)
                                                     : (ST_BYTES > OUT_BYTES ? ST_BYTES : OUT_BYTES));
    static constexpr int KCH = BN * CPR / NT;    // K chunks per thread per tile
};

// Position of key (kv mod 64) inside a V^T row: swap bits 2 and 3.
__device__ __forceinline__ int vt_pos(int kvl)
{
    return (kvl & ~12) | ((kvl & 4) << 1) | ((kvl & 8) >> 1);
}

template <int D>
__global__ __launch_bounds__(NT, 2) void fwd_bf16_kernel(FwdArgs a, int n_qtiles, float scale_log2)
{
    using C = FwdCfg<D>;
    __shared__ __attribute__((aligned(16))) unsigned char smem[C::SMEM];
    unsigned char *smK = smem;
    unsigned char *smV = smem + C::K_BYTES;

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, c = lane & 31, hh = lane >> 5;

    const int work = xcd_contiguous_id(blockIdx.x, gridDim.x);
    const int qt = work % n_qtiles;
    const int bh = work / n_qtiles;
    const int h = bh % a.H, b = bh / a.H;
    const int H = a.H, Lq = a.Lq, Lkv = a.Lkv;

    const bf16_t *qg = (const bf16_t *)a.q;
    const bf16_t *kg = (const bf16_t *)a.k + ((size_t)b * Lkv * H + h) * D;
    const bf16_t *vg = (const bf16_t *)a.v + ((size_t)b * Lkv * H + h) * D;
    const size_t tok_stride = (size_t)H * D;

    // ---- Q fragments (B operand of S^T = K Q^T): lane (c, hh) holds Q[row c][16 t + 8 hh + 0..7]
    const int q0 = qt * BM;
    const int qrow = q0 + wave * 32 + c;
    bf16x8 qf[C::KS];
    float qss = 0.f;
    {
        const bf16_t *qp = qg + ((size_t)(b * (size_t)Lq + (qrow < Lq ? qrow : 0)) * H + h) * D + 8 * hh;
#pragma unroll
        for (int t = 0; t < C::KS; ++t) {
            bf16x8 x = {0, 0, 0, 0, 0, 0, 0, 0};
            if (qrow < Lq) x = *(const bf16x8 *)(qp + 16 * t);
            qf[t] = x;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float f = (float)x[j];
                qss = fmaf(f, f, qss);
            }
        }
        qss = xhalf_sum(qss);   // |q_row|^2 over the full head dimension
    }

    // ---- per-thread roles for the global -> LDS copies
    // K: 16-byte chunks, chunk id = tid + NT*i -> (row, col)
    // V: one 4-key x 8-dim block per thread, transposed in registers
    const int v_dg = tid % C::CPR, v_u = tid / C::CPR;
    const bool v_active = v_u < BN / 4;
    const int v_p0 = vt_pos(4 * v_u);

    u32x4 kreg[C::KCH];
    u32x4 vreg[4];

    auto load_tile = [&](int kv0) {
#pragma unroll
        for (int i = 0; i < C::KCH; ++i) {
            const int id = tid + NT * i;
            const int row = id / C::CPR, col = id % C::CPR;
            u32x4 x = {0, 0, 0, 0};
            if (kv0 + row < Lkv) x = *(const u32x4 *)(kg + (size_t)(kv0 + row) * tok_stride + 8 * col);
            kreg[i] = x;
        }
        if (v_active) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int kv = kv0 + 4 * v_u + e;
                u32x4 x = {0, 0, 0, 0};
                if (kv < Lkv) x = *(const u32x4 *)(vg + (size_t)kv * tok_stride + 8 * v_dg);
                vreg[e] = x;
            }
        }
    };

    auto store_tile = [&]() {
#pragma unroll
        for (int i = 0; i < C::KCH; ++i) {
            const int id = tid + NT * i;
            const int row = id / C::CPR, col = id % C::CPR;
            *(u32x4 *)(smK + row * C::KROW + 16 * col) = kreg[i];
        }
        if (v_active) {
#pragma unroll
            for (int m = 0; m < 8; ++m) {
                const int w = m >> 1;
                const uint32_t sel = (m & 1) ? 0x07060302u : 0x05040100u;
                u32x2 o;
                o[0] = __builtin_amdgcn_perm(vreg[1][w], vreg[0][w], sel);
                o[1] = __builtin_amdgcn_perm(vreg[3][w], vreg[2][w], sel);
                *(u32x2 *)(smV + (8 * v_dg + m) * C::VROW + 2 * v_p0) = o;
            }
        }
    };

    // ---- running softmax state and O^T accumulators
    f32x16 o_acc[C::DB];
#pragma unroll
    for (int db = 0; db < C::DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o_acc[db][r] = 0.f;
    float m_run = -INFINITY;   // running max of scaled logits (log2 domain)
    float l_run = 0.f;         // this lane's share of the running sum

    const int ntiles = (Lkv + BN - 1) / BN;
    load_tile(0);

    for (int it = 0; it < ntiles; ++it) {
        const int kv0 = it * BN;
        __syncthreads();            // all waves are done reading the previous tile
        store_tile();
        __syncthreads();
        if (it + 1 < ntiles) load_tile(kv0 + BN);

        // S^T = K Q^T for two 32-key blocks
        f32x16 s[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
#pragma unroll
            for (int t = 0; t < C::KS; ++t) {
                const bf16x8 ka = *(const bf16x8 *)(smK + (32 * kb + c) * C::KROW + 32 * t + 16 * hh);
                s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qf[t], s[kb], 0, 0, 0);
            }
        }
        // keys past the end of the sequence (last tile only)
        if (kv0 + BN > Lkv) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int kvl = 32 * kb + 8 * (r >> 2) + 4 * hh + (r & 3);
                    if (kv0 + kvl >= Lkv) s[kb][r] = -INFINITY;
                }
        }
        // online softmax for this lane's query column
        float mx = s[0][0];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kb][r]);
        mx = xhalf_max(mx);
        const float m_new = fmaxf(m_run, mx * scale_log2);
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        m_run = m_new;
        float psum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float pv = __builtin_amdgcn_exp2f(fmaf(s[kb][r], scale_log2, -m_new));
                s[kb][r] = pv;
                psum += pv;
            }
        l_run = fmaf(l_run, alpha, psum);
#pragma unroll
        for (int db = 0; db < C::DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) o_acc[db][r] *= alpha;

        // P^T fragments: accumulator registers 8*(t&1)..+7 of block t/2 are one B operand
        bf16x8 pf[4];
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int j = 0; j < 8; ++j) pf[t][j] = to_bf16(s[t >> 1][8 * (t & 1) + j]);

        // O^T += V^T P^T
#pragma unroll
        for (int db = 0; db < C::DB; ++db) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const unsigned char *vp = smV + (32 * db + c) * C::VROW + 32 * t + 16 * hh;
                union { u32x2 u[2]; bf16x8 v; } va;
                va.u[0] = *(const u32x2 *)(vp);
                va.u[1] = *(const u32x2 *)(vp + 8);
                o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va.v, pf[t], o_acc[db], 0, 0, 0);
            }
        }
    }

    // ---- epilogue ------------------------------------------------------------------------
    const float l_tot = xhalf_sum(l_run);
    const float inv_l = 1.0f / l_tot;
#pragma unroll
    for (int db = 0; db < C::DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o_acc[db][r] *= inv_l;

    if (a.S != nullptr) {
        // O_inter^T[e][q] = sum_d S[d][e] * q[q][d], state as bf16 hi + lo, fp32 accumulate
        const float *Sg = a.S + ((size_t)b * H + h) * D * D;
        f32x16 inter[C::DB];
#pragma unroll
        for (int db = 0; db < C::DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) inter[db][r] = 0.f;

        constexpr int NBLK = D * D / 32;              // 4(d) x 8(e) blocks of the state
        constexpr int BPT = (NBLK + NT - 1) / NT;
#pragma unroll 1
        for (int part = 0; part < 2; ++part) {        // 0: hi part, 1: lo part
            __syncthreads();                          // LDS free (main loop / previous part done)
#pragma unroll
            for (int i = 0; i < BPT; ++i) {
                const int id = tid + NT * i;
                if (id < NBLK) {
                    const int eg = id % C::CPR, du = id / C::CPR;
                    const float *sp = Sg + (size_t)(4 * du) * D + 8 * eg;
                    float x[4][8];
#pragma unroll
                    for (int dd = 0; dd < 4; ++dd) {
                        const f32x4 lo4 = *(const f32x4 *)(sp + dd * D);
                        const f32x4 hi4 = *(const f32x4 *)(sp + dd * D + 4);
#pragma unroll
                        for (int j = 0; j < 4; ++j) { x[dd][j] = lo4[j]; x[dd][4 + j] = hi4[j]; }
                    }
#pragma unroll
                    for (int m = 0; m < 8; ++m) {
                        bf16x4 w;
#pragma unroll
                        for (int dd = 0; dd < 4; ++dd) {
                            const bf16_t hi = to_bf16(x[dd][m]);
                            w[dd] = part == 0 ? hi : to_bf16(x[dd][m] - (float)hi);
                        }
                        *(bf16x4 *)(smem + (8 * eg + m) * C::KROW + 8 * du) = w;
                    }
                }
            }
            __syncthreads();
#pragma unroll
            for (int db = 0; db < C::DB; ++db)
#pragma unroll
                for (int t = 0; t < C::KS; ++t) {
                    const bf16x8 sa = *(const bf16x8 *)(smem + (32 * db + c) * C::KROW + 32 * t + 16 * hh);
                    inter[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(sa, qf[t], inter[db], 0, 0, 0);
                }
        }
        // gate * L2 norm scale for this lane's query row
        float gq = 1.0f / sqrtf(qss + a.l2_eps);
        if (a.g != nullptr && qrow < Lq) {
            const size_t gi = ((size_t)b * Lq + qrow) * H + h;
            gq *= a.g_is_bf16 ? (float)((const bf16_t *)a.g)[gi] : ((const float *)a.g)[gi];
        }
#pragma unroll
        for (int db = 0; db < C::DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) o_acc[db][r] = fmaf(gq, inter[db][r], o_acc[db][r]);
    }

    // transpose through LDS so that every output row is written as contiguous 16-byte pieces
    __syncthreads();
    unsigned char *region = smem + wave * 32 * C::KROW;
#pragma unroll
    for (int db = 0; db < C::DB; ++db)
#pragma unroll
        for (int j4 = 0; j4 < 4; ++j4) {
            bf16x4 w;
#pragma unroll
            for (int i = 0; i < 4; ++i) w[i] = to_bf16(o_acc[db][4 * j4 + i]);
            const int e = 32 * db + 8 * j4 + 4 * hh;
            *(bf16x4 *)(region + c * C::KROW + 2 * e) = w;
        }
    __syncthreads();
    bf16_t *og = (bf16_t *)a.out;
#pragma unroll
    for (int i = 0; i < 32 * C::CPR / 64; ++i) {
        const int idx = lane + 64 * i;
        const int row = idx / C::CPR, col = idx % C::CPR;
        const int orow = q0 + wave * 32 + row;
        if (orow < Lq) {
            const u32x4 x = *(const u32x4 *)(region + row * C::KROW + 16 * col);
            *(u32x4 *)(og + ((size_t)(b * (size_t)Lq + orow) * H + h) * D + 8 * col) = x;
        }
    }
}

}  // namespace

hipError_t launch_fwd_bf16(const FwdArgs &a, hipStream_t stream)
{
    const int n_qtiles = (a.Lq + BM - 1) / BM;
    const long long nwg = (long long)n_qtiles * a.B * a.H;
    if (nwg <= 0 || nwg > 0x7fffffffLL) return hipErrorInvalidValue;
    const float scale_log2 = a.sm_scale * 1.4426950408889634f;
    const dim3 grid((unsigned)nwg), block(NT);
    if (a.D == 128)
        hipLaunchKernelGGL(fwd_bf16_kernel<128>, grid, block, 0, stream, a, n_qtiles, scale_log2);
    else if (a.D == 64)
        hipLaunchKernelGGL(fwd_bf16_kernel<64>, grid, block, 0, stream, a, n_qtiles, scale_log2);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace arl2
