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
// the second GEMM (k-slot j of half-wave hh is key 16t + 8(j/4) + 4hh + j%4); the matching
// V^T fragments come from the row-major V tile in LDS through the transposing LDS read
// (ds_read_b64_tr_b16), four keys per read.
//
// K/V tiles are double-buffered in LDS (one barrier per tile); the running maximum is only
// raised when a row's tile maximum exceeds it by more than 2^8, which removes the
// accumulator rescale from almost every tile without changing the normalised result.
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
    static constexpr int VROW = 2 * D + 64;      // LDS bytes per V row (padded: conflict-free transposing reads)
    static constexpr int K_BYTES = BN * KROW;
    static constexpr int V_BYTES = BN * VROW;
    static constexpr int STAGE = K_BYTES + V_BYTES;   // one K/V tile
    static constexpr int KV_BYTES = 2 * STAGE;        // double-buffered
    static constexpr int ST_BYTES = D * KROW;    // state staging [e][d]
    static constexpr int OUT_BYTES = BM * KROW;  // output staging [q][e]
    static constexpr int SMEM = (KV_BYTES > ST_BYTES ? (KV_BYTES > OUT_BYTES ? KV_BYTES : OUT_BYTES)
                                                     : (ST_BYTES > OUT_BYTES ? ST_BYTES : OUT_BYTES));
    static constexpr int KCH = BN * CPR / NT;    // K chunks per thread per tile
};

// Raise the running maximum only when the tile maximum exceeds it by more than this (log2 units).
constexpr float kRescaleThreshold = 8.0f;

typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;

// Transposing LDS read: within each group of 16 lanes, lane i receives element i of the four
// 16-element rows whose 8-byte pieces are addressed by lanes 4j..4j+3 (j = 0..3).
__device__ __forceinline__ bf16x4 lds_read_tr(const unsigned char *p)
{
    return __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4 *)(p));
}

template <int D>
__global__ __launch_bounds__(NT, 2) void fwd_bf16_kernel(FwdArgs a, int n_qtiles, float scale_log2)
{
    using C = FwdCfg<D>;
    __shared__ __attribute__((aligned(16))) unsigned char smem[C::SMEM];

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

    // ---- global -> LDS copies: 16-byte chunks, chunk id = tid + NT*i -> (row, col), for K and V alike
    u32x4 kreg[C::KCH];
    u32x4 vreg[C::KCH];

    // transposing-read role of this lane: row offset and byte offset inside a 32-column block
    const int tr_row = ((lane & 15) >> 2) + 4 * hh;
    const int tr_col = 32 * ((lane >> 4) & 1) + 8 * (lane & 3);

    auto load_tile = [&](int kv0) {
#pragma unroll
        for (int i = 0; i < C::KCH; ++i) {
            const int id = tid + NT * i;
            const int row = id / C::CPR, col = id % C::CPR;
            u32x4 x = {0, 0, 0, 0}, y = {0, 0, 0, 0};
            if (kv0 + row < Lkv) {
                x = *(const u32x4 *)(kg + (size_t)(kv0 + row) * tok_stride + 8 * col);
                y = *(const u32x4 *)(vg + (size_t)(kv0 + row) * tok_stride + 8 * col);
            }
            kreg[i] = x;
            vreg[i] = y;
        }
    };

    auto store_tile = [&](int stage) {
        unsigned char *smK = smem + stage * C::STAGE;
        unsigned char *smV = smK + C::K_BYTES;
#pragma unroll
        for (int i = 0; i < C::KCH; ++i) {
            const int id = tid + NT * i;
            const int row = id / C::CPR, col = id % C::CPR;
            *(u32x4 *)(smK + row * C::KROW + 16 * col) = kreg[i];
            *(u32x4 *)(smV + row * C::VROW + 16 * col) = vreg[i];
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
    store_tile(0);
    __syncthreads();

    for (int it = 0; it < ntiles; ++it) {
        const int kv0 = it * BN;
        const unsigned char *smK = smem + (it & 1) * C::STAGE;
        const unsigned char *smV = smK + C::K_BYTES;
        if (it + 1 < ntiles) load_tile(kv0 + BN);   // lands in registers while this tile is computed

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
        mx = xhalf_max(mx) * scale_log2;
        if (__any(mx > m_run + kRescaleThreshold)) {      // wave-uniform: rare after the first tiles
            const float m_new = fmaxf(m_run, mx);
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
            m_run = m_new;
            l_run *= alpha;
#pragma unroll
            for (int db = 0; db < C::DB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) o_acc[db][r] *= alpha;
        }
        float psum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float pv = __builtin_amdgcn_exp2f(fmaf(s[kb][r], scale_log2, -m_run));
                s[kb][r] = pv;
                psum += pv;
            }
        l_run += psum;

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
                const unsigned char *vp = smV + (16 * t + tr_row) * C::VROW + 64 * db + tr_col;
                const bf16x4 lo = lds_read_tr(vp);                    // keys 16t + 4hh + 0..3
                const bf16x4 hi = lds_read_tr(vp + 8 * C::VROW);      // keys 16t + 8 + 4hh + 0..3
                const bf16x8 va = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pf[t], o_acc[db], 0, 0, 0);
            }
        }
        if (it + 1 < ntiles) store_tile((it + 1) & 1);   // the other buffer was last read one tile ago
        __syncthreads();
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
