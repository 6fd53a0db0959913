// Read-only denoising pass on bf16 MFMA (gfx950):
//   out = softmax(q k^T * sm_scale) v + g * L2Norm(q) S            paper Eq. (2), (3), (5), (6)
//
// One workgroup (8 wavefronts, two per SIMD, 256 registers each) owns 256 query rows of one
// (stream, head); each wavefront owns 32 of them.  Everything is computed transposed so that
// no operand is re-laid out between the two GEMMs:
//
//   S^T[kv][q]  = K[kv][:] . Q[q][:]      A = K tile rows from LDS,  B = Q fragments in registers
//   O^T[d][q]  += V^T[d][kv] . P^T[kv][q] A = V^T fragments from LDS, B = exp'd S^T accumulators
//
// With v_mfma_f32_32x32x16_bf16 a lane holds one query column (lane % 32) of the S^T
// accumulator, so the softmax row statistics are in-lane reductions plus one exchange
// between the two half-waves.  The accumulator registers of S^T are exactly a B operand of
// the second GEMM (k-slot j of half-wave hh is key 16t + 8(j/4) + 4hh + j%4); the matching
// V^T fragments come from the row-major V tile in LDS through the transposing LDS read
// (ds_read_b64_tr_b16), four keys per read.
//
// Per key tile every wavefront runs S = K Q^T (16 MFMAs), the online softmax of its 32 logits
// per lane (VALU), then O += V^T P^T (16 MFMAs).  On this hardware a wavefront does not overlap
// its own VALU work with its own MFMAs; the overlap comes from the second wavefront on the
// same SIMD, which the MFMA arbitration keeps about one phase behind the first.  Inside an MFMA
// chain every step issues one MFMA and the LDS read of the operand fragment needed seven MFMAs
// later, across chain boundaries, so the matrix pipe never waits for LDS latency.
//
// K/V tiles travel HBM/L2 -> registers (buffer loads, zero beyond the last key) -> a 3-stage
// LDS ring with one workgroup barrier per tile.  The softmax is optimistic: probabilities are
// taken relative to the running maximum as it stands, and only when a lane's share of the row
// sum shows that a logit exceeded it by more than ~2^7 (or on the first tile) is the true tile
// maximum computed, the running maximum raised, the accumulators rescaled and the tile redone.
// This removes the per-tile maximum reduction and the accumulator rescale from the steady
// state without changing the normalised result.  (Row sums use plain fp32 adds: the bf16
// dot-product instruction measured far slower next to MFMAs.)
//
// Epilogue (fused linear readout): O_inter^T[e][q] = S^T[e][d] . Q^T[d][q] with the fp32
// state split into bf16 hi + lo parts, staged row-major through the (now free) LDS and read
// transposed like V, the raw bf16 q fragments as B operand, and the L2 norm of q applied as an
// fp32 per-column scale.  The linear branch may read a query of its own (Eq. (3): RoPE(phi_q(Q))):
// either given as an array, or computed here from the pre-map rows and the head's D x D matrix, in
// which case the rotated, rounded accumulators of that small GEMM are used as the B fragments
// directly.  The gate is one value per (token, head) (Eq. (6)), per token, or per output feature.
#include "arl2_device.h"

#include <type_traits>

namespace arl2 {
namespace {

constexpr int BM = 256;   // query rows per workgroup
constexpr int BN = 64;    // keys per tile
constexpr int NT = 512;   // threads per workgroup
constexpr int NSTAGE = 4; // LDS ring depth (a power of two)
constexpr int kStoreStep0 = 4;   // the tile copy's LDS writes go into steps 4, 6, ... of an interval's second slot

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
    static constexpr int KV_BYTES = NSTAGE * STAGE;
    static constexpr int SS_BYTES = D * VROW;    // one bf16 part of the state staged [d][e]
    static constexpr int ST_BYTES = 2 * SS_BYTES;
    static constexpr int SCH = (D * CPR + NT - 1) / NT;   // 8-float state pieces per thread
    static constexpr int OUT_BYTES = BM * KROW;  // output staging [q][e]
    // fused feature map: half of Wq[h] (D/2 rows) plus, per wavefront, the rotation tables of its 32 tokens
    static constexpr int WH_BYTES = (D / 2) * KROW;
    static constexpr int TST = D / 2 + 2;        // floats per staged table row (conflict-free 8-byte reads)
    static constexpr int TAB_BYTES = 2 * 32 * TST * 4;
    static constexpr int FM_BYTES = WH_BYTES + (NT / 64) * TAB_BYTES;
    static constexpr int WCH = ((D / 2) * CPR + NT - 1) / NT;     // 16-byte chunks of the Wq half per thread
    static constexpr int TCH = 32 * (D / 8) / 64;                 // 16-byte chunks of one table tile per lane
    static constexpr int SMEM0 = (KV_BYTES > ST_BYTES ? (KV_BYTES > OUT_BYTES ? KV_BYTES : OUT_BYTES)
                                                      : (ST_BYTES > OUT_BYTES ? ST_BYTES : OUT_BYTES));
    static constexpr int SMEM = SMEM0 > FM_BYTES ? SMEM0 : FM_BYTES;
    static constexpr int KCH = BN * CPR / NT;    // 16-byte chunks per thread per tile (K and V each)
    static constexpr int ROWS_PER_PASS = NT / CPR;
    static constexpr int S_LEN = KS;             // MFMAs of the S^T chain of one 32-key block
    static constexpr int PV_LEN = 2 * DB;        // MFMAs of the PV chain of one 32-key block
    static constexpr int RING = 4;               // fragment registers in flight from LDS
    static constexpr int PF = RING - 1;          // operand fragments are read from LDS this many MFMAs ahead
    // LDS reads a full slot issues after step `first` (its own fragments, then the next slot's; S fragments,
    // at even positions, are one read, V^T fragments two)
    static constexpr int lds_reads_from(int first)
    {
        int c = 0;
        for (int n = first; n < S_LEN + PV_LEN; ++n) c += ((n + PF) & 1) == 0 ? 1 : 2;
        return c;
    }
    static constexpr int LDS_AFTER_COPY = lds_reads_from(kStoreStep0 + 4 * KCH - 1);
    static_assert(kStoreStep0 + 4 * KCH - 2 < S_LEN + PV_LEN && 2 * KCH - 1 < S_LEN + PV_LEN, "the copy must fit into one slot");
    static_assert(KCH >= 1, "tile too small for the workgroup");
    static_assert(S_LEN % RING == 0 && PV_LEN % RING == 0, "chain lengths must be multiples of the fragment ring");
};

// The running maximum is raised only when a lane's share of a tile's row sum (32 probabilities taken
// relative to the running maximum) reaches this value, i.e. some logit exceeded it by more than ~2^7.
constexpr float kRowSumLimit = 4096.0f;


template <int D>
__global__ __launch_bounds__(NT, 2) void fwd_bf16_kernel(FwdArgs a, int n_qtiles, float scale_log2, int ragged_last)
{
    using C = FwdCfg<D>;
    __shared__ __attribute__((aligned(16))) unsigned char smem[C::SMEM];

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, c = lane & 31, hh = lane >> 5;

    int qt, bh;
    if (ragged_last) {
        // Several rounds of workgroups, and the last query tile of every head is ragged (its workgroup has
        // idle wavefronts and finishes early): every XCD takes B H / 8 heads, their full tiles first, head
        // by head, and their ragged tiles at the end of its dispatch order, where a short job shortens the
        // last, partly filled round (workgroup ids go round the 8 XCDs in dispatch order).
        const int x = blockIdx.x % kNumXcd, loc = blockIdx.x / kNumXcd;
        const int heads_x = a.B * a.H / kNumXcd, n_full = n_qtiles - 1;
        if (loc < heads_x * n_full) {
            bh = x * heads_x + loc / n_full;
            qt = loc % n_full;
        } else {
            bh = x * heads_x + (loc - heads_x * n_full);
            qt = n_full;
        }
    } else {
        const int work = xcd_contiguous_id(blockIdx.x, gridDim.x);
        qt = work % n_qtiles;
        bh = work / n_qtiles;
    }
    const int h = bh % a.H, b = bh / a.H;
    const int H = a.H, Lq = a.Lq, Lkv = a.Lkv;

    const bf16_t *qg = (const bf16_t *)a.q;
    const bf16_t *kg = (const bf16_t *)a.k + ((size_t)b * Lkv * H + h) * D;
    const bf16_t *vg = (const bf16_t *)a.v + ((size_t)b * Lkv * H + h) * D;
    const uint32_t tok_bytes = (uint32_t)H * D * 2;                       // one token, all heads
    const uint32_t kv_range = (uint32_t)(Lkv - 1) * tok_bytes + 2 * D;    // bytes of this head's K (or V) slice
    const __amdgpu_buffer_rsrc_t k_rsrc = make_rsrc(kg, kv_range);
    const __amdgpu_buffer_rsrc_t v_rsrc = make_rsrc(vg, kv_range);

    // ---- Q fragments (B operand of S^T = K Q^T): lane (c, hh) holds Q[row][16 t + 8 hh + 0..7]
    const int q0 = qt * BM + wave * 32;
    const int qrow = q0 + c;
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

    // ---- global -> registers -> LDS copies: 16-byte chunks, chunk id = tid + NT*i -> (row, col)
    u32x4 kst[C::KCH], vst[C::KCH];
    uint32_t g_off = (uint32_t)(tid / C::CPR) * tok_bytes + 16 * (tid % C::CPR);   // chunk 0 of tile 0
    const int lds_k_off = (tid / C::CPR) * C::KROW + 16 * (tid % C::CPR);
    const int lds_v_off = (tid / C::CPR) * C::VROW + 16 * (tid % C::CPR);

    auto load_tile = [&]() {       // loads the tile at g_off and advances g_off by one tile
#pragma unroll
        for (int i = 0; i < C::KCH; ++i) {
            const uint32_t off = g_off + (uint32_t)i * C::ROWS_PER_PASS * tok_bytes;
            kst[i] = __builtin_amdgcn_raw_buffer_load_b128(k_rsrc, off, 0, 0);
            vst[i] = __builtin_amdgcn_raw_buffer_load_b128(v_rsrc, off, 0, 0);
        }
        g_off += BN * tok_bytes;
    };
    // the same copy in pieces: part h of the loads (chunk h of K and of V), piece p of the stores
    auto load_tile_part = [&](auto h_) {
        constexpr int h = decltype(h_)::value;
        const uint32_t off = g_off + (uint32_t)h * C::ROWS_PER_PASS * tok_bytes;
        kst[h] = __builtin_amdgcn_raw_buffer_load_b128(k_rsrc, off, 0, 0);
        vst[h] = __builtin_amdgcn_raw_buffer_load_b128(v_rsrc, off, 0, 0);
        if constexpr (h == C::KCH - 1) g_off += BN * tok_bytes;
    };
    auto store_tile_part = [&](int stage, auto p_) {
        constexpr int p = decltype(p_)::value;
        unsigned char *smK = smem + stage * C::STAGE;
        if constexpr ((p & 1) == 0) *(u32x4 *)(smK + lds_k_off + (p >> 1) * C::ROWS_PER_PASS * C::KROW) = kst[p >> 1];
        else *(u32x4 *)(smK + C::K_BYTES + lds_v_off + (p >> 1) * C::ROWS_PER_PASS * C::VROW) = vst[p >> 1];
    };
    auto store_tile = [&](int stage) {
        unsigned char *smK = smem + stage * C::STAGE;
        unsigned char *smV = smK + C::K_BYTES;
#pragma unroll
        for (int i = 0; i < C::KCH; ++i) {
            *(u32x4 *)(smK + lds_k_off + i * C::ROWS_PER_PASS * C::KROW) = kst[i];
            *(u32x4 *)(smV + lds_v_off + i * C::ROWS_PER_PASS * C::VROW) = vst[i];
        }
    };

    // lane roles inside a 32-key block
    const int k_frag_off = c * C::KROW + 16 * hh;                                   // + 32*t
    const int v_frag_off = (((lane & 15) >> 2) + 4 * hh) * C::VROW + 32 * ((lane >> 4) & 1) + 8 * (lane & 3);

    // ---- running softmax state and accumulators
    f32x16 o_acc[C::DB];         // O^T blocks
    f32x16 s_acc[2];             // S^T of the key block whose softmax runs, and of the next one
    bf16x8 pf[4];                // P^T fragments (B operands of the second GEMM): two per key block
    bf16x8 fr[C::RING];          // A-operand fragments in flight from LDS
    float m_run = -INFINITY;     // running max of scaled logits (log2 domain)
    float l_run = 0.f;           // this lane's share of the running sum
#pragma unroll
    for (int db = 0; db < C::DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o_acc[db][r] = 0.f;

    // Byte offsets in the ring of the K rows / V rows of 32-key block `blk` (tile blk / 2, half blk % 2).
    auto k_block = [&](int blk) -> int { return ((blk >> 1) & (NSTAGE - 1)) * C::STAGE + (blk & 1) * 32 * C::KROW; };
    auto v_block = [&](int blk) -> int { return ((blk >> 1) & (NSTAGE - 1)) * C::STAGE + C::K_BYTES + (blk & 1) * 32 * C::VROW; };
    // A-operand fragments: k-step n of S^T = K Q^T (a K row piece), and MFMA n of O^T += V^T P^T
    // (16-key step n / DB, row block n % DB: a transposed V piece).
    auto k_frag = [&](const unsigned char *kp, auto n_) -> bf16x8 {
        return *(const bf16x8 *)(kp + 32 * decltype(n_)::value);
    };
    auto v_frag = [&](const unsigned char *vp, auto n_) -> bf16x8 {
        constexpr int n = decltype(n_)::value;
        const unsigned char *p = vp + 16 * (n / C::DB) * C::VROW + 64 * (n % C::DB);
        const bf16x4 lo = lds_read_tr(p);                    // keys 16u + 4hh + 0..3
        const bf16x4 hi = lds_read_tr(p + 8 * C::VROW);      // keys 16u + 8 + 4hh + 0..3
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    };
    // exp2 of the 16 logits per lane of one key block relative to the running maximum -> its two P^T
    // fragments; returns this lane's share of the row sum.  (Only on the rare path that raises the maximum.)
    auto exp_block = [&](auto par_) -> float {
        constexpr int PAR = decltype(par_)::value;
        const float mneg = -m_run;
        float psum = 0.f;
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
            const float p0 = __builtin_amdgcn_exp2f(fmaf(s_acc[PAR][r], scale_log2, mneg));
            const float p1 = __builtin_amdgcn_exp2f(fmaf(s_acc[PAR][r + 1], scale_log2, mneg));
            psum += p0 + p1;
            pf[2 * PAR + (r >> 3)][r & 7] = to_bf16(p0);
            pf[2 * PAR + (r >> 3)][(r & 7) + 1] = to_bf16(p1);
        }
        return psum;
    };

    // One slot of the software pipeline, on key block j (logits in s_acc[j % 2], produced one slot earlier):
    //   matrix pipe:  S(j+1) = K_{j+1} Q^T  -> s_acc[(j+1) % 2]     (KS MFMAs, if the block exists)
    //                 O^T += V_{j-1}^T P_{j-1}^T                      (2 DB MFMAs, if j > 0)
    //   vector ALU:   softmax of block j -> its P^T fragments and row-sum share
    // Neither MFMA chain depends on this slot's vector work, so every step issues one MFMA, the LDS read of
    // the operand fragment needed PF MFMAs later (at the end of the slot: of the next slot's first chain)
    // and a slice of the softmax; the slices are themselves staggered (scale of logit v+2, exponential of
    // logit v+1, sum and conversion of logit v) so that no instruction waits for the one before it.
    // copy_: 0 nothing; 1 this slot also requests the next K/V tile from global memory (early steps);
    // 2 it also writes that tile, by now in registers, into ring stage `cstage`, one 16-byte piece per thread
    // every other step, so that the copy runs under the MFMAs instead of in a burst before the barrier.
    auto slot = [&](auto par_, auto has_s_, auto has_pv_, auto next_s_, auto masked_, int j, auto copy_, int cstage) {
        constexpr int PAR = decltype(par_)::value;
        constexpr int COPY = decltype(copy_)::value;
        constexpr bool HAS_S = decltype(has_s_)::value, HAS_PV = decltype(has_pv_)::value;
        constexpr bool NEXT_S = decltype(next_s_)::value, MASKED = decltype(masked_)::value;
        constexpr int SL = HAS_S ? C::S_LEN : 0, NS = SL + (HAS_PV ? C::PV_LEN : 0);
        constexpr int LPS = 16 / NS;                 // logits per step
        static_assert(NS % C::RING == 0 && 16 % NS == 0, "slot length");
        const unsigned char *kp = smem + k_block(j + 1) + k_frag_off;
        const unsigned char *vp = smem + v_block(j - 1) + v_frag_off;
        const unsigned char *np = smem + k_block(j + 2) + k_frag_off;      // next slot: S(j+2) (if any) and PV(j)
        const unsigned char *nvp = smem + v_block(j) + v_frag_off;
        const float mneg = -m_run;
        float x[16], ps0 = 0.f, ps1 = 0.f;
        auto op_scale = [&](auto v_) {               // logit v: scaled, relative to the running maximum
            constexpr int v = decltype(v_)::value;
            if constexpr (v < 16) {
                if constexpr (MASKED) {              // keys past the end of the sequence (last tile only)
                    const int kvl = 8 * (v >> 2) + 4 * hh + (v & 3);
                    if (32 * j + kvl >= Lkv) s_acc[PAR][v] = -INFINITY;
                }
                x[v] = fmaf(s_acc[PAR][v], scale_log2, mneg);
            }
        };
        auto op_exp = [&](auto v_) {
            constexpr int v = decltype(v_)::value;
            if constexpr (v < 16) x[v] = __builtin_amdgcn_exp2f(x[v]);
        };
        auto op_sum = [&](auto v_) {                 // row-sum share, and the P^T pair (v-1, v) for odd v
            constexpr int v = decltype(v_)::value;
            if constexpr (v & 1) {
                ps1 += x[v];
                bf16x2 pk = {to_bf16(x[v - 1]), to_bf16(x[v])};
                asm volatile("" : "+v"(pk));         // the conversion stays in this step
                pf[2 * PAR + (v >> 3)][(v & 7) - 1] = pk[0];
                pf[2 * PAR + (v >> 3)][v & 7] = pk[1];
            } else {
                ps0 += x[v];
            }
        };
        // MFMA n of the slot: with both chains present they alternate (S at even n), so that MFMAs which
        // accumulate into the same registers are never issued back to back
        auto is_s = [](int n) constexpr { return HAS_S && (!HAS_PV || (n & 1) == 0); };
        auto idx = [](int n) constexpr { return HAS_S && HAS_PV ? n >> 1 : n; };
        auto fetch = [&](auto m_) {                  // requests the A fragment of MFMA m (m >= NS: of the next slot)
            constexpr int m = decltype(m_)::value;
            if constexpr (m < NS) {
                if constexpr (is_s(m)) fr[m % C::RING] = k_frag(kp, std::integral_constant<int, idx(m)>{});
                else fr[m % C::RING] = v_frag(vp, std::integral_constant<int, idx(m)>{});
            } else {
                // the next slot has a second GEMM (this slot's block) in every case; its S chain alternates with it
                constexpr int mm = m - NS;
                if constexpr (NEXT_S && (mm & 1) == 0) fr[m % C::RING] = k_frag(np, std::integral_constant<int, (mm >> 1)>{});
                else fr[m % C::RING] = v_frag(nvp, std::integral_constant<int, (NEXT_S ? mm >> 1 : mm)>{});
            }
        };
        static_for<0, NS>([&](auto n_) {
            constexpr int n = decltype(n_)::value;
            fetch(std::integral_constant<int, n + C::PF>{});
            if constexpr (is_s(n)) {
                constexpr int t = idx(n);
                if constexpr (t == 0) {
                    const f32x16 zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
                    s_acc[PAR ^ 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[n % C::RING], qf[t], zero, 0, 0, 0);
                } else {
                    s_acc[PAR ^ 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[n % C::RING], qf[t], s_acc[PAR ^ 1], 0, 0, 0);
                }
            } else {
                constexpr int u = idx(n) / C::DB, db = idx(n) % C::DB;
                o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[n % C::RING], pf[2 * (PAR ^ 1) + u], o_acc[db], 0, 0, 0);
            }
            if constexpr (COPY == 1 && (n & 1) == 1 && n / 2 < C::KCH) load_tile_part(std::integral_constant<int, n / 2>{});
            if constexpr (COPY == 2 && n >= kStoreStep0 && n < kStoreStep0 + 4 * C::KCH && ((n - kStoreStep0) & 1) == 0)
                store_tile_part(cstage, std::integral_constant<int, (n - kStoreStep0) / 2>{});
            if constexpr (n == 0) {
                op_scale(std::integral_constant<int, 0>{});
                op_scale(std::integral_constant<int, 1>{});
                op_exp(std::integral_constant<int, 0>{});
            }
            static_for<0, LPS>([&](auto i_) {
                constexpr int v = n * LPS + decltype(i_)::value;
                op_scale(std::integral_constant<int, v + 2>{});
                op_exp(std::integral_constant<int, v + 1>{});
                op_sum(std::integral_constant<int, v>{});
            });
            __builtin_amdgcn_sched_barrier(0);
        });
        float psum = ps0 + ps1;
        // Rarely (always on the first block) a logit exceeded the running maximum by more than the
        // threshold: take the true block maximum, raise the running maximum, rescale, redo the block.
        if (__any(!(psum < kRowSumLimit))) {      // wave-uniform; also true for inf and NaN
            float mx = s_acc[PAR][0];
#pragma unroll
            for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s_acc[PAR][r]);
            mx = xhalf_max(mx) * scale_log2;
            const float m_new = fmaxf(m_run, mx);
            const float alpha = m_new == m_run ? 1.0f : __builtin_amdgcn_exp2f(m_run - m_new);
            m_run = m_new;
            l_run *= alpha;
#pragma unroll
            for (int db = 0; db < C::DB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) o_acc[db][r] *= alpha;
            psum = exp_block(par_);
        }
        l_run += psum;
    };

    const int ntiles = (Lkv + BN - 1) / BN;
    const std::false_type no{};
    const std::true_type yes{};
    const std::integral_constant<int, 0> par0{};
    const std::integral_constant<int, 1> par1{};
    const std::integral_constant<int, 0> copy0{};
    const std::integral_constant<int, 1> copy1{};
    const std::integral_constant<int, 2> copy2{};

    // ---- prologue: tiles 0 and 1 into the ring
    load_tile();
    store_tile(0);
    load_tile();
    store_tile(1);
    __syncthreads();

    // Barrier interval i covers the slots of key blocks 2i and 2i+1: they read K of tiles i and i+1 and V of
    // tiles i-1 and i.  Tile i+2 is fetched into registers at its start and written at its end to the ring
    // stage of tile i-2 (four stages); the barrier that closes the interval publishes it.
    auto close_interval = [&](int i) {
        store_tile((i + 2) & (NSTAGE - 1));
        __syncthreads();
    };

    if (q0 < Lq) {
        // S(0), plain: nothing to overlap it with
        {
            const unsigned char *kp = smem + k_block(0) + k_frag_off;
            const unsigned char *np = smem + k_block(1) + k_frag_off;
            static_for<0, C::PF>([&](auto m_) { fr[decltype(m_)::value] = k_frag(kp, m_); });
            static_for<0, C::S_LEN>([&](auto n_) {
                constexpr int n = decltype(n_)::value;
                constexpr int m = n + C::PF;
                if constexpr (m < C::S_LEN) fr[m % C::RING] = k_frag(kp, std::integral_constant<int, m>{});
                else fr[m % C::RING] = k_frag(np, std::integral_constant<int, m - C::S_LEN>{});
                if constexpr (n == 0) {
                    const f32x16 zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
                    s_acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[n % C::RING], qf[n], zero, 0, 0, 0);
                } else {
                    s_acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[n % C::RING], qf[n], s_acc[0], 0, 0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
            });
        }
        load_tile();
        if (ntiles == 1) {
            slot(par0, yes, no, no, yes, 0, copy0, 0);
            slot(par1, no, yes, no, yes, 1, copy0, 0);
        } else {
            slot(par0, yes, no, yes, no, 0, copy0, 0);
            slot(par1, yes, yes, yes, no, 1, copy0, 0);
        }
        close_interval(0);
#pragma unroll 1
        for (int i = 1; i < ntiles - 1; ++i) {
            slot(par0, yes, yes, yes, no, 2 * i, copy1, 0);
            slot(par1, yes, yes, yes, no, 2 * i + 1, copy2, (i + 2) & (NSTAGE - 1));
            // the writes are complete once at most the LDS reads issued after the last of them are still
            // outstanding (LDS operations complete in order); those reads stay in flight across the barrier
            lds_barrier_keep<C::LDS_AFTER_COPY>();
        }
        if (ntiles > 1) {
            const int i = ntiles - 1;
            slot(par0, yes, yes, no, yes, 2 * i, copy0, 0);
            slot(par1, no, yes, no, yes, 2 * i + 1, copy0, 0);
        }
        // second GEMM of the last key block (its first fragments are in flight)
        {
            const unsigned char *vp = smem + v_block(2 * ntiles - 1) + v_frag_off;
            static_for<0, C::PV_LEN>([&](auto n_) {
                constexpr int n = decltype(n_)::value;
                constexpr int m = n + C::PF;
                if constexpr (m < C::PV_LEN) fr[m % C::RING] = v_frag(vp, std::integral_constant<int, m>{});
                o_acc[n % C::DB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[n % C::RING], pf[2 + n / C::DB], o_acc[n % C::DB], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            });
        }
    } else {
        // A wavefront whose 32 rows all lie past the last query (the ragged last workgroup of a head) only
        // helps to move the tiles: the same loads, stores and barriers, no arithmetic.  Its rows are never
        // stored.
        load_tile();
        close_interval(0);
#pragma unroll 1
        for (int i = 1; i < ntiles - 1; ++i) {
            load_tile();
            close_interval(i);
        }
        l_run = 1.0f;
    }

    // ---- epilogue ------------------------------------------------------------------------
    {
        const float inv_l = 1.0f / xhalf_sum(l_run);
#pragma unroll
        for (int db = 0; db < C::DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) o_acc[db][r] *= inv_l;
    }

    if (a.S != nullptr) {
        // O_inter^T[e][q] = sum_d S[d][e] * q[q][d]: the fp32 state is split into bf16 hi + lo parts
        // (fp32 accumulate), both staged row-major [d][e] in LDS and read as S^T fragments through the
        // transposing LDS read, exactly like V.
        const float *Sg = a.S + ((size_t)b * H + h) * D * D;
        if (a.q_lin != nullptr) {
            // the linear branch has a query of its own (Eq. (3): its feature map differs from the
            // softmax branch's): take its fragments and its squared norm instead
            const bf16_t *qp = (const bf16_t *)a.q_lin + ((size_t)(b * (size_t)Lq + (qrow < Lq ? qrow : 0)) * H + h) * D + 8 * hh;
            qss = 0.f;
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
            qss = xhalf_sum(qss);
        }
        // Fused feature map of the linear branch (Eq. (3)): q_lin^T[e][row] = sum_d Wq[e][d] xq[row][d], rotated
        // pair by pair, is never stored: the accumulator registers, rounded to bf16, are the B fragments of
        // the readout (k-slot j of half-wave hh is feature 16t + 8(j/4) + 4hh + j%4, as for P^T above).
        // Wq[h] passes through LDS in two halves of D/2 output rows (whole rows in, fragments out) and every
        // wavefront stages the rotation table rows of its 32 tokens in a region of its own: read straight
        // from global memory, fragment by fragment, these operands cost ~13 us of cache-line requests.
        const bool fused_map = a.xq != nullptr;
        if (fused_map) {
            const size_t row_off = ((size_t)(b * (size_t)Lq + (qrow < Lq ? qrow : 0)) * H + h) * D;
            bf16x8 xf[C::KS];
#pragma unroll
            for (int t = 0; t < C::KS; ++t) {
                bf16x8 x = {0, 0, 0, 0, 0, 0, 0, 0};
                if (qrow < Lq) x = *(const bf16x8 *)((const bf16_t *)a.xq + row_off + 16 * t + 8 * hh);
                xf[t] = x;
            }
            unsigned char *smW = smem;                                           // D/2 rows of Wq[h], KROW bytes each
            float *cosT = (float *)(smem + C::WH_BYTES + wave * C::TAB_BYTES);   // this wavefront's [32][TST] tables
            float *sinT = cosT + 32 * C::TST;
            const bool rope = a.cs != nullptr;
            qss = 0.f;
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                __syncthreads();                      // the K/V ring (or the previous half of Wq) is no longer read
#pragma unroll
                for (int i = 0; i < C::WCH; ++i) {    // chunk id: row id / CPR of this half, 16-byte column id % CPR
                    const int id = tid + NT * i;
                    const int wr = id / C::CPR, wc = id % C::CPR;
                    if (wr < D / 2)
                        *(u32x4 *)(smW + wr * C::KROW + 16 * wc) =
                            *(const u32x4 *)((const bf16_t *)a.Wq + ((size_t)h * D + half * (D / 2) + wr) * D + 8 * wc);
                }
                if (half == 0 && rope) {
#pragma unroll
                    for (int i = 0; i < C::TCH; ++i) {
                        const int id = lane + 64 * i;
                        const int tk = id / (D / 8), col = id % (D / 8);
                        const int trow = q0 + tk < Lq ? q0 + tk : Lq - 1;
                        const u32x4 cv = *(const u32x4 *)(a.cs + (size_t)trow * (D / 2) + 4 * col);
                        const u32x4 sv = *(const u32x4 *)(a.sn + (size_t)trow * (D / 2) + 4 * col);
                        u32x2 *cd = (u32x2 *)(cosT + tk * C::TST + 4 * col), *sd = (u32x2 *)(sinT + tk * C::TST + 4 * col);
                        cd[0] = u32x2{cv[0], cv[1]};
                        cd[1] = u32x2{cv[2], cv[3]};
                        sd[0] = u32x2{sv[0], sv[1]};
                        sd[1] = u32x2{sv[2], sv[3]};
                    }
                }
                __syncthreads();
#pragma unroll
                for (int e2 = 0; e2 < C::DB / 2; ++e2) {
                    const int eb = half * (C::DB / 2) + e2;
                    f32x16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
                    for (int t = 0; t < C::KS; ++t) {
                        const bf16x8 wf = *(const bf16x8 *)(smW + (32 * e2 + c) * C::KROW + 32 * t + 16 * hh);
                        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, xf[t], acc, 0, 0, 0);
                    }
                    if (rope) {
#pragma unroll
                        for (int j4 = 0; j4 < 4; ++j4) {      // registers 4 j4 .. +3: features 32 eb + 8 j4 + 4 hh + 0..3
                            const f32x2 c2 = *(const f32x2 *)(cosT + c * C::TST + 16 * eb + 4 * j4 + 2 * hh);
                            const f32x2 s2 = *(const f32x2 *)(sinT + c * C::TST + 16 * eb + 4 * j4 + 2 * hh);
#pragma unroll
                            for (int p = 0; p < 2; ++p) {
                                const float y0 = acc[4 * j4 + 2 * p], y1 = acc[4 * j4 + 2 * p + 1];
                                acc[4 * j4 + 2 * p] = y0 * c2[p] - y1 * s2[p];
                                acc[4 * j4 + 2 * p + 1] = fmaf(y0, s2[p], y1 * c2[p]);
                            }
                        }
                    }
#pragma unroll
                    for (int tt = 0; tt < 2; ++tt)
#pragma unroll
                        for (int j = 0; j < 8; ++j) {
                            const bf16_t y = to_bf16(acc[8 * tt + j]);
                            qf[2 * eb + tt][j] = y;
                            qss = fmaf((float)y, (float)y, qss);
                        }
                }
            }
            qss = xhalf_sum(qss);
        }
        unsigned char *smHi = smem, *smLo = smem + C::SS_BYTES;
        __syncthreads();                              // every wave is done with the K/V ring
#pragma unroll
        for (int i = 0; i < C::SCH; ++i) {
            const int id = tid + NT * i;              // 8-float piece: row id / CPR, column piece id % CPR
            if (id < D * C::CPR) {
                const float *sp = Sg + (size_t)(id / C::CPR) * D + 8 * (id % C::CPR);
                const f32x4 x0 = *(const f32x4 *)(sp);
                const f32x4 x1 = *(const f32x4 *)(sp + 4);
                union { u32x4 u; bf16x8 v; } hi, lo;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const float x = j < 4 ? x0[j] : x1[j - 4];
                    const bf16_t hb = to_bf16(x);
                    hi.v[j] = hb;
                    lo.v[j] = to_bf16(x - (float)hb);
                }
                const int off = (id / C::CPR) * C::VROW + 16 * (id % C::CPR);
                *(u32x4 *)(smHi + off) = hi.u;
                *(u32x4 *)(smLo + off) = lo.u;
            }
        }
        __syncthreads();
        f32x16 inter[C::DB];
#pragma unroll
        for (int db = 0; db < C::DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) inter[db][r] = 0.f;
        // k-slot j of half-wave hh must be d = 16t + 8hh + j to match q fragments loaded from memory, and
        // d = 16t + 8(j/4) + 4hh + j%4 to match fragments that were accumulator registers (fused feature map)
        const int s_row = fused_map ? ((lane & 15) >> 2) + 4 * hh : 8 * hh + ((lane & 15) >> 2);
        const int s_second = (fused_map ? 8 : 4) * C::VROW;
        const int s_frag_off = s_row * C::VROW + 32 * ((lane >> 4) & 1) + 8 * (lane & 3);
#pragma unroll
        for (int t = 0; t < C::KS; ++t)
#pragma unroll
            for (int db = 0; db < C::DB; ++db) {
                const unsigned char *p = smHi + s_frag_off + 16 * t * C::VROW + 64 * db;
                const bf16x8 sh = __builtin_shufflevector(lds_read_tr(p), lds_read_tr(p + s_second), 0, 1, 2, 3, 4, 5, 6, 7);
                const bf16x8 sl = __builtin_shufflevector(lds_read_tr(p + C::SS_BYTES), lds_read_tr(p + C::SS_BYTES + s_second),
                                                          0, 1, 2, 3, 4, 5, 6, 7);
                inter[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(sh, qf[t], inter[db], 0, 0, 0);
                inter[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(sl, qf[t], inter[db], 0, 0, 0);
            }
        // gate * L2 norm scale for this lane's query row
        float gq = 1.0f / sqrtf(qss + a.l2_eps);
        const size_t gtok = (size_t)b * Lq + (qrow < Lq ? qrow : 0);
        const size_t gi = a.g_per_token ? gtok : gtok * H + h;
        if (a.g != nullptr && !a.g_per_element && qrow < Lq)
            gq *= a.g_is_bf16 ? (float)((const bf16_t *)a.g)[gi] : ((const float *)a.g)[gi];
        if (a.g != nullptr && a.g_per_element) {
            // one gate per output feature: registers 4 j .. 4 j + 3 of block db are features 32 db + 8 j + 4 hh + 0..3
#pragma unroll
            for (int db = 0; db < C::DB; ++db)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const size_t ge = gi * D + 32 * db + 8 * j + 4 * hh;
                    float g4[4];
                    if (a.g_is_bf16) {
                        const bf16x4 x = *(const bf16x4 *)((const bf16_t *)a.g + ge);
#pragma unroll
                        for (int i = 0; i < 4; ++i) g4[i] = (float)x[i];
                    } else {
                        const f32x4 x = *(const f32x4 *)((const float *)a.g + ge);
#pragma unroll
                        for (int i = 0; i < 4; ++i) g4[i] = x[i];
                    }
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        o_acc[db][4 * j + i] = fmaf(gq * g4[i], inter[db][4 * j + i], o_acc[db][4 * j + i]);
                }
        } else {
#pragma unroll
            for (int db = 0; db < C::DB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) o_acc[db][r] = fmaf(gq, inter[db][r], o_acc[db][r]);
        }
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
    for (int i = 0; i < C::CPR / 2; ++i) {
        const int idx = lane + 64 * i;
        const int row = idx / C::CPR, col = idx % C::CPR;
        const int orow = q0 + row;
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
    // the kernel addresses one stream's K (or V) with 32-bit byte offsets
    if ((long long)(a.Lkv + 4 * BN) * a.H * a.D * 2 > 0x7fffffffLL) return hipErrorInvalidValue;
    const float scale_log2 = a.sm_scale * 1.4426950408889634f;
    const dim3 grid((unsigned)nwg), block(NT);
    // more workgroups than CUs, a ragged last query tile per head, and whole heads per XCD
    const int ragged_last = nwg > kNumCu && a.Lq % BM != 0 && n_qtiles > 1 && ((long long)a.B * a.H) % kNumXcd == 0;
    if (a.D == 128) return launch_kernel(fwd_bf16_kernel<128>, grid, block, stream, a, n_qtiles, scale_log2, ragged_last);
    if (a.D == 64) return launch_kernel(fwd_bf16_kernel<64>, grid, block, stream, a, n_qtiles, scale_log2, ragged_last);
    return hipErrorInvalidValue;
}

}  // namespace arl2
