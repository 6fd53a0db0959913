// Post-denoise state commit on bf16 MFMA (gfx950):
//   S <- gate * S + sum_i k'_i^T v_i,   k'_i = k_i / sqrt(|k_i|^2 + eps)     paper Eq. (3), Eq. (4)
//
// HBM-bound: every k and v element is read once.  The contraction runs over tokens, so both MFMA
// operands are needed token-major per feature; 64-token tiles of K and V are written to LDS row-major
// (as they arrive, 16-byte pieces) and read back through the transposing LDS read
// (ds_read_b64_tr_b16), which hands every lane four tokens of one feature.  To keep the fp32 state
// accurate the raw bf16 K (exact) is one operand and the row-scaled values r_i * v_i, split into
// bf16 hi + lo parts, are the other (two MFMAs per step, error ~2^-17; one bf16 rounding of the
// scaled values would cost ~1e-3 on the state).  The scale r_i = 1/sqrt(|k_i|^2 + eps) is computed
// from the K registers on their way to LDS (lane shuffles across the 16 lanes that share a row).
//
// Tokens are split over `nsplit` workgroups per (stream, head); each keeps the next tile's loads in
// flight while it works on the current one (8 wavefronts, each a 64 x 32 block of the partial, operand
// fragments of the next 16-token step requested before the MFMAs of the current one) and finally
// writes a D x D fp32 partial to the workspace.
// A second kernel adds the partials in split order and applies the gate to the old state, so the
// result is bit-identical from run to run (no floating-point atomics).
//
// Delta-rule variant (Eq. (4) literally, frame level):
//   S <- alpha S + beta K'^T (V - K' S) = alpha S + beta (K'^T V - (K'^T K') S)
// needs no [L x D] intermediate: the same pass over the tokens also accumulates the Gram matrix
// K'^T K' (raw K against r_i^2 k_i split into hi + lo), and the reduce kernel multiplies the summed
// Gram matrix with a snapshot of the old state in fp32.
#include "arl2_device.h"

#include <type_traits>

namespace arl2 {
namespace {

constexpr int BT = 64;    // tokens per tile
constexpr int NT = 512;    // partial kernel: 8 wavefronts, two per SIMD
constexpr int NTR = 256;   // reduce kernels


constexpr int PFT = 3;     // tiles whose loads are in flight (register ring): HBM latency is several tile times
constexpr int PFW = 3;     // the same for the producer wavefronts of the plain commit, which hold no accumulators

template <int D, bool DELTA>
struct CommitCfg {
    static constexpr int CPR = D / 8;                   // 16-byte chunks per row
    static constexpr int ROW = 2 * D + 64;              // LDS bytes per tile row (conflict-free transposing reads)
    static constexpr int MAT = BT * ROW;                // one 64-token tile
    static constexpr int NMAT = DELTA ? 5 : 3;          // K, V' hi, V' lo (, K'' hi, K'' lo with K'' = r^2 k)
    static constexpr int STAGE = NMAT * MAT;
    static constexpr int NSTG = DELTA ? 1 : 2;          // LDS stages (160 KB of LDS hold two 3-matrix stages or one 5-matrix stage)
    static constexpr int NACC = DELTA ? 2 : 1;          // accumulated D x D matrices
    static constexpr int KCH = BT * CPR / NT;           // chunks per thread per tile (K and V each)
    static constexpr int ROWS_PER_PASS = NT / CPR;
    static constexpr int DH = D / 64;                   // 64-row halves of the output
    static constexpr int EB = D / 32;                   // 32-column blocks of the output
    static constexpr int WAVES_USED = DH * EB;          // wavefronts that own a 64 x 32 output block (8 for D = 128)
    static_assert(KCH >= 1, "tile too small for the workgroup");
};

template <int D, bool DELTA>
__global__ __launch_bounds__(NT, 2) void commit_partial_kernel(CommitArgs a)
{
    using C = CommitCfg<D, DELTA>;
    __shared__ __attribute__((aligned(16))) unsigned char smem[C::NSTG * C::STAGE];

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, hh = lane >> 5;
    const int split = blockIdx.x % a.nsplit;
    const int bh = blockIdx.x / a.nsplit;
    const int h = bh % a.H, b = bh / a.H;
    const int L = a.L, H = a.H;
    const uint32_t tok_bytes = (uint32_t)H * D * 2;
    const bf16_t *kg = (const bf16_t *)a.k + ((size_t)b * L * H + h) * D;
    const bf16_t *vg = (const bf16_t *)a.v + ((size_t)b * L * H + h) * D;
    const uint32_t range = (uint32_t)(L - 1) * tok_bytes + 2 * D;      // bytes of this head's slice
    const __amdgpu_buffer_rsrc_t k_rsrc = make_rsrc(kg, range);
    const __amdgpu_buffer_rsrc_t v_rsrc = make_rsrc(vg, range);

    const int ntiles = (L + BT - 1) / BT;
    const int t_begin = (int)((long long)split * ntiles / a.nsplit);
    const int t_end = (int)((long long)(split + 1) * ntiles / a.nsplit);

    // chunk i of this thread: row (tid / CPR) + ROWS_PER_PASS * i, 16-byte column tid % CPR
    const int lds_off = (tid / C::CPR) * C::ROW + 16 * (tid % C::CPR);
    u32x4 kr[PFT][C::KCH], vr[PFT][C::KCH];
    // Requests tile `tile` into register buffer `buf` (rows past the end of the sequence read as zero; a
    // tile that is not this workgroup's is not requested at all: its offsets are put beyond the buffer,
    // which keeps the loop free of branches around loads).
    auto load_tile = [&](int tile, auto buf_) {
        constexpr int buf = decltype(buf_)::value;
        const uint32_t base = tile < t_end ? ((uint32_t)tile * BT + tid / C::CPR) * tok_bytes + 16 * (tid % C::CPR) : 0x80000000u;
#pragma unroll
        for (int i = 0; i < C::KCH; ++i) {
            const uint32_t off = base + (uint32_t)i * C::ROWS_PER_PASS * tok_bytes;
            kr[buf][i] = __builtin_amdgcn_raw_buffer_load_b128(k_rsrc, off, 0, 0);
            vr[buf][i] = __builtin_amdgcn_raw_buffer_load_b128(v_rsrc, off, 0, 0);
        }
    };
    // K as it is, and r * V split into bf16 hi + lo, into the LDS stage
    auto stage_tile = [&](int stage, auto buf_) {
        constexpr int buf = decltype(buf_)::value;
        unsigned char *sm = smem + stage * C::STAGE + lds_off;
#pragma unroll
        for (int i = 0; i < C::KCH; ++i) {
            float ss = 0.f;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float lo = __uint_as_float(kr[buf][i][w] << 16);
                const float hi = __uint_as_float(kr[buf][i][w] & 0xffff0000u);
                ss = fmaf(lo, lo, ss);
                ss = fmaf(hi, hi, ss);
            }
            ss = lane_group_sum<C::CPR>(ss);
            const float rn = fast_rsqrt(ss + a.l2_eps);
            const float rn2 = rn * rn;
            union { u32x4 u; bf16x8 v; } vh, vl;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float s0 = __uint_as_float(vr[buf][i][w] << 16) * rn;
                const float s1 = __uint_as_float(vr[buf][i][w] & 0xffff0000u) * rn;
                const bf16_t h0 = to_bf16(s0), h1 = to_bf16(s1);
                vh.v[2 * w] = h0;
                vh.v[2 * w + 1] = h1;
                vl.v[2 * w] = to_bf16(s0 - (float)h0);
                vl.v[2 * w + 1] = to_bf16(s1 - (float)h1);
            }
            unsigned char *p = sm + i * C::ROWS_PER_PASS * C::ROW;
            *(u32x4 *)(p) = kr[buf][i];
            *(u32x4 *)(p + C::MAT) = vh.u;
            *(u32x4 *)(p + 2 * C::MAT) = vl.u;
            if constexpr (DELTA) {
                union { u32x4 u; bf16x8 v; } kh, kl;
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    const float s0 = __uint_as_float(kr[buf][i][w] << 16) * rn2;
                    const float s1 = __uint_as_float(kr[buf][i][w] & 0xffff0000u) * rn2;
                    const bf16_t h0 = to_bf16(s0), h1 = to_bf16(s1);
                    kh.v[2 * w] = h0;
                    kh.v[2 * w + 1] = h1;
                    kl.v[2 * w] = to_bf16(s0 - (float)h0);
                    kl.v[2 * w + 1] = to_bf16(s1 - (float)h1);
                }
                *(u32x4 *)(p + 3 * C::MAT) = kh.u;
                *(u32x4 *)(p + 4 * C::MAT) = kl.u;
            }
        }
    };

    // this wavefront's 64 x 32 block of the D x D partial: feature blocks d0, d0+1 x e0
    const bool compute = wave < C::WAVES_USED;
    const int d0 = 2 * (wave / C::EB), e0 = wave % C::EB;
    const int tr_off = (((lane & 15) >> 2) + 4 * hh) * C::ROW + 32 * ((lane >> 4) & 1) + 8 * (lane & 3);
    f32x16 acc[C::NACC][2];
#pragma unroll
    for (int m = 0; m < C::NACC; ++m)
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[m][i][r] = 0.f;

    if constexpr (DELTA) {
        // the reduce kernel multiplies the Gram matrix with the old state while it overwrites S:
        // split 0 of every (stream, head) leaves a snapshot of the old state in the workspace
        if (split == 0) {
            const f32x4 *src = (const f32x4 *)(a.S + (size_t)bh * D * D);
            f32x4 *dst = (f32x4 *)((float *)a.workspace + (size_t)a.B * H * a.nsplit * 2 * D * D + (size_t)bh * D * D);
            for (int i = tid; i < D * D / 4; i += NT) dst[i] = src[i];
        }
    }

    static_for<0, PFT>([&](auto i_) { load_tile(t_begin + decltype(i_)::value, i_); });
    for (int tile0 = t_begin; tile0 < t_end; tile0 += PFT) {
        static_for<0, PFT>([&](auto i_) {
            const int tile = tile0 + decltype(i_)::value;
            if (tile >= t_end) return;                  // uniform over the workgroup
            const int stage = C::NSTG == 2 ? ((tile - t_begin) & 1) : 0;
            if constexpr (C::NSTG == 1) __syncthreads();   // single stage: the previous tile's MFMAs are done
            stage_tile(stage, i_);           // waits for this tile's loads
            __syncthreads();                 // two stages: every wave is also done with the tile before last
            load_tile(tile + PFT, i_);
            if (compute) {
                const unsigned char *sm = smem + stage * C::STAGE + tr_off;
                // operand fragments of 16-token step t: tokens 16t + 4hh + 0..3 and 16t + 8 + 4hh + 0..3
                bf16x8 ka[2][2], bh_[2][C::NACC], bl_[2][C::NACC];
                auto load_step = [&](int t, int buf) {
                    const unsigned char *row = sm + 16 * t * C::ROW;
#pragma unroll
                    for (int i = 0; i < 2; ++i) ka[buf][i] = lds_read_tr_pair(row + 64 * (d0 + i), 8 * C::ROW);
#pragma unroll
                    for (int m = 0; m < C::NACC; ++m) {      // m = 0: r V,  m = 1: r^2 K
                        bh_[buf][m] = lds_read_tr_pair(row + (1 + 2 * m) * C::MAT + 64 * e0, 8 * C::ROW);
                        bl_[buf][m] = lds_read_tr_pair(row + (2 + 2 * m) * C::MAT + 64 * e0, 8 * C::ROW);
                    }
                };
                load_step(0, 0);
#pragma unroll
                for (int t = 0; t < BT / 16; ++t) {
                    if (t + 1 < BT / 16) load_step(t + 1, (t + 1) & 1);
#pragma unroll
                    for (int m = 0; m < C::NACC; ++m)
#pragma unroll
                        for (int i = 0; i < 2; ++i) {
                            acc[m][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[t & 1][i], bh_[t & 1][m], acc[m][i], 0, 0, 0);
                            acc[m][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[t & 1][i], bl_[t & 1][m], acc[m][i], 0, 0, 0);
                        }
                }
            }
        });
    }

    // partial[bh][split][matrix][d][e]
    if (compute) {
#pragma unroll
        for (int m = 0; m < C::NACC; ++m) {
            float *part = (float *)a.workspace + (((size_t)bh * a.nsplit + split) * C::NACC + m) * D * D;
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int d = 32 * (d0 + i) + 8 * (r >> 2) + 4 * hh + (r & 3);
                    const int e = 32 * e0 + (lane & 31);
                    part[(size_t)d * D + e] = acc[m][i][r];
                }
        }
    }
}

// Plain commit, producer / consumer form of the kernel above.  Staging a tile (row norms, scaling, hi/lo
// split: vector ALU) and contracting it (MFMA) take about the same time, and a wavefront does not overlap
// its own VALU work with its own MFMAs: wavefronts 0..3 (one per SIMD) only fetch and stage tile i + 1 into
// the other LDS stage while wavefronts 4..7 (one per SIMD) only run the MFMAs of tile i, each on a 64 x 64
// block of the partial; one workgroup barrier per tile hands the stages over.
template <int D>
__global__ __launch_bounds__(NT, 2) void commit_partial_ws_kernel(CommitArgs a)
{
    using C = CommitCfg<D, false>;
    constexpr int PT = NT / 2;                           // producer threads
    constexpr int KCHP = BT * C::CPR / PT;               // chunks per producer thread per tile (K and V each)
    constexpr int RPP = PT / C::CPR;                     // rows per pass of the producers
    constexpr int NE = D / 64;                           // 32-column blocks per consumer wavefront
    static_assert(KCHP >= 1 && NE >= 1, "unsupported head dimension");
    __shared__ __attribute__((aligned(16))) unsigned char smem[2 * C::STAGE];

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, hh = lane >> 5;
    const bool producer = wave < 4;
    const int split = blockIdx.x % a.nsplit;
    const int bh = blockIdx.x / a.nsplit;
    const int h = bh % a.H, b = bh / a.H;
    const int L = a.L, H = a.H;
    const uint32_t tok_bytes = (uint32_t)H * D * 2;
    const bf16_t *kg = (const bf16_t *)a.k + ((size_t)b * L * H + h) * D;
    const bf16_t *vg = (const bf16_t *)a.v + ((size_t)b * L * H + h) * D;
    const uint32_t range = (uint32_t)(L - 1) * tok_bytes + 2 * D;      // bytes of this head's slice
    const __amdgpu_buffer_rsrc_t k_rsrc = make_rsrc(kg, range);
    const __amdgpu_buffer_rsrc_t v_rsrc = make_rsrc(vg, range);

    const int ntiles = (L + BT - 1) / BT;
    const int t_begin = (int)((long long)split * ntiles / a.nsplit);
    const int t_end = (int)((long long)(split + 1) * ntiles / a.nsplit);
    const int n = t_end - t_begin;

    // ---- producers: chunk i of a thread is row (tid / CPR) + RPP * i, 16-byte column tid % CPR
    const int lds_off = (tid / C::CPR) * C::ROW + 16 * (tid % C::CPR);
    u32x4 kr[PFW][KCHP], vr[PFW][KCHP];
    auto load_tile = [&](int tile, auto buf_) {     // a tile that is not this workgroup's is not requested
        constexpr int buf = decltype(buf_)::value;
        const uint32_t base = tile < t_end ? ((uint32_t)tile * BT + tid / C::CPR) * tok_bytes + 16 * (tid % C::CPR) : 0x80000000u;
#pragma unroll
        for (int i = 0; i < KCHP; ++i) {
            const uint32_t off = base + (uint32_t)i * RPP * tok_bytes;
            kr[buf][i] = __builtin_amdgcn_raw_buffer_load_b128(k_rsrc, off, 0, 0);
            vr[buf][i] = __builtin_amdgcn_raw_buffer_load_b128(v_rsrc, off, 0, 0);
        }
    };
    auto stage_tile = [&](int stage, auto buf_) {   // K as it is, and r * V split into bf16 hi + lo
        constexpr int buf = decltype(buf_)::value;
        unsigned char *sm = smem + stage * C::STAGE + lds_off;
#pragma unroll
        for (int i = 0; i < KCHP; ++i) {
            float ss = 0.f;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float lo = __uint_as_float(kr[buf][i][w] << 16);
                const float hi = __uint_as_float(kr[buf][i][w] & 0xffff0000u);
                ss = fmaf(lo, lo, ss);
                ss = fmaf(hi, hi, ss);
            }
            ss = lane_group_sum<C::CPR>(ss);
            const float rn = fast_rsqrt(ss + a.l2_eps);
            // r * v as bf16 hi (truncated) + lo (rounded remainder): both members of a pair packed into one word
            u32x4 vh, vl;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                uint32_t h0, h1;
                float l0, l1;
                split_bf16_trunc(__uint_as_float(vr[buf][i][w] << 16) * rn, h0, l0);
                split_bf16_trunc(__uint_as_float(vr[buf][i][w] & 0xffff0000u) * rn, h1, l1);
                vh[w] = (h0 >> 16) | h1;
                union { bf16x2 v; uint32_t u; } pk;
                pk.v[0] = to_bf16(l0);
                pk.v[1] = to_bf16(l1);
                vl[w] = pk.u;
            }
            unsigned char *p = sm + i * RPP * C::ROW;
            *(u32x4 *)(p) = kr[buf][i];
            *(u32x4 *)(p + C::MAT) = vh;
            *(u32x4 *)(p + 2 * C::MAT) = vl;
        }
    };

    // ---- consumers: wavefront 4 + cw owns rows 64 dh .. 64 dh + 63, column blocks e0 .. e0 + NE - 1
    const int cw = wave - 4;
    const bool consumer = !producer && cw * NE < C::DH * C::EB;
    const int dh = (cw * NE) / C::EB, e0 = (cw * NE) % C::EB;
    const int tr_off = (((lane & 15) >> 2) + 4 * hh) * C::ROW + 32 * ((lane >> 4) & 1) + 8 * (lane & 3);
    f32x16 acc[2][NE];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int e = 0; e < NE; ++e)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][e][r] = 0.f;
    auto consume = [&](int stage) {
        const unsigned char *sm = smem + stage * C::STAGE + tr_off;
        // operand fragments of 16-token step t: tokens 16t + 4hh + 0..3 and 16t + 8 + 4hh + 0..3
        bf16x8 ka[2][2], bh_[2][NE], bl_[2][NE];
        auto load_step = [&](int t, int buf) {
            const unsigned char *row = sm + 16 * t * C::ROW;
#pragma unroll
            for (int i = 0; i < 2; ++i) ka[buf][i] = lds_read_tr_pair(row + 64 * (2 * dh + i), 8 * C::ROW);
#pragma unroll
            for (int e = 0; e < NE; ++e) {
                bh_[buf][e] = lds_read_tr_pair(row + C::MAT + 64 * (e0 + e), 8 * C::ROW);
                bl_[buf][e] = lds_read_tr_pair(row + 2 * C::MAT + 64 * (e0 + e), 8 * C::ROW);
            }
        };
        load_step(0, 0);
#pragma unroll
        for (int t = 0; t < BT / 16; ++t) {
            if (t + 1 < BT / 16) load_step(t + 1, (t + 1) & 1);
#pragma unroll
            for (int e = 0; e < NE; ++e)
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    acc[i][e] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[t & 1][i], bh_[t & 1][e], acc[i][e], 0, 0, 0);
                    acc[i][e] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[t & 1][i], bl_[t & 1][e], acc[i][e], 0, 0, 0);
                }
        }
    };

    // tile k of this workgroup (k = 0 .. n - 1) travels through register buffer k % PFW and LDS stage k % 2
    if (producer) {
        static_for<0, PFW>([&](auto i_) { load_tile(t_begin + decltype(i_)::value, i_); });
        if (n > 0) {
            stage_tile(0, std::integral_constant<int, 0>{});
            load_tile(t_begin + PFW, std::integral_constant<int, 0>{});
        }
    }
    __syncthreads();
    for (int i0 = 0; i0 < n; i0 += PFW) {
        static_for<0, PFW>([&](auto j_) {
            constexpr int j = decltype(j_)::value;
            const int i = i0 + j;
            if (i >= n) return;                          // uniform over the workgroup
            if (producer) {
                if (i + 1 < n) {
                    const std::integral_constant<int, (j + 1) % PFW> nb{};
                    stage_tile((i + 1) & 1, nb);
                    load_tile(t_begin + i + 1 + PFW, nb);
                }
            } else if (consumer) {
                consume(i & 1);
            }
            __syncthreads();
        });
    }

    // partial[bh][split][d][e]
    if (consumer) {
        float *part = (float *)a.workspace + ((size_t)bh * a.nsplit + split) * D * D;
#pragma unroll
        for (int e = 0; e < NE; ++e)
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int d = 32 * (2 * dh + i) + 8 * (r >> 2) + 4 * hh + (r & 3);
                    const int col = 32 * (e0 + e) + (lane & 31);
                    part[(size_t)d * D + col] = acc[i][e][r];
                }
    }
}

// Delta rule: S[bh] = alpha S_old + beta (M - G S_old) with M, G the split-ordered sums of the two
// partial matrices and S_old the snapshot taken by the partial kernel.  One workgroup owns 8 rows d.
template <int D>
__global__ __launch_bounds__(NTR) void commit_delta_reduce_kernel(CommitArgs a)
{
    constexpr int ROWS = NTR / (D / 4);                // rows per workgroup (8 for D = 128, 16 for D = 64)
    __shared__ float Gs[ROWS][D];
    const int wg_per_head = D / ROWS;
    const int bh = blockIdx.x / wg_per_head;
    const int r = threadIdx.x / (D / 4), e4 = threadIdx.x % (D / 4);
    const int d = (blockIdx.x % wg_per_head) * ROWS + r;
    const size_t dd = (size_t)D * D;
    const float *part = (const float *)a.workspace + (size_t)bh * a.nsplit * 2 * dd + (size_t)d * D + 4 * e4;
    const float *Sold = (const float *)a.workspace + (size_t)a.B * a.H * a.nsplit * 2 * dd + (size_t)bh * dd;
    f32x4 m = {0.f, 0.f, 0.f, 0.f}, g = {0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < a.nsplit; ++s) {
        const f32x4 pm = *(const f32x4 *)(part + (size_t)s * 2 * dd);
        const f32x4 pg = *(const f32x4 *)(part + (size_t)s * 2 * dd + dd);
#pragma unroll
        for (int c = 0; c < 4; ++c) { m[c] += pm[c]; g[c] += pg[c]; }
    }
    *(f32x4 *)&Gs[r][4 * e4] = g;
    __syncthreads();
    f32x4 t = {0.f, 0.f, 0.f, 0.f};                    // (G S_old)[d][4 e4 .. +3]
    for (int j = 0; j < D; ++j) {
        const float gj = Gs[r][j];
        const f32x4 sj = *(const f32x4 *)(Sold + (size_t)j * D + 4 * e4);
#pragma unroll
        for (int c = 0; c < 4; ++c) t[c] = fmaf(gj, sj[c], t[c]);
    }
    const float alpha = a.gate[bh], beta = a.beta[bh];
    const f32x4 old = *(const f32x4 *)(Sold + (size_t)d * D + 4 * e4);
    f32x4 res;
#pragma unroll
    for (int c = 0; c < 4; ++c) res[c] = fmaf(alpha, old[c], beta * (m[c] - t[c]));
    *(f32x4 *)(a.S + (size_t)bh * dd + (size_t)d * D + 4 * e4) = res;
}

// S[bh] = gate[bh] * S[bh] + sum_{split ascending} partial[bh][split]
template <int NS>
__global__ __launch_bounds__(NTR) void commit_reduce_kernel(CommitArgs a, int vec_per_head)
{
    const int bh = blockIdx.x / (vec_per_head / NTR);
    const int vi = (blockIdx.x % (vec_per_head / NTR)) * NTR + threadIdx.x;
    const size_t head_elems = (size_t)vec_per_head * 4;
    const f32x4 *part = (const f32x4 *)((const float *)a.workspace + (size_t)bh * a.nsplit * head_elems) + vi;
    f32x4 *Sg = (f32x4 *)(a.S + (size_t)bh * head_elems);
    const float gate = a.gate[bh];
    const f32x4 old = Sg[vi];
    f32x4 sum = {0.f, 0.f, 0.f, 0.f};
    // all loads of a batch are issued before the adds; the adds run in split order
    for (int s0 = 0; s0 < a.nsplit; s0 += NS) {
        f32x4 x[NS];
#pragma unroll
        for (int j = 0; j < NS; ++j) {
            const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
            x[j] = (s0 + j < a.nsplit) ? part[(size_t)(s0 + j) * vec_per_head] : zero;
        }
#pragma unroll
        for (int j = 0; j < NS; ++j)
#pragma unroll
            for (int c = 0; c < 4; ++c) sum[c] += x[j][c];
    }
    f32x4 res;
#pragma unroll
    for (int c = 0; c < 4; ++c) res[c] = fmaf(gate, old[c], sum[c]);
    Sg[vi] = res;
}

}  // namespace

int commit_nsplit(int B, int H, int L)
{
    const int ntiles = (L + BT - 1) / BT;
    const long long bh = (long long)B * H;
    long long want = (192 + bh - 1) / bh;      // enough workgroups in flight to saturate HBM
    if (want < 1) want = 1;
    if (want > ntiles) want = ntiles;
    if (want > 32) want = 32;
    return (int)want;
}

hipError_t launch_commit_reduce_bf16(const CommitArgs &a, hipStream_t stream)
{
    const int vec_per_head = a.D * a.D / 4;        // multiple of 256 for D in {64, 128}
    const long long rwg = (long long)a.B * a.H * (vec_per_head / NTR);
    if (rwg <= 0 || rwg > 0x7fffffffLL) return hipErrorInvalidValue;
    return launch_kernel(commit_reduce_kernel<8>, dim3((unsigned)rwg), dim3(NTR), stream, a, vec_per_head);
}

hipError_t launch_commit_bf16(const CommitArgs &a, hipStream_t stream)
{
    const long long nwg = (long long)a.B * a.H * a.nsplit;
    if (nwg <= 0 || nwg > 0x7fffffffLL) return hipErrorInvalidValue;
    // the kernel addresses one stream's K (or V) with 32-bit byte offsets
    if ((long long)(a.L + 4 * BT) * a.H * a.D * 2 > 0x7fffffffLL) return hipErrorInvalidValue;
    const bool delta = a.beta != nullptr;
    hipError_t e;
    if (a.D == 128 && !delta)
        e = launch_kernel(commit_partial_ws_kernel<128>, dim3((unsigned)nwg), dim3(NT), stream, a);
    else if (a.D == 64 && !delta)
        e = launch_kernel(commit_partial_ws_kernel<64>, dim3((unsigned)nwg), dim3(NT), stream, a);
    else if (a.D == 128)
        e = launch_kernel(commit_partial_kernel<128, true>, dim3((unsigned)nwg), dim3(NT), stream, a);
    else if (a.D == 64)
        e = launch_kernel(commit_partial_kernel<64, true>, dim3((unsigned)nwg), dim3(NT), stream, a);
    else
        return hipErrorInvalidValue;
    if (e != hipSuccess) return e;
    if (delta) {
        const int rows = NTR / (a.D / 4);
        const long long rwg = (long long)a.B * a.H * (a.D / rows);
        if (a.D == 128) return launch_kernel(commit_delta_reduce_kernel<128>, dim3((unsigned)rwg), dim3(NTR), stream, a);
        return launch_kernel(commit_delta_reduce_kernel<64>, dim3((unsigned)rwg), dim3(NTR), stream, a);
    }
    return launch_commit_reduce_bf16(a, stream);
}

}  // namespace arl2
