// Token-sequential gated delta rule on bf16 MFMA (gfx950):
//   for j = 1..L:  S <- alpha_j S + beta_j k'_j^T (v_j - k'_j S),   k'_j = L2Norm(k_j)
// (paper Eq. (4) applied one token at a time with per-token gates, Sec. 3.2; Alg. 1 clean pass).
//
// Only the state after the last token is wanted: every denoising pass reads the state as it stood
// before the chunk (Sec. 3.3), so no per-token output exists.  That makes each block of 64 tokens a
// single affine map of the state, and the maps of all blocks can be built independently of S:
//
//   inside a block (gamma-_i = alpha_1..alpha_{i-1}, tail_i = alpha_{i+1}..alpha_64, gam = alpha_1..alpha_64)
//     A_ij  = beta_i (alpha_{j+1}..alpha_{i-1}) k'_i.k'_j   for j < i, else 0      (unit lower triangular I + A)
//     Z     = (I + A)^-T diag(tail) K'                       [64 x D]   back substitution
//     E     = (diag(beta gamma-) Z)^T K'                     [D x D]
//     Psi   = (diag(beta) Z)^T V                             [D x D]
//     S_out = gam S_in - E S_in + Psi
//
// Kernel 1 (one workgroup per block of tokens, all blocks in parallel) builds -E (as bf16 hi + lo parts),
// Psi (fp32) and gam.  The Gram matrix uses the raw bf16 keys (exact products) and is scaled in fp32;
// the triangular solve runs in fp32 on the vector ALU, one thread per feature; the two contractions
// over tokens run on MFMA with Z split into bf16 hi + lo against the raw bf16 K and V.
// Kernel 2 walks the blocks in order: one workgroup per (stream, head, 32 state columns), the state
// slice in accumulator registers, S <- gam S + Psi + (-E) S with -E hi/lo against S hi/lo (three MFMA
// terms, the lo x lo term is below fp32 rounding), the slice exchanged between wavefronts through LDS.
// All products of gates are formed by multiplication only, so gates of exactly zero are handled.
#include "arl2_device.h"

#include <type_traits>

namespace arl2 {
namespace {

constexpr int CT = 64;     // tokens per block
constexpr int NTA = 256;   // threads of the block kernel

typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;

__device__ __forceinline__ bf16x8 lds_read_tr_pair(const unsigned char *p, int second_row_bytes)
{
    const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4 *)(p));
    const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4 *)(p + second_row_bytes));
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}

template <int I, int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

template <int D>
struct GdnCfg {
    static constexpr int CPR = D / 8;                   // 16-byte chunks per row
    static constexpr int ROW = 2 * D + 32;              // LDS bytes per tile row
    static constexpr int TILE = CT * ROW;               // one 64-token bf16 tile
    static constexpr int KCH = CT * CPR / NTA;          // chunks per thread per tile
    static constexpr int ROWS_PER_PASS = NTA / CPR;
    static constexpr int AST = 68;                      // floats per row of the 64 x 64 fp32 matrices
    static constexpr int NB = D / 32;                   // 32-wide blocks per side of a D x D matrix
    static constexpr int EPW = NB * NB / 4;             // output blocks per wavefront (all in one block row)
    static constexpr int REG = TILE > CT * AST * 4 ? TILE : CT * AST * 4;   // a region holds a tile or a 64 x 64 fp32 matrix
    static constexpr int SC_OFF = 4 * REG;              // per-token scalars behind the four regions
    static constexpr int SMEM = SC_OFF + 5 * CT * 4 + 16;
    static_assert(KCH >= 1 && EPW >= 1, "unsupported head dimension");
};

// Bytes of workspace per block of tokens: -E hi, -E lo (bf16), Psi (fp32), gam (padded).
__host__ __device__ constexpr size_t gdn_block_bytes(int D) { return (size_t)D * D * 8 + 16; }

// ---- kernel 1: the affine map of one block of tokens -------------------------------------------------
template <int D>
__global__ __launch_bounds__(NTA, 2) void gdn_block_kernel(GdnArgs a, int nblk)
{
    using C = GdnCfg<D>;
    __shared__ __attribute__((aligned(16))) unsigned char smem[C::SMEM];
    unsigned char *R0 = smem, *R1 = smem + C::REG, *R2 = smem + 2 * C::REG, *R3 = smem + 3 * C::REG;
    float *sc_r = (float *)(smem + C::SC_OFF);          // 1 / sqrt(|k_i|^2 + eps)
    float *sc_al = sc_r + CT, *sc_be = sc_al + CT, *sc_gp = sc_be + CT, *sc_tl = sc_gp + CT, *sc_gam = sc_tl + CT;

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, hh = lane >> 5, c32 = lane & 31;
    const int blk = blockIdx.x % nblk;
    const int bh = blockIdx.x / nblk;
    const int h = bh % a.H, b = bh / a.H;
    const int L = a.L, H = a.H;
    const int tok0 = blk * CT;
    const uint32_t tok_bytes = (uint32_t)H * D * 2;
    const bf16_t *kg = (const bf16_t *)a.k + ((size_t)b * L * H + h) * D;
    const bf16_t *vg = (const bf16_t *)a.v + ((size_t)b * L * H + h) * D;
    const uint32_t range = (uint32_t)(L - 1) * tok_bytes + 2 * D;
    const __amdgpu_buffer_rsrc_t k_rsrc = make_rsrc(kg, range);
    const __amdgpu_buffer_rsrc_t v_rsrc = make_rsrc(vg, range);

    // ---- 1. K, V tiles (rows past the end read as zero), per-token scalars
    {
        const int row0 = tid / C::CPR, col = tid % C::CPR;
#pragma unroll
        for (int i = 0; i < C::KCH; ++i) {
            const int row = row0 + i * C::ROWS_PER_PASS;
            const uint32_t off = (uint32_t)(tok0 + row) * tok_bytes + 16 * col;
            const u32x4 kr = __builtin_amdgcn_raw_buffer_load_b128(k_rsrc, off, 0, 0);
            const u32x4 vr = __builtin_amdgcn_raw_buffer_load_b128(v_rsrc, off, 0, 0);
            float ss = 0.f;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float lo = __uint_as_float(kr[w] << 16);
                const float hi = __uint_as_float(kr[w] & 0xffff0000u);
                ss = fmaf(lo, lo, ss);
                ss = fmaf(hi, hi, ss);
            }
#pragma unroll
            for (int o = 1; o < C::CPR; o <<= 1) ss += __shfl_xor(ss, o, kWave);
            if (col == 0) sc_r[row] = 1.0f / sqrtf(ss + a.l2_eps);
            *(u32x4 *)(R0 + row * C::ROW + 16 * col) = kr;
            *(u32x4 *)(R1 + row * C::ROW + 16 * col) = vr;
        }
        if (tid < CT) {
            const int tok = tok0 + tid;
            float al = 1.f, be = 0.f;                    // padding tokens leave the state alone
            if (tok < L) {
                const size_t gi = ((size_t)b * L + tok) * H + h;
                al = a.alpha[gi];
                be = a.beta[gi];
            }
            sc_al[tid] = al;
            sc_be[tid] = be;
        }
    }
    __syncthreads();

    // ---- 2. products of gates (wavefront 0) and the Gram matrix of the raw keys (all wavefronts)
    if (tid < CT) {
        float gp = 1.f, tl = 1.f;
        for (int m = 0; m < tid; ++m) gp *= sc_al[m];
        for (int m = tid + 1; m < CT; ++m) tl *= sc_al[m];
        sc_gp[tid] = gp;
        sc_tl[tid] = tl;
        if (tid == CT - 1) sc_gam[0] = gp * sc_al[tid];
    }
    {
        const int ib = wave >> 1, jb = wave & 1;         // rows i, columns j of the 64 x 64 Gram matrix
        if (jb <= ib) {                                  // the strictly upper block is never used
            f32x16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int t = 0; t < D / 16; ++t) {
                const bf16x8 ka = *(const bf16x8 *)(R0 + (32 * ib + c32) * C::ROW + 32 * t + 16 * hh);
                const bf16x8 kb = *(const bf16x8 *)(R0 + (32 * jb + c32) * C::ROW + 32 * t + 16 * hh);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, kb, acc, 0, 0, 0);
            }
            float *Gs = (float *)R2;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int i = 32 * ib + 8 * (r >> 2) + 4 * hh + (r & 3);
                Gs[i * C::AST + 32 * jb + c32] = acc[r];
            }
        }
    }
    __syncthreads();

    // ---- 3. At[j][i] = A_ij = beta_i (alpha_{j+1} .. alpha_{i-1}) r_i r_j G_ij  (i > j), thread = column j
    if (tid < CT) {
        const float *Gs = (const float *)R2;
        float *At = (float *)R3;
        const int j = tid;
        const float rj = sc_r[j];
        float rho = 1.f;
        for (int i = j + 1; i < CT; ++i) {
            At[j * C::AST + i] = sc_be[i] * rho * sc_r[i] * rj * Gs[i * C::AST + j];
            rho *= sc_al[i];
        }
    }
    __syncthreads();

    // ---- 4. back substitution (I + A)^T Z = diag(tail r) K, thread = feature
    float z[CT];
    if (tid < D) {
        const float *At = (const float *)R3;
        static_for<0, CT>([&](auto ii_) {
            constexpr int i = CT - 1 - decltype(ii_)::value;
            float acc = sc_tl[i] * sc_r[i] * (float)*(const bf16_t *)(R0 + i * C::ROW + 2 * tid);
            static_for<(i + 1) / 4, CT / 4>([&](auto q_) {
                constexpr int q = decltype(q_)::value;
                const f32x4 a4 = *(const f32x4 *)(At + i * C::AST + 4 * q);
                static_for<0, 4>([&](auto e_) {
                    constexpr int j = 4 * q + decltype(e_)::value;
                    if constexpr (j > i) acc = fmaf(-a4[j - 4 * q], z[j], acc);
                });
            });
            z[i] = acc;
        });
    }
    __syncthreads();                                     // At and G are dead: R2, R3 become the Z tiles

    // Z scaled per token, negated if asked, split into bf16 hi (R2) + lo (R3)
    auto put_z = [&](bool for_e) {
        if (tid < D) {
#pragma unroll
            for (int i = 0; i < CT; ++i) {
                const float s = for_e ? -(sc_be[i] * sc_gp[i] * sc_r[i]) : sc_be[i];
                const float x = s * z[i];
                const bf16_t hi = to_bf16(x);
                *(bf16_t *)(R2 + i * C::ROW + 2 * tid) = hi;
                *(bf16_t *)(R3 + i * C::ROW + 2 * tid) = to_bf16(x - (float)hi);
            }
        }
    };
    // acc[n] = (Z tile)^T (X tile) for this wavefront's blocks: rows d in block dblk, columns in blocks eblk0 + n
    const int dblk = (wave * C::EPW) / C::NB, eblk0 = (wave * C::EPW) % C::NB;
    const int tr_off = (((lane & 15) >> 2) + 4 * hh) * C::ROW + 32 * ((lane >> 4) & 1) + 8 * (lane & 3);
    f32x16 acc[C::EPW];
    auto contract = [&](const unsigned char *X) {
#pragma unroll
        for (int n = 0; n < C::EPW; ++n)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[n][r] = 0.f;
#pragma unroll
        for (int t = 0; t < CT / 16; ++t) {
            const int row = tr_off + 16 * t * C::ROW;
            const bf16x8 zh = lds_read_tr_pair(R2 + row + 64 * dblk, 8 * C::ROW);
            const bf16x8 zl = lds_read_tr_pair(R3 + row + 64 * dblk, 8 * C::ROW);
#pragma unroll
            for (int n = 0; n < C::EPW; ++n) {
                const bf16x8 xb = lds_read_tr_pair(X + row + 64 * (eblk0 + n), 8 * C::ROW);
                acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(zh, xb, acc[n], 0, 0, 0);
                acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(zl, xb, acc[n], 0, 0, 0);
            }
        }
    };

    unsigned char *out = (unsigned char *)a.workspace + ((size_t)bh * nblk + blk) * gdn_block_bytes(D);
    bf16_t *Ehi = (bf16_t *)out, *Elo = Ehi + D * D;
    float *Psi = (float *)(out + (size_t)D * D * 4);
    float *gam = (float *)(out + (size_t)D * D * 8);

    // ---- 5. -E = (-diag(beta gamma- r) Z)^T K
    put_z(true);
    __syncthreads();
    contract(R0);
#pragma unroll
    for (int n = 0; n < C::EPW; ++n)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int d = 32 * dblk + 8 * (r >> 2) + 4 * hh + (r & 3);
            const int e = 32 * (eblk0 + n) + c32;
            const float x = acc[n][r];
            const bf16_t hi = to_bf16(x);
            Ehi[d * D + e] = hi;
            Elo[d * D + e] = to_bf16(x - (float)hi);
        }
    __syncthreads();                                     // every wavefront is done reading the Z tiles

    // ---- 6. Psi = (diag(beta) Z)^T V
    put_z(false);
    __syncthreads();
    contract(R1);
#pragma unroll
    for (int n = 0; n < C::EPW; ++n)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int d = 32 * dblk + 8 * (r >> 2) + 4 * hh + (r & 3);
            const int e = 32 * (eblk0 + n) + c32;
            Psi[d * D + e] = acc[n][r];
        }
    if (tid == 0) gam[0] = sc_gam[0];
}

// ---- kernel 2: S <- gam S + Psi + (-E) S over the blocks in order ---------------------------------------
template <int D>
__global__ __launch_bounds__(2 * D) void gdn_scan_kernel(GdnArgs a, int nblk)
{
    constexpr int KS = D / 16;                           // k-steps of the D-long contraction
    constexpr int SROW = 2 * D + 16;                     // LDS bytes per state column (conflict-free b128 reads)
    constexpr int SBUF = 32 * SROW;                      // one bf16 part of the 32-column slice, stored [column][row]
    __shared__ __attribute__((aligned(16))) unsigned char smem[4 * SBUF];   // [buffer][hi, lo]

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, hh = lane >> 5, c32 = lane & 31;
    const int slice = blockIdx.x % (D / 32);
    const int bh = blockIdx.x / (D / 32);
    float *Sg = a.S + (size_t)bh * D * D + 32 * slice + c32;
    const int row0 = 32 * wave + 4 * hh;                 // accumulator register r holds row row0 + 8 (r / 4) + r % 4

    f32x16 s_acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) s_acc[r] = Sg[(size_t)(row0 + 8 * (r >> 2) + (r & 3)) * D];

    const unsigned char *ws = (const unsigned char *)a.workspace + (size_t)bh * nblk * gdn_block_bytes(D);
    bf16x8 ehi[2][KS], elo[2][KS];
    float psi[2][16], gam[2];
    auto fetch = [&](int blk, int buf) {                 // this wavefront's rows of -E, its block of Psi
        const unsigned char *p = ws + (size_t)blk * gdn_block_bytes(D);
        const bf16_t *Ehi = (const bf16_t *)p + (size_t)(32 * wave + c32) * D + 8 * hh;
#pragma unroll
        for (int t = 0; t < KS; ++t) {
            ehi[buf][t] = *(const bf16x8 *)(Ehi + 16 * t);
            elo[buf][t] = *(const bf16x8 *)(Ehi + D * D + 16 * t);
        }
        const float *Psi = (const float *)(p + (size_t)D * D * 4) + 32 * slice + c32;
#pragma unroll
        for (int r = 0; r < 16; ++r) psi[buf][r] = Psi[(size_t)(row0 + 8 * (r >> 2) + (r & 3)) * D];
        gam[buf] = *(const float *)(p + (size_t)D * D * 8);
    };
    auto step = [&](int blk, int buf) {
        if (blk + 1 < nblk) fetch(blk + 1, buf ^ 1);
        // publish this wavefront's 32 rows of the slice as bf16 hi + lo, [column][row]
        unsigned char *sb = smem + (blk & 1) * 2 * SBUF;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            bf16x4 h4, l4;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float x = s_acc[4 * q + i];
                h4[i] = to_bf16(x);
                l4[i] = to_bf16(x - (float)h4[i]);
            }
            const int off = c32 * SROW + 2 * (row0 + 8 * q);
            *(bf16x4 *)(sb + off) = h4;
            *(bf16x4 *)(sb + SBUF + off) = l4;
        }
        __syncthreads();
        f32x16 acc0, acc1, acc2;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            acc0[r] = fmaf(gam[buf], s_acc[r], psi[buf][r]);
            acc1[r] = 0.f;
            acc2[r] = 0.f;
        }
#pragma unroll
        for (int t = 0; t < KS; ++t) {
            const bf16x8 sh = *(const bf16x8 *)(sb + c32 * SROW + 32 * t + 16 * hh);
            const bf16x8 sl = *(const bf16x8 *)(sb + SBUF + c32 * SROW + 32 * t + 16 * hh);
            acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ehi[buf][t], sh, acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ehi[buf][t], sl, acc1, 0, 0, 0);
            acc2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(elo[buf][t], sh, acc2, 0, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) s_acc[r] = acc0[r] + (acc1[r] + acc2[r]);
    };

    fetch(0, 0);
    int blk = 0;
#pragma unroll 1
    for (; blk + 1 < nblk; blk += 2) {
        step(blk, 0);
        step(blk + 1, 1);
    }
    if (blk < nblk) step(blk, 0);

#pragma unroll
    for (int r = 0; r < 16; ++r) Sg[(size_t)(row0 + 8 * (r >> 2) + (r & 3)) * D] = s_acc[r];
}

}  // namespace

size_t gdn_workspace_bytes(int B, int H, int L, int D)
{
    return (size_t)B * H * ((L + CT - 1) / CT) * gdn_block_bytes(D);
}

hipError_t launch_commit_gdn_bf16(const GdnArgs &a, hipStream_t stream)
{
    const int nblk = (a.L + CT - 1) / CT;
    const long long nwg = (long long)a.B * a.H * nblk;
    if (nwg <= 0 || nwg > 0x7fffffffLL) return hipErrorInvalidValue;
    // the block kernel addresses one stream's K (or V) with 32-bit byte offsets
    if ((long long)(a.L + 4 * CT) * a.H * a.D * 2 > 0x7fffffffLL) return hipErrorInvalidValue;
    const unsigned nscan = (unsigned)(a.B * a.H * (a.D / 32));
    if (a.D == 128) {
        hipLaunchKernelGGL(gdn_block_kernel<128>, dim3((unsigned)nwg), dim3(NTA), 0, stream, a, nblk);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(gdn_scan_kernel<128>, dim3(nscan), dim3(256), 0, stream, a, nblk);
    } else if (a.D == 64) {
        hipLaunchKernelGGL(gdn_block_kernel<64>, dim3((unsigned)nwg), dim3(NTA), 0, stream, a, nblk);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(gdn_scan_kernel<64>, dim3(nscan), dim3(128), 0, stream, a, nblk);
    } else {
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace arl2
