// Token-sequential gated delta rule on bf16 MFMA (gfx950):
//   for j = 1..L:  S <- alpha_j S + beta_j k'_j^T (v_j - k'_j S),   k'_j = L2Norm(k_j)
// (paper Eq. (4) applied one token at a time with per-token gates, Sec. 3.2; Alg. 1 clean pass).
//
// Only the state after the last token is wanted: every denoising pass reads the state as it stood
// before the chunk (Sec. 3.3), so no per-token output exists.  That makes each block of 64 tokens a
// single affine map of the state, whose ingredients can be built independently of S:
//
//   inside a block (gamma-_i = alpha_1..alpha_{i-1}, tail_i = alpha_{i+1}..alpha_64, gam = alpha_1..alpha_64)
//     A_ij  = beta_i (alpha_{j+1}..alpha_{i-1}) k'_i.k'_j   for j < i, else 0      (unit lower triangular I + A)
//     Z     = (I + A)^-T diag(tail) K'                       [64 x D]   back substitution
//     S_out = gam S_in + Z^T (diag(beta) V - diag(beta gamma-) K' S_in)
//   (composed: S_out = gam S_in - E S_in + Psi with E = (diag(beta gamma-) Z)^T K', Psi = (diag(beta) Z)^T V)
//
// Kernel 1 (one workgroup per block of tokens, all blocks in parallel) builds Z and leaves it, with K, V^T
// and the per-token scalars, in the workspace in the operand-fragment order of kernel 2.  The Gram matrix
// uses the raw bf16 keys (exact products) and is scaled in fp32; the triangular solve runs in fp32 in
// blocks of 16 tokens, the diagonal systems on the vector ALU (one thread per feature), the off-diagonal
// updates on MFMA with hi + lo splits.  K and V^T leave for the workspace as soon as the tiles are in LDS, Z
// straight from the solver's registers.
// Kernel 2 walks the blocks in order, one workgroup per 64 state columns (eight wavefronts at D = 128, four at
// D = 64), with two dependent contractions per block (K S, then Z^T R).  With few heads the blocks of a head are cut into runs that are walked at
// the same time: the first run on the real state, every later run on the columns of the identity and on
// zero, which yields its composite map (M_g, c_g); kernel 3 applies those D x D maps in order.
// (A first version composed E and Psi per block in kernel 1 and walked on those: twice the workspace
// traffic, which is what bounds the walk.)
// All products of gates are formed by multiplication only, so gates of exactly zero are handled.
#include "arl2_device.h"

#include <type_traits>

namespace arl2 {
namespace {

constexpr int CT = 64;     // tokens per block
constexpr int NTA = 256;   // threads of the block kernel
constexpr int GDN_PFD = 2;    // blocks whose operands the scan keeps in flight
constexpr int GDN_EARLY = 2;  // k-steps of the next operands that the scan requests before its MFMAs start


template <int D>
struct GdnCfg {
    static constexpr int CPR = D / 8;                   // 16-byte chunks per row
    static constexpr int ROW = 2 * D + 32;              // LDS bytes per row of a token-major tile (K, V)
    static constexpr int TILE = CT * ROW;               // one 64-token bf16 tile
    static constexpr int ZROW = 2 * CT + 16;            // LDS bytes per row of a feature-major tile (Z^T)
    static constexpr int KCH = CT * CPR / NTA;          // chunks per thread per tile
    static constexpr int ROWS_PER_PASS = NTA / CPR;
    static constexpr int AST = 68;                      // floats per row of the 64 x 64 fp32 matrix
    static constexpr int NB = D / 32;                   // 32-wide blocks per side of a D x D matrix
    static constexpr int KS = D / 16;                   // k-steps of a D-long contraction
    static constexpr int REG = TILE > CT * AST * 4 ? TILE : CT * AST * 4;   // a region holds a tile or the fp32 matrix
    static constexpr int SC_OFF = 4 * REG;              // per-token scalars behind the four regions
    static constexpr int SMEM = SC_OFF + 8 * CT * 4 + 16;
    static_assert(D * ZROW <= REG, "a feature-major tile must fit into one region");
    static_assert(KCH >= 1, "unsupported head dimension");
};

// Bytes of a composed D x D map record: -E hi, -E lo (bf16, fragment order), Psi (fp32, accumulator order), gam.
__host__ __device__ constexpr size_t gdn_block_bytes(int D) { return (size_t)D * D * 8 + 16; }

// Products over the 64 lanes of a wavefront, by multiplication only (a factor of exactly zero is handled):
// lane l receives x_0 .. x_{l-1} (prefix) or x_{l+1} .. x_63 (suffix); six doubling steps each.
__device__ __forceinline__ float lane_prefix_product(float x, int lane)
{
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const float y = __shfl_up(x, d, 64);
        x *= lane >= d ? y : 1.f;
    }
    const float e = __shfl_up(x, 1, 64);
    return lane == 0 ? 1.f : e;
}
__device__ __forceinline__ float lane_suffix_product(float x, int lane)
{
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const float y = __shfl_down(x, d, 64);
        x *= lane + d < 64 ? y : 1.f;
    }
    const float e = __shfl_down(x, 1, 64);
    return lane == 63 ? 1.f : e;
}

// ---- kernel 1: the affine map of one block of tokens -------------------------------------------------
// Workspace per block of tokens: Z^T hi, Z^T lo (bf16, A fragments: [32-feature block][16-token step][lane]), K (bf16, A fragments:
// [32-token block][k-step][lane]), V^T (bf16, fragments [16-token step][32-column block][lane], tokens in
// k-slot order = accumulator order), then beta_i, -beta_i gamma-_i r_i (fp32 [64] each) and gam.
__host__ __device__ constexpr size_t gdn_ops_bytes(int D) { return (size_t)CT * D * 8 + 1024; }

// Kernel 1: the operands of one block's solve,
//   S_out = gam S + Z^T (diag(beta) V + diag(-beta gamma- r) (K S)),    Z = (I + A)^-T diag(tail r) K.
template <int D>
__global__ __launch_bounds__(NTA, 2) void gdn_block_kernel(GdnArgs a, int nblk)
{
    using C = GdnCfg<D>;
    __shared__ __attribute__((aligned(16))) unsigned char smem[C::SMEM];
    unsigned char *R0 = smem, *R1 = smem + C::REG, *R2 = smem + 2 * C::REG, *R3 = smem + 3 * C::REG;
    float *sc_r = (float *)(smem + C::SC_OFF);          // 1 / sqrt(|k_i|^2 + eps)
    float *sc_al = sc_r + CT, *sc_be = sc_al + CT;      // alpha_i, beta_i
    float *sc_tr = sc_be + CT;                          // (alpha_{i+1} .. alpha_64) r_i
    float *sc_se = sc_tr + CT;                          // -beta_i (alpha_1 .. alpha_{i-1}) r_i
    float *sc_gam = sc_se + CT;

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
            ss = lane_group_sum<C::CPR>(ss);
            if (col == 0) sc_r[row] = fast_rsqrt(ss + a.l2_eps);
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

    // The record of this block in the workspace.  K and V^T depend on the tiles alone: they leave now, in
    // fragment order, and their stores drain while the solve runs.
    unsigned char *rec = (unsigned char *)a.workspace + ((size_t)bh * nblk + blk) * gdn_ops_bytes(D);
    bf16x8 *Zhi = (bf16x8 *)rec, *Zlo = Zhi + CT * D / 8, *Kf = Zlo + CT * D / 8, *Vf = Kf + CT * D / 8;
    float *scal = (float *)(rec + (size_t)CT * D * 8);
    {
        // K: fragment (rbT, t), lane (token c32, hh) = K[32 rbT + c32][16 t + 8 hh + 0..7]
        for (int p = tid; p < 2 * C::KS * 64; p += NTA) {
            const int ln = p & 63, t = (p >> 6) % C::KS, rbT = p / (64 * C::KS);
            Kf[p] = *(const bf16x8 *)(R0 + (32 * rbT + (ln & 31)) * C::ROW + 2 * (16 * t + 8 * (ln >> 5)));
        }
        // V^T: fragment (t, eblk), lane (column c32, hh) = V[16 t + 8 (j / 4) + 4 hh + j % 4][32 eblk + c32].
        // A token-major tile is read through the transposing LDS read: lanes (column c32, hh) get eight tokens of
        // their column, k-slot j <-> token 16 t + 8 (j / 4) + 4 hh + j % 4 (the order of accumulator registers).
        const int tr_off = (((lane & 15) >> 2) + 4 * hh) * C::ROW + 32 * ((lane >> 4) & 1) + 8 * (lane & 3);
        for (int f = wave; f < 4 * C::NB; f += NTA / 64) {
            const int t = f / C::NB, eblk = f % C::NB;
            Vf[f * 64 + lane] = lds_read_tr_pair(R1 + tr_off + 16 * t * C::ROW + 64 * eblk, 8 * C::ROW);
        }
    }

    // ---- 2. products of gates (wavefront 0) and the Gram matrix of the raw keys (three wavefronts)
    if (tid < CT) {
        // alpha_1 .. alpha_{i-1} and alpha_{i+1} .. alpha_64: exclusive prefix and suffix products over the lanes
        const float al = sc_al[tid];
        const float gp = lane_prefix_product(al, lane), tl = lane_suffix_product(al, lane);
        const float r = sc_r[tid], be = sc_be[tid];
        sc_tr[tid] = tl * r;
        sc_se[tid] = -(be * gp * r);
        if (tid == CT - 1) sc_gam[0] = gp * al;
    }
    {
        const int ib = wave >> 1, jb = wave & 1;         // rows i, columns j of the 64 x 64 Gram matrix
        if (jb <= ib) {                                  // the strictly upper block is never used
            f32x16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int t = 0; t < C::KS; ++t) {
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

    // ---- 3. A_ij = beta_i (alpha_{j+1} .. alpha_{i-1}) r_i r_j G_ij for i > j, in place;
    //         thread = (column j, rows 16 wave .. 16 wave + 15)
    {
        float *As = (float *)R2;
        const int j = lane, i0 = 16 * wave;
        float g[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) g[e] = As[(i0 + e) * C::AST + j];
        // alpha_{j+1} .. alpha_{i0-1}: exclusive suffix product over the lanes of the gates before row i0
        float rho = lane_suffix_product(j < i0 ? sc_al[j] : 1.f, lane);
        const float rj = sc_r[j];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const f32x4 al4 = *(const f32x4 *)(sc_al + i0 + 4 * q);
            const f32x4 be4 = *(const f32x4 *)(sc_be + i0 + 4 * q);
            const f32x4 r4 = *(const f32x4 *)(sc_r + i0 + 4 * q);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int i = i0 + 4 * q + e;
                if (i > j) {
                    As[i * C::AST + j] = be4[e] * rho * r4[e] * rj * g[4 * q + e];
                    rho *= al4[e];
                }
            }
        }
    }
    __syncthreads();

    // ---- 4. back substitution (I + A)^T Z = diag(tail r) K in blocks of 16 tokens, last block first.
    // The 16 x 16 diagonal systems are solved on the vector ALU, thread = feature (row i of A updates
    // rows j < i, all independent).  What a solved block contributes to the rows before it,
    // U[j][f] = sum_{i in block} A_ij Z_i[f], is one MFMA k-step: A from the fp32 matrix in LDS and the
    // block of Z passed through LDS, both split into bf16 hi + lo (three terms); U stays in accumulators
    // (wavefront = 32 features, rows 0..63 as two 32-row blocks) and only the 16 rows the next block
    // needs travel back through LDS.
    float z[CT];
    {
        const float *As = (const float *)R2;
        unsigned char *Zb = R3;                                   // [feature][16 tokens] bf16, hi then lo
        float *Ux = (float *)(R3 + 2 * D * 32);                   // [16 rows][D + 4] fp32
        constexpr int UST = D + 4;
        if (tid < D) {
#pragma unroll
            for (int i = 0; i < CT; ++i) z[i] = sc_tr[i] * (float)*(const bf16_t *)(R0 + i * C::ROW + 2 * tid);
        }
        f32x16 U[2];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r) U[rb][r] = 0.f;
        static_for<0, 4>([&](auto bb_) {
            constexpr int b4 = 3 - decltype(bb_)::value, i0 = 16 * b4;          // token block 3, 2, 1, 0
            if (tid < D) {
                // the block's 120 entries of A first, so that their LDS latency is paid once
                f32x4 a4[15][4];
                static_for<1, 16>([&](auto il_) {
                    constexpr int il = decltype(il_)::value;
                    static_for<0, (il + 3) / 4>([&](auto q_) {
                        constexpr int q = decltype(q_)::value;
                        a4[il - 1][q] = *(const f32x4 *)(As + (i0 + il) * C::AST + i0 + 4 * q);
                    });
                });
                if constexpr (b4 < 3) {
#pragma unroll
                    for (int e = 0; e < 16; ++e) z[i0 + e] -= Ux[e * UST + tid];
                }
                static_for<0, 15>([&](auto ii_) {
                    constexpr int il = 15 - decltype(ii_)::value;                  // z[i0 + il] is final
                    static_for<0, il>([&](auto jl_) {
                        constexpr int jl = decltype(jl_)::value;
                        z[i0 + jl] = fmaf(-a4[il - 1][jl / 4][jl % 4], z[i0 + il], z[i0 + jl]);
                    });
                });
                if constexpr (b4 > 0) {
#pragma unroll
                    for (int half = 0; half < 2; ++half) {
                        bf16x8 h8, l8;
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const float x = z[i0 + 8 * half + e];
                            h8[e] = to_bf16(x);
                            l8[e] = to_bf16(x - (float)h8[e]);
                        }
                        *(bf16x8 *)(Zb + tid * 32 + 16 * half) = h8;
                        *(bf16x8 *)(Zb + D * 32 + tid * 32 + 16 * half) = l8;
                    }
                }
            }
            if constexpr (b4 > 0) {
                __syncthreads();
                if (wave < C::NB) {
                    const bf16x8 zh = *(const bf16x8 *)(Zb + (32 * wave + c32) * 32 + 16 * hh);
                    const bf16x8 zl = *(const bf16x8 *)(Zb + D * 32 + (32 * wave + c32) * 32 + 16 * hh);
                    constexpr int NRB = (i0 + 31) / 32;                                 // 32-row blocks that hold rows < i0
                    static_for<0, NRB>([&](auto rb_) {
                        constexpr int rb = decltype(rb_)::value;
                        const int j = 32 * rb + c32;
                        bf16x8 ah, al;
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const float x = j < i0 ? As[(i0 + 8 * hh + e) * C::AST + j] : 0.f;
                            ah[e] = to_bf16(x);
                            al[e] = to_bf16(x - (float)ah[e]);
                        }
                        U[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, zh, U[rb], 0, 0, 0);
                        U[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, zl, U[rb], 0, 0, 0);
                        U[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, zh, U[rb], 0, 0, 0);
                    });
                    // rows i0 - 16 .. i0 - 1 of U go to the feature threads
                    constexpr int rb = (i0 - 16) / 32, r0 = ((i0 - 16) % 32) / 8 * 4;  // 32-row block, first register
#pragma unroll
                    for (int r = 0; r < 8; ++r)
                        Ux[(8 * (r >> 2) + 4 * hh + (r & 3)) * UST + 32 * wave + c32] = U[rb][r0 + r];
                }
                __syncthreads();
            }
        });
    }
    // Z^T leaves straight from the registers of the feature threads, split into bf16 hi + lo:
    // fragment (rb, t), lane (feature c32, hh) = Z^T[32 rb + c32][16 t + 8 hh + 0..7]; consecutive threads
    // (features) write consecutive 16-byte pieces
    if (tid < D) {
        const int rb = tid >> 5, f32 = tid & 31;
#pragma unroll
        for (int q = 0; q < CT / 8; ++q) {               // q = 2 t + hh
            bf16x8 h8, l8;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float x = z[8 * q + e];
                h8[e] = to_bf16(x);
                l8[e] = to_bf16(x - (float)h8[e]);
            }
            const int p = (rb * 4 + (q >> 1)) * 64 + f32 + 32 * (q & 1);
            Zhi[p] = h8;
            Zlo[p] = l8;
        }
    }
    if (tid < CT) {
        scal[tid] = sc_be[tid];
        scal[CT + tid] = sc_se[tid];
    }
    if (tid == 0) scal[2 * CT] = sc_gam[0];
}

// ---- kernel 3: composed maps applied in order, S <- gam S + Psi + (-E) S ---------------------------------
// One workgroup per (stream, head, 32 state columns) applies the `count` records stored at `maps` (per
// head `count` records) to the state in a.S.  A record holds -E as bf16 hi + lo A fragments (k-slot j of
// half-wave hh <-> column 16 t + 8 (j / 4) + 4 hh + j % 4), Psi in accumulator order and gam: the composite
// maps that the walk below leaves for its runs of blocks.
// Workspace per composed map: -E hi, -E lo (bf16, fragment order), Psi (fp32, accumulator order), gam.
template <int D>
__global__ __launch_bounds__(2 * D) void gdn_apply_kernel(GdnArgs a, const unsigned char *maps, int count)
{
    constexpr int KS = D / 16;                           // k-steps of the D-long contraction
    constexpr int NSL = D / 32;                          // 32-column slices of the state
    constexpr int SROW = 2 * D + 16;                     // LDS bytes per state column (conflict-free b128 reads)
    constexpr int SBUF = 32 * SROW;                      // one bf16 part of the 32-column slice, stored [column][row slot]
    constexpr int PFD = GDN_PFD, NBUF = PFD + 1;
    constexpr int EARLY = GDN_EARLY;                             // k-steps whose loads are issued before the MFMAs start
    __shared__ __attribute__((aligned(16))) unsigned char smem[4 * SBUF];   // [buffer][hi, lo]

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, hh = lane >> 5, c32 = lane & 31;
    // The column slices of a head read the same -E: they run on one XCD (consecutive workgroup ids go
    // round the 8 XCDs), so that its L2 serves the re-reads.  The grid is padded to whole heads per XCD.
    const int heads = a.B * a.H;
    const int xcd = blockIdx.x % kNumXcd, loc = blockIdx.x / kNumXcd;
    const int slice = loc % NSL;
    const int bh = (loc / NSL) * kNumXcd + xcd;
    const int n = count;
    if (bh >= heads || n <= 0) return;
    float *Sg = a.S + (size_t)bh * D * D + 32 * slice + c32;
    const int row0 = 32 * wave + 4 * hh;                 // accumulator register r holds row row0 + 8 (r / 4) + r % 4

    f32x16 s_acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) s_acc[r] = Sg[(size_t)(row0 + 8 * (r >> 2) + (r & 3)) * D];

    const unsigned char *ws = maps + (size_t)bh * count * gdn_block_bytes(D);
    // operands of the next PFD blocks are kept in flight (registers), a ring of NBUF = PFD + 1 buffers
    bf16x8 ehi[NBUF][KS], elo[NBUF][KS];
    f32x4 psi[NBUF][4];
    float gam[NBUF];
    // Loads of one block's operands, in KS + 1 parts so that they can be issued between the MFMAs of a
    // step: the workgroup's loads of a step (80 KB at D = 128) keep the CU's 64-byte-per-clock load path
    // busy about as long as the step's MFMAs take.
    auto fetch_part = [&](int blk, auto buf_, auto part_) {
        constexpr int buf = decltype(buf_)::value, part = decltype(part_)::value;
        const unsigned char *p = ws + (size_t)blk * gdn_block_bytes(D);
        if constexpr (part < KS) {                       // this wavefront's rows of -E, fragment order [row block][k-step][lane]
            const bf16x8 *Ehi = (const bf16x8 *)p + wave * KS * 64 + lane;
            ehi[buf][part] = Ehi[part * 64];
            elo[buf][part] = Ehi[D * D / 8 + part * 64];
        } else {                                         // its block of Psi, accumulator order
            const f32x4 *Psi = (const f32x4 *)(p + (size_t)D * D * 4) + (wave * NSL + slice) * 4 * 64 + lane;
#pragma unroll
            for (int q = 0; q < 4; ++q) psi[buf][q] = Psi[q * 64];
            gam[buf] = *(const float *)(p + (size_t)D * D * 8);
        }
    };
    auto fetch = [&](int blk, auto buf_) {
        static_for<0, KS + 1>([&](auto part_) { fetch_part(blk, buf_, part_); });
    };
    // The slice is published [column][slot] with the rows of each 16-row group in k-slot order: slot
    // 8 hh + j holds row 16 t + 8 (j / 4) + 4 hh + j % 4, so that one 16-byte read is a B operand that
    // matches the stored A fragments of -E.  This lane's register quads 2 p, 2 p + 1 are slots 0..7 of
    // its half of group 2 wave + p.
    const int st_w = c32 * SROW + 2 * (32 * wave + 8 * hh);
    const int st_r = c32 * SROW + 16 * hh;
    auto step = [&](int blk, auto buf_) {
        constexpr int buf = decltype(buf_)::value;
        // past the last block this re-reads the last one (unused), which keeps the loop free of branches
        const int nxt = blk + PFD < n ? blk + PFD : n - 1;
        const std::integral_constant<int, (buf + PFD) % NBUF> nbuf{};
        fetch_part(nxt, nbuf, std::integral_constant<int, KS>{});
        static_for<0, EARLY>([&](auto part_) { fetch_part(nxt, nbuf, part_); });
        unsigned char *sb = smem + (blk & 1) * 2 * SBUF;
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            bf16x8 h8, l8;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float x = s_acc[8 * p + e];
                h8[e] = to_bf16(x);
                l8[e] = to_bf16(x - (float)h8[e]);
            }
            *(bf16x8 *)(sb + st_w + 32 * p) = h8;
            *(bf16x8 *)(sb + SBUF + st_w + 32 * p) = l8;
        }
        __syncthreads();
        f32x16 acc0 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}, acc1 = acc0, acc2 = acc0;
        static_for<0, KS>([&](auto t_) {
            constexpr int t = decltype(t_)::value;
            const bf16x8 sh = *(const bf16x8 *)(sb + st_r + 32 * t);
            const bf16x8 sl = *(const bf16x8 *)(sb + SBUF + st_r + 32 * t);
            acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ehi[buf][t], sh, acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ehi[buf][t], sl, acc1, 0, 0, 0);
            acc2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(elo[buf][t], sh, acc2, 0, 0, 0);
            if constexpr (t + EARLY < KS) fetch_part(nxt, nbuf, std::integral_constant<int, t + EARLY>{});
            __builtin_amdgcn_sched_barrier(0);
        });
#pragma unroll
        for (int r = 0; r < 16; ++r)
            s_acc[r] = (fmaf(gam[buf], s_acc[r], psi[buf][r >> 2][r & 3]) + acc0[r]) + (acc1[r] + acc2[r]);
    };

    static_for<0, PFD>([&](auto i_) { fetch(decltype(i_)::value < n ? decltype(i_)::value : n - 1, i_); });
    int blk = 0;
#pragma unroll 1
    for (; blk + NBUF <= n; blk += NBUF)
        static_for<0, NBUF>([&](auto i_) { step(blk + decltype(i_)::value, i_); });
    static_for<0, NBUF - 1>([&](auto i_) {
        if (blk + decltype(i_)::value < n) step(blk + decltype(i_)::value, i_);
    });

#pragma unroll
    for (int r = 0; r < 16; ++r) Sg[(size_t)(row0 + 8 * (r >> 2) + (r & 3)) * D] = s_acc[r];
}

// ---- kernel 2: the walk on the operands of the solve ---------------------------------------------------
// One workgroup (four wavefronts) per 64 state columns; per block of tokens
//   T = K S            [64 tokens x 64 columns], K raw bf16 against S hi + lo
//   R = beta (.) V + (-beta gamma- r) (.) T      (fp32, then hi + lo)
//   S <- gam S + Z^T R [D x 64], Z^T hi/lo against R hi/lo (three terms)
// Wavefront w computes T and R for token block w & 1 and column block w >> 1, and updates the state rows
// D/2 (w & 1) .. + D/2 of column block w >> 1.  S and R pass between the wavefronts through LDS ([column]
// [row] and [column][token], 16-byte reads are B operands).
//   GROUPED == false: one run, the whole chunk, on the state in a.S.
//   GROUPED == true: the blocks of a head are cut into `groups` runs of consecutive blocks that are walked
//     at the same time.  Run 0 starts from the state in a.S and leaves X_0 there.  Every later run g
//     applies the walk to the columns of the identity (giving M_g = prod (gam_n I - E_n)) and to zero
//     (giving c_g) and stores them as a composed-map record, -E := M_g - gam_g I with gam_g = prod gam_n
//     (the multiple of the identity stays an exact fp32 scalar), Psi := c_g; kernel 3 then applies the
//     groups - 1 records to X_0.  The chain shrinks from nblk steps to nblk / groups + groups - 1.
//   The workgroups of a (head, run) pair read the same records: they run on one XCD (workgroup ids go round
//   the 8 XCDs), the later runs first in the grid, the first runs after them, each kind dealt round the
//   XCDs on its own so that every XCD gets the same number of busy workgroups.
template <int D, bool GROUPED>
__global__ __launch_bounds__(256) void gdn_walk_kernel(GdnArgs a, const unsigned char *recs, int nblk, int groups, unsigned char *gmaps)
{
    constexpr int KS = D / 16, NB = D / 32, NSL = D / 64, NRB = D / 64;   // k-steps, 32-blocks, 64-column slices, row blocks per wavefront
    constexpr int SROW = 2 * D + 16, RROW = 2 * CT + 16;
    constexpr int S_BYTES = 64 * SROW, R_BYTES = 64 * RROW;
    constexpr int TROW = 2 * 64 + 16;                    // row of the [D][64] bf16 tile that transposes M_g
    static_assert(2 * D * TROW <= 2 * S_BYTES + 2 * R_BYTES, "the transposing tiles reuse the exchange buffers");
    __shared__ __attribute__((aligned(16))) unsigned char smem[2 * S_BYTES + 2 * R_BYTES];
    unsigned char *Shi = smem, *Slo = smem + S_BYTES, *Rhi = smem + 2 * S_BYTES, *Rlo = Rhi + R_BYTES;

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, hh = lane >> 5, c32 = lane & 31;
    const int rbT = wave & 1, cb = wave >> 1, rbF0 = NRB * (wave & 1);
    const int heads = a.B * a.H;
    const int n_late = GROUPED ? (heads * (groups - 1) + kNumXcd - 1) / kNumXcd * kNumXcd * 2 * NSL : 0;
    const bool late = (int)blockIdx.x < n_late;
    const int id = late ? blockIdx.x : blockIdx.x - n_late;
    const int xcd = id % kNumXcd, loc = id / kNumXcd;
    const int units = late ? 2 * NSL : NSL;
    const int unit = loc % units;
    const int owner = (loc / units) * kNumXcd + xcd;
    const int slice = unit % NSL;
    const bool is_m = unit >= NSL;
    int bh = owner, grp = 0, first = 0, n = nblk;
    if constexpr (GROUPED) {
        if (late) {
            bh = owner / (groups - 1);
            grp = 1 + owner % (groups - 1);
        }
        first = (int)((long long)grp * nblk / groups);
        n = (int)((long long)(grp + 1) * nblk / groups) - first;
    }
    if (bh >= heads || n <= 0) return;
    const int col = 32 * cb + c32, gcol = 64 * slice + col;          // column within the slice / within the state
    float *Sg = a.S + (size_t)bh * D * D + gcol;

    f32x16 s_acc[NRB];
#pragma unroll
    for (int i = 0; i < NRB; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = 32 * (rbF0 + i) + 8 * (r >> 2) + 4 * hh + (r & 3);
            if (!GROUPED || grp == 0) s_acc[i][r] = Sg[(size_t)row * D];
            else s_acc[i][r] = (is_m && row == gcol) ? 1.0f : 0.0f;
        }
    const float v_on = is_m ? 0.0f : 1.0f;               // the identity's columns take no V term
    float gprod = 1.0f;

    const unsigned char *ws = recs + ((size_t)bh * nblk + first) * gdn_ops_bytes(D);
    // Two register sets per operand.  A set is refilled with the operands of the block after next as soon
    // as it has been consumed (K after the first contraction, V^T and the per-token scalars after R, Z^T
    // after the second contraction), so every load has almost two steps to arrive: the records are read
    // once and come from HBM or the memory-side cache, about a step away.
    bf16x8 kf[2][KS], zh[2][NRB][4], zl[2][NRB][4], vf[2][2];
    f32x4 be[2][4], se[2][4];
    float gam[2];
    auto rec_of = [&](int blk) { return ws + (size_t)(blk < n ? blk : n - 1) * gdn_ops_bytes(D); };   // past the end: the last one again (unused)
    auto fetch_k = [&](int blk, auto b_) __attribute__((always_inline)) {
        constexpr int bi = decltype(b_)::value;
        const bf16x8 *Kf = (const bf16x8 *)rec_of(blk) + 2 * (CT * D / 8);
        static_for<0, KS>([&](auto t_) { kf[bi][decltype(t_)::value] = Kf[(rbT * KS + decltype(t_)::value) * 64 + lane]; });
    };
    auto fetch_v = [&](int blk, auto b_) __attribute__((always_inline)) {
        constexpr int bi = decltype(b_)::value;
        const unsigned char *p = rec_of(blk);
        const bf16x8 *Vf = (const bf16x8 *)p + 3 * (CT * D / 8);
        const float *scal = (const float *)(p + (size_t)CT * D * 8);
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) vf[bi][tt] = Vf[((2 * rbT + tt) * NB + 2 * slice + cb) * 64 + lane];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            be[bi][q] = *(const f32x4 *)(scal + 32 * rbT + 8 * q + 4 * hh);
            se[bi][q] = *(const f32x4 *)(scal + CT + 32 * rbT + 8 * q + 4 * hh);
        }
        gam[bi] = scal[2 * CT];
    };
    auto fetch_z = [&](int blk, auto b_) __attribute__((always_inline)) {
        constexpr int bi = decltype(b_)::value;
        const bf16x8 *Zhi = (const bf16x8 *)rec_of(blk), *Zlo = Zhi + CT * D / 8;
        static_for<0, NRB>([&](auto i_) {
            constexpr int i = decltype(i_)::value;
            static_for<0, 4>([&](auto t_) {
                constexpr int t = decltype(t_)::value;
                zh[bi][i][t] = Zhi[((rbF0 + i) * 4 + t) * 64 + lane];
                zl[bi][i][t] = Zlo[((rbF0 + i) * 4 + t) * 64 + lane];
            });
        });
    };
    auto step = [&](int blk, auto b_) __attribute__((always_inline)) {
        constexpr int bi = decltype(b_)::value;
        const float gam_cur = gam[bi];
        // ---- the state slice to LDS, [column][row], hi and lo
        static_for<0, NRB>([&](auto i_) {
            constexpr int i = decltype(i_)::value;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                bf16x4 h4, l4;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float x = s_acc[i][4 * q + e];
                    h4[e] = to_bf16(x);
                    l4[e] = to_bf16(x - (float)h4[e]);
                }
                const int off = col * SROW + 2 * (32 * (rbF0 + i) + 8 * q + 4 * hh);
                *(bf16x4 *)(Shi + off) = h4;
                *(bf16x4 *)(Slo + off) = l4;
            }
        });
        lds_barrier();                                   // (not __syncthreads: the operand loads stay in flight)
        // ---- T = K S for this wavefront's 32 tokens x 32 columns
        // (independent accumulator chains: a dependent MFMA waits ~50 cycles for its predecessor, an
        // independent one issues after 32)
        f32x16 t_h = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}, t_l = t_h;
        static_for<0, KS>([&](auto t_) {
            constexpr int t = decltype(t_)::value;
            const bf16x8 sh = *(const bf16x8 *)(Shi + col * SROW + 32 * t + 16 * hh);
            const bf16x8 sl = *(const bf16x8 *)(Slo + col * SROW + 32 * t + 16 * hh);
            t_h = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[bi][t], sh, t_h, 0, 0, 0);
            t_l = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[bi][t], sl, t_l, 0, 0, 0);
        });
        fetch_k(blk + 2, b_);
        // ---- R = beta V + (-beta gamma- r) T, register r <-> token 32 rbT + 8 (r / 4) + 4 hh + r % 4
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            bf16x4 h4, l4;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int r = 4 * q + e;
                const float v = (float)vf[bi][r >> 3][r & 7];
                const float x = fmaf(se[bi][q][e], t_h[r] + t_l[r], GROUPED ? v_on * be[bi][q][e] * v : be[bi][q][e] * v);
                h4[e] = to_bf16(x);
                l4[e] = to_bf16(x - (float)h4[e]);
            }
            const int off = col * RROW + 2 * (32 * rbT + 8 * q + 4 * hh);
            *(bf16x4 *)(Rhi + off) = h4;
            *(bf16x4 *)(Rlo + off) = l4;
        }
        fetch_v(blk + 2, b_);
        lds_barrier();
        // ---- S <- gam S + Z^T R
        bf16x8 rh[4], rl[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            rh[t] = *(const bf16x8 *)(Rhi + col * RROW + 32 * t + 16 * hh);
            rl[t] = *(const bf16x8 *)(Rlo + col * RROW + 32 * t + 16 * hh);
        }
        f32x16 acc[NRB][2];                              // [0] hi x hi, [1] the two cross terms
        static_for<0, NRB>([&](auto i_) {
            static_for<0, 2>([&](auto j_) {
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[decltype(i_)::value][decltype(j_)::value][r] = 0.f;
            });
        });
        static_for<0, 4>([&](auto t_) {
            constexpr int t = decltype(t_)::value;
            static_for<0, NRB>([&](auto i_) {
                constexpr int i = decltype(i_)::value;
                acc[i][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(zh[bi][i][t], rh[t], acc[i][0], 0, 0, 0);
                acc[i][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(zh[bi][i][t], rl[t], acc[i][1], 0, 0, 0);
                acc[i][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(zl[bi][i][t], rh[t], acc[i][1], 0, 0, 0);
            });
        });
        fetch_z(blk + 2, b_);
        static_for<0, NRB>([&](auto i_) {
            constexpr int i = decltype(i_)::value;
#pragma unroll
            for (int r = 0; r < 16; ++r) s_acc[i][r] = fmaf(gam_cur, s_acc[i][r], acc[i][0][r]) + acc[i][1][r];
        });
        if constexpr (GROUPED) gprod *= gam_cur;
    };

    const std::integral_constant<int, 0> B0{};
    const std::integral_constant<int, 1> B1{};
    fetch_k(0, B0); fetch_v(0, B0); fetch_z(0, B0);
    fetch_k(1, B1); fetch_v(1, B1); fetch_z(1, B1);
    int blk = 0;
#pragma unroll 1
    for (; blk + 2 <= n; blk += 2) {
        step(blk, B0);
        step(blk + 1, B1);
    }
    if (blk < n) step(blk, B0);

    if (!GROUPED || grp == 0) {
#pragma unroll
        for (int i = 0; i < NRB; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) Sg[(size_t)(32 * (rbF0 + i) + 8 * (r >> 2) + 4 * hh + (r & 3)) * D] = s_acc[i][r];
        return;
    }
    if constexpr (GROUPED) {
        // the composite map of run grp >= 1 as one record of the composed-map format
        unsigned char *rec = gmaps + ((size_t)bh * (groups - 1) + grp - 1) * gdn_block_bytes(D);
        if (!is_m) {                                     // c_g, accumulator order [row block][column block][quad][lane]
#pragma unroll
            for (int i = 0; i < NRB; ++i) {
                f32x4 *Psi = (f32x4 *)(rec + (size_t)D * D * 4) + ((rbF0 + i) * NB + 2 * slice + cb) * 4 * 64 + lane;
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    Psi[q * 64] = f32x4{s_acc[i][4 * q], s_acc[i][4 * q + 1], s_acc[i][4 * q + 2], s_acc[i][4 * q + 3]};
            }
            if (slice == 0 && tid == 0) *(float *)(rec + (size_t)D * D * 8) = gprod;
            return;
        }
        // M_g - gam_g I, columns 64 slice .. + 63: through LDS into A-fragment order (lane = row, eight
        // columns of k-steps 4 slice .. 4 slice + 3 in k-slot order), hi and lo parts
        __syncthreads();                                 // the exchange buffers are no longer read
        unsigned char *Thi = smem, *Tlo = smem + D * TROW;
#pragma unroll
        for (int i = 0; i < NRB; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = 32 * (rbF0 + i) + 8 * (r >> 2) + 4 * hh + (r & 3);
                const float x = s_acc[i][r] - (row == gcol ? gprod : 0.0f);
                const bf16_t h = to_bf16(x);
                *(bf16_t *)(Thi + row * TROW + 2 * col) = h;
                *(bf16_t *)(Tlo + row * TROW + 2 * col) = to_bf16(x - (float)h);
            }
        __syncthreads();
        bf16x8 *Ehi = (bf16x8 *)rec, *Elo = Ehi + D * D / 8;
#pragma unroll
        for (int i = 0; i < NB; ++i) {                   // NB * 4 * 64 fragment pieces, 256 threads
            const int p = tid + 256 * i;
            const int ln = p & 63, tl = (p >> 6) & 3, rb = p >> 8;
            const int off = (32 * rb + (ln & 31)) * TROW + 2 * (16 * tl + 4 * (ln >> 5));
            const bf16x4 h0 = *(const bf16x4 *)(Thi + off), h1 = *(const bf16x4 *)(Thi + off + 16);
            const bf16x4 l0 = *(const bf16x4 *)(Tlo + off), l1 = *(const bf16x4 *)(Tlo + off + 16);
            const int idx = (rb * KS + 4 * slice + tl) * 64 + ln;
            Ehi[idx] = __builtin_shufflevector(h0, h1, 0, 1, 2, 3, 4, 5, 6, 7);
            Elo[idx] = __builtin_shufflevector(l0, l1, 0, 1, 2, 3, 4, 5, 6, 7);
        }
    }
}


// ---- kernel 2, D = 128: the same walk with eight wavefronts per 64 state columns ------------------------------
// A step of the walk is a chain (split S, contract, form R, contract, update S) that a single wavefront per
// SIMD runs at the sum of its matrix-core and vector-ALU times.  Here two wavefronts share each SIMD and each
// carries half of a step's work, so a SIMD issues the vector-ALU parts at twice the rate and every chain link
// is half as long:
//   * state: wavefront w owns rows 32 rbF .. + 31 (rbF = w % 2 + 2 (w / 4)) of column block cb = w / 2 % 2;
//   * T = K S: the 32 x 32 block (token block rbT = w % 2, column block cb) belongs to the pair (w, w + 4);
//     member m = w / 4 takes tokens 16 m .. 16 m + 15 of it, as 16 x 16 x 32 MFMAs over two column halves (K raw
//     against S hi and S lo, one accumulator per half; the K operand is gathered from the record's 32 x 32 x 16
//     fragments, 16 bytes per lane), and forms R for those tokens;
//   * S <- gam S + Z^T R for its own 32 rows: Z^T hi/lo against R hi/lo, three terms.
// Two LDS-only barriers per step (S published, R published).  K and Z^T fragments have two register sets
// (refilled two steps ahead), V^T and the per-token scalars one (refilled one step ahead).
// Run decoding, identity columns and the composite-map record are those of the four-wavefront kernel above.
template <bool GROUPED>
__global__ __launch_bounds__(512) void gdn_walk8_kernel(GdnArgs a, const unsigned char *recs, int nblk, int groups, unsigned char *gmaps)
{
    constexpr int D = 128;
    constexpr int KS = D / 16, NB = D / 32, NSL = D / 64;
    constexpr int SROW = 2 * D + 16, RROW = 2 * CT + 16;
    constexpr int S_BYTES = 64 * SROW, R_BYTES = 64 * RROW;
    constexpr int TROW = 2 * 64 + 16;                    // row of the [D][64] bf16 tile that transposes M_g
    static_assert(2 * D * TROW <= 2 * S_BYTES + 2 * R_BYTES, "the transposing tiles reuse the exchange buffers");
    __shared__ __attribute__((aligned(16))) unsigned char smem[2 * S_BYTES + 2 * R_BYTES];
    unsigned char *Shi = smem, *Slo = smem + S_BYTES, *Rhi = smem + 2 * S_BYTES, *Rlo = Rhi + R_BYTES;

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, hh = lane >> 5, c32 = lane & 31;
    const int rbT = wave & 1, cb = (wave >> 1) & 1, m = wave >> 2, rbF = (wave & 1) + 2 * m;
    const int c16 = lane & 15, g = lane >> 4;            // operand coordinates of the 16 x 16 x 32 MFMA
    const int heads = a.B * a.H;
    const int n_late = GROUPED ? (heads * (groups - 1) + kNumXcd - 1) / kNumXcd * kNumXcd * 2 * NSL : 0;
    const bool late = (int)blockIdx.x < n_late;
    const int id = late ? blockIdx.x : blockIdx.x - n_late;
    const int xcd = id % kNumXcd, loc = id / kNumXcd;
    const int units = late ? 2 * NSL : NSL;
    const int unit = loc % units;
    const int owner = (loc / units) * kNumXcd + xcd;
    const int slice = unit % NSL;
    const bool is_m = unit >= NSL;
    int bh = owner, grp = 0, first = 0, n = nblk;
    if constexpr (GROUPED) {
        if (late) {
            bh = owner / (groups - 1);
            grp = 1 + owner % (groups - 1);
        }
        first = (int)((long long)grp * nblk / groups);
        n = (int)((long long)(grp + 1) * nblk / groups) - first;
    }
    if (bh >= heads || n <= 0) return;
    const int col = 32 * cb + c32, gcol = 64 * slice + col;          // column within the slice / within the state
    float *Sg = a.S + (size_t)bh * D * D + gcol;

    f32x16 s_acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int row = 32 * rbF + 8 * (r >> 2) + 4 * hh + (r & 3);
        if (!GROUPED || grp == 0) s_acc[r] = Sg[(size_t)row * D];
        else s_acc[r] = (is_m && row == gcol) ? 1.0f : 0.0f;
    }
    const float v_on = is_m ? 0.0f : 1.0f;               // the identity's columns take no V term
    float gprod = 1.0f;

    const unsigned char *ws = recs + ((size_t)bh * nblk + first) * gdn_ops_bytes(D);
    bf16x8 kf[2][4], zh[2][4], zl[2][4];
    bf16x4 vf[2];
    f32x4 be, se;
    float gam[2];
    auto rec_of = [&](int blk) { return ws + (size_t)(blk < n ? blk : n - 1) * gdn_ops_bytes(D); };   // past the end: the last one again (unused)
    auto fetch_k = [&](int blk, auto b_) __attribute__((always_inline)) {
        constexpr int bi = decltype(b_)::value;
        const bf16x8 *Kf = (const bf16x8 *)rec_of(blk) + 2 * (CT * D / 8);
        // A operand of feature step s (32 features): lane (token 16 m + c16, g) holds K[..][32 s + 8 g + 0..7], which
        // the record keeps in its 32 x 32 x 16 fragment (rbT, 2 s + g / 2) at lane 16 m + c16 + 32 (g % 2)
        static_for<0, 4>([&](auto s_) {
            constexpr int sx = decltype(s_)::value;
            kf[bi][sx] = Kf[(rbT * KS + 2 * sx + (g >> 1)) * 64 + 16 * m + c16 + 32 * (g & 1)];
        });
    };
    auto fetch_v = [&](int blk) __attribute__((always_inline)) {     // V^T of this member's 16 tokens, their scalars
        const unsigned char *p = rec_of(blk);
        const bf16x8 *Vf = (const bf16x8 *)p + 3 * (CT * D / 8);
        const float *scal = (const float *)(p + (size_t)CT * D * 8);
        // tokens 4 g + 0..3 of the 16-token step 2 rbT + m, columns 16 ch + c16 of the block: k-slots 4 (g / 2) + 0..3
        // of lane 16 ch + c16 + 32 (g % 2) in the record's V^T fragment
        const bf16x4 *V4 = (const bf16x4 *)(Vf + ((2 * rbT + m) * NB + 2 * slice + cb) * 64);
#pragma unroll
        for (int ch = 0; ch < 2; ++ch) vf[ch] = V4[2 * (16 * ch + c16 + 32 * (g & 1)) + (g >> 1)];
        be = *(const f32x4 *)(scal + 32 * rbT + 16 * m + 4 * g);
        se = *(const f32x4 *)(scal + CT + 32 * rbT + 16 * m + 4 * g);
    };
    auto fetch_z = [&](int blk, auto b_) __attribute__((always_inline)) {
        constexpr int bi = decltype(b_)::value;
        const unsigned char *p = rec_of(blk);
        const bf16x8 *Zhi = (const bf16x8 *)p, *Zlo = Zhi + CT * D / 8;
        static_for<0, 4>([&](auto t_) {
            constexpr int t = decltype(t_)::value;
            zh[bi][t] = Zhi[(rbF * 4 + t) * 64 + lane];
            zl[bi][t] = Zlo[(rbF * 4 + t) * 64 + lane];
        });
        gam[bi] = *(const float *)(p + (size_t)CT * D * 8 + 2 * CT * 4);
    };
    auto step = [&](int blk, auto b_) __attribute__((always_inline)) {
        constexpr int bi = decltype(b_)::value;
        const float gam_cur = gam[bi];
        // ---- this wavefront's 32 rows of the state slice to LDS, [column][row], hi and lo
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            bf16x4 h4, l4;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float x = s_acc[4 * q + e];
                h4[e] = to_bf16(x);
                l4[e] = to_bf16(x - (float)h4[e]);
            }
            const int off = col * SROW + 2 * (32 * rbF + 8 * q + 4 * hh);
            *(bf16x4 *)(Shi + off) = h4;
            *(bf16x4 *)(Slo + off) = l4;
        }
        lds_barrier();                                   // (not __syncthreads: the operand loads stay in flight)
        // ---- T = K S for this member's 16 tokens x 32 columns, all 128 features: 16 x 16 x 32 MFMAs, two column
        // halves; lane (column c16, g) ends up with tokens 4 g + 0..3 of both halves
        f32x4 tq[2] = {{0, 0, 0, 0}, {0, 0, 0, 0}};
        static_for<0, 4>([&](auto s_) {
            constexpr int sx = decltype(s_)::value;
#pragma unroll
            for (int ch = 0; ch < 2; ++ch) {
                const int o = (32 * cb + 16 * ch + c16) * SROW + 64 * sx + 16 * g;
                tq[ch] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[bi][sx], *(const bf16x8 *)(Shi + o), tq[ch], 0, 0, 0);
                tq[ch] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[bi][sx], *(const bf16x8 *)(Slo + o), tq[ch], 0, 0, 0);
            }
        });
        fetch_k(blk + 2, b_);
        // ---- R = beta V + (-beta gamma- r) T for tokens 32 rbT + 16 m + 4 g + e
#pragma unroll
        for (int ch = 0; ch < 2; ++ch) {
            bf16x4 h4, l4;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float v = (float)vf[ch][e];
                const float x = fmaf(se[e], tq[ch][e], GROUPED ? v_on * be[e] * v : be[e] * v);
                h4[e] = to_bf16(x);
                l4[e] = to_bf16(x - (float)h4[e]);
            }
            const int off = (32 * cb + 16 * ch + c16) * RROW + 2 * (32 * rbT + 16 * m + 4 * g);
            *(bf16x4 *)(Rhi + off) = h4;
            *(bf16x4 *)(Rlo + off) = l4;
        }
        fetch_v(blk + 1);
        lds_barrier();
        // ---- S <- gam S + Z^T R for this wavefront's 32 rows
        f32x16 acc0 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}, acc1 = acc0;   // hi x hi, the two cross terms
        static_for<0, 4>([&](auto t_) {
            constexpr int t = decltype(t_)::value;
            const bf16x8 rh = *(const bf16x8 *)(Rhi + col * RROW + 32 * t + 16 * hh);
            const bf16x8 rl = *(const bf16x8 *)(Rlo + col * RROW + 32 * t + 16 * hh);
            acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(zh[bi][t], rh, acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(zh[bi][t], rl, acc1, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(zl[bi][t], rh, acc1, 0, 0, 0);
        });
        fetch_z(blk + 2, b_);
#pragma unroll
        for (int r = 0; r < 16; ++r) s_acc[r] = fmaf(gam_cur, s_acc[r], acc0[r]) + acc1[r];
        if constexpr (GROUPED) gprod *= gam_cur;
    };

    const std::integral_constant<int, 0> B0{};
    const std::integral_constant<int, 1> B1{};
    fetch_k(0, B0); fetch_v(0); fetch_z(0, B0);
    fetch_k(1, B1); fetch_z(1, B1);
    int blk = 0;
#pragma unroll 1
    for (; blk + 2 <= n; blk += 2) {
        step(blk, B0);
        step(blk + 1, B1);
    }
    if (blk < n) step(blk, B0);

    if (!GROUPED || grp == 0) {
#pragma unroll
        for (int r = 0; r < 16; ++r) Sg[(size_t)(32 * rbF + 8 * (r >> 2) + 4 * hh + (r & 3)) * D] = s_acc[r];
        return;
    }
    if constexpr (GROUPED) {
        // the composite map of run grp >= 1 as one record of the composed-map format
        unsigned char *rec = gmaps + ((size_t)bh * (groups - 1) + grp - 1) * gdn_block_bytes(D);
        if (!is_m) {                                     // c_g, accumulator order [row block][column block][quad][lane]
            f32x4 *Psi = (f32x4 *)(rec + (size_t)D * D * 4) + (rbF * NB + 2 * slice + cb) * 4 * 64 + lane;
#pragma unroll
            for (int q = 0; q < 4; ++q)
                Psi[q * 64] = f32x4{s_acc[4 * q], s_acc[4 * q + 1], s_acc[4 * q + 2], s_acc[4 * q + 3]};
            if (slice == 0 && tid == 0) *(float *)(rec + (size_t)D * D * 8) = gprod;
            return;
        }
        // M_g - gam_g I, columns 64 slice .. + 63: through LDS into A-fragment order (lane = row, eight
        // columns of k-steps 4 slice .. 4 slice + 3 in k-slot order), hi and lo parts
        __syncthreads();                                 // the exchange buffers are no longer read
        unsigned char *Thi = smem, *Tlo = smem + D * TROW;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = 32 * rbF + 8 * (r >> 2) + 4 * hh + (r & 3);
            const float x = s_acc[r] - (row == gcol ? gprod : 0.0f);
            const bf16_t h = to_bf16(x);
            *(bf16_t *)(Thi + row * TROW + 2 * col) = h;
            *(bf16_t *)(Tlo + row * TROW + 2 * col) = to_bf16(x - (float)h);
        }
        __syncthreads();
        bf16x8 *Ehi = (bf16x8 *)rec, *Elo = Ehi + D * D / 8;
#pragma unroll
        for (int i = 0; i < NB * 4 * 64 / 512; ++i) {    // NB * 4 * 64 fragment pieces, 512 threads
            const int p = tid + 512 * i;
            const int ln = p & 63, tl = (p >> 6) & 3, rb = p >> 8;
            const int off = (32 * rb + (ln & 31)) * TROW + 2 * (16 * tl + 4 * (ln >> 5));
            const bf16x4 h0 = *(const bf16x4 *)(Thi + off), h1 = *(const bf16x4 *)(Thi + off + 16);
            const bf16x4 l0 = *(const bf16x4 *)(Tlo + off), l1 = *(const bf16x4 *)(Tlo + off + 16);
            const int idx = (rb * KS + 4 * slice + tl) * 64 + ln;
            Ehi[idx] = __builtin_shufflevector(h0, h1, 0, 1, 2, 3, 4, 5, 6, 7);
            Elo[idx] = __builtin_shufflevector(l0, l1, 0, 1, 2, 3, 4, 5, 6, 7);
        }
    }
}

}  // namespace

// Runs of blocks that are walked at the same time: as many as keep the walk within about one workgroup
// per CU (the runs after the first cost twice the work), each at least four blocks long.
static int gdn_groups(int B, int H, int nblk, int D)
{
    const long long heads = (long long)B * H;
    int g = (int)((kNumCu / (heads * (D / 64)) + 1) / 2);   // (2 g - 1) * D / 64 slices * heads <= CUs
    if (g > nblk / 4) g = nblk / 4;
    if (g > 8) g = 8;
    return g < 1 ? 1 : g;
}

size_t gdn_workspace_bytes(int B, int H, int L, int D)
{
    const int nblk = (L + CT - 1) / CT;
    return (size_t)B * H * (nblk * gdn_ops_bytes(D) + (gdn_groups(B, H, nblk, D) - 1) * gdn_block_bytes(D));
}

template <int D>
static hipError_t launch_gdn(const GdnArgs &a, int nblk, unsigned nwg, hipStream_t stream)
{
    constexpr int NSL = D / 64;
    const int heads = a.B * a.H;
    const int groups = gdn_groups(a.B, a.H, nblk, D);
    const unsigned char *recs = (const unsigned char *)a.workspace;
    unsigned char *gmaps = (unsigned char *)a.workspace + (size_t)heads * nblk * gdn_ops_bytes(D);
    hipError_t e = launch_kernel(gdn_block_kernel<D>, dim3(nwg), dim3(NTA), stream, a, nblk);
    if (e != hipSuccess) return e;
    // whole owners per XCD: ceil(owners / 8) on each of the 8 XCDs
    const unsigned owners8 = (unsigned)((heads + kNumXcd - 1) / kNumXcd * kNumXcd);
    if (groups == 1) {
        if constexpr (D == 128)
            return launch_kernel(gdn_walk8_kernel<false>, dim3(owners8 * NSL), dim3(512), stream, a, recs, nblk, 1,
                                 (unsigned char *)nullptr);
        return launch_kernel(gdn_walk_kernel<D, false>, dim3(owners8 * NSL), dim3(256), stream, a, recs, nblk, 1,
                             (unsigned char *)nullptr);
    }
    // the runs after the first (c and M slices), then the first runs (c slices)
    const unsigned late8 = (unsigned)((heads * (groups - 1) + kNumXcd - 1) / kNumXcd * kNumXcd);
    if constexpr (D == 128)
        e = launch_kernel(gdn_walk8_kernel<true>, dim3(late8 * 2 * NSL + owners8 * NSL), dim3(512), stream, a, recs, nblk,
                          groups, gmaps);
    else
        e = launch_kernel(gdn_walk_kernel<D, true>, dim3(late8 * 2 * NSL + owners8 * NSL), dim3(256), stream, a, recs, nblk,
                          groups, gmaps);
    if (e != hipSuccess) return e;
    // the composite maps of the later runs, applied in order to what the first run left in S
    return launch_kernel(gdn_apply_kernel<D>, dim3(owners8 * (D / 32)), dim3(2 * D), stream, a, (const unsigned char *)gmaps,
                         groups - 1);
}

hipError_t launch_commit_gdn_bf16(const GdnArgs &a, hipStream_t stream)
{
    const int nblk = (a.L + CT - 1) / CT;
    const long long nwg = (long long)a.B * a.H * nblk;
    if (nwg <= 0 || nwg > 0x7fffffffLL) return hipErrorInvalidValue;
    // the block kernel addresses one stream's K (or V) with 32-bit byte offsets
    if ((long long)(a.L + 4 * CT) * a.H * a.D * 2 > 0x7fffffffLL) return hipErrorInvalidValue;
    if (a.D == 128) return launch_gdn<128>(a, nblk, (unsigned)nwg, stream);
    if (a.D == 64) return launch_gdn<64>(a, nblk, (unsigned)nwg, stream);
    return hipErrorInvalidValue;
}

}  // namespace arl2
