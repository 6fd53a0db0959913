// Post-denoise state commit with the key and value feature maps of the linear branch fused in (gfx950):
//   S <- gate * S + sum_i L2Norm(RoPE_i(Wk[h] xk_i))^T (Wv[h] xv_i)             paper Eq. (3), Eq. (4)
// What arl2_feature_map (twice) followed by the plain commit computes, without the two [B][L][H][D]
// intermediates and their launches: a 64-token tile of xk and xv is mapped on MFMA inside the commit's
// token loop and handed, through LDS, to the contraction over tokens.
//
// One workgroup of eight wavefronts owns a share of the tokens of one (stream, head), as in the plain commit
// (token splits, fp32 D x D partial per split, the same reduce kernel).  Per tile:
//   1. the raw rows of xk, xv and of the rotation tables go from the prefetch registers to LDS;
//   2. wavefront (fb, tb) computes the 32-feature x 32-token blocks y_k^T = Wk x^T and y_v^T = Wv x^T (its rows of
//      Wk and Wv stay in registers as A fragments for the whole kernel; lanes hold one token's features, both
//      members of a rotation pair in one lane), rotates y_k, rounds it to bf16 -- the key operand of the
//      contraction -- and adds up the squares of the rounded values per token;
//   3. with the token's norm complete (sum over the feature blocks, fixed order), y_v is scaled by
//      r = 1/sqrt(|k'|^2 + eps) in fp32 and split into bf16 hi (truncated) + lo (rounded remainder): the
//      mapped values are never rounded to bf16 on their own, unlike in the two-launch path;
//   4. every wavefront contracts its 64 x 32 block of K'^T (r V') over the tile's tokens (transposing LDS reads,
//      two MFMAs per step as in the plain commit).
// The phases are separated by LDS-only barriers; the rows of the tile after next are in flight meanwhile.
//
// Operand tiles in LDS: token-major rows of 2 D + 64 bytes, which the transposing read of phase 4 needs (four
// consecutive rows start 16 banks apart).  Phases 2 and 3 write them one token per lane, 8 bytes at the same
// column of 32 rows: only four different bank phases, an 8-way conflict.  The 8-byte piece a value goes to is
// therefore XORed, within its 64-byte group, with bits 2..4 of the row: the eight rows that share a bank phase
// use eight different pieces, and the four rows a transposing read takes (one value of bits 2..4) still find
// their pieces side by side, permuted by a value the reader knows.
#include "arl2_device.h"

#include <type_traits>

namespace arl2 {
namespace {

constexpr int BT = 64;     // tokens per tile
constexpr int NT = 512;    // eight wavefronts
constexpr int PF = 2;      // tiles whose rows are in flight (register ring)

template <int D>
struct FmCfg {
    static constexpr int CPR = D / 8;                   // 16-byte chunks per row of x
    static constexpr int KS = D / 16;                   // k-steps of a D-long contraction
    static constexpr int EB = D / 32;                   // 32-wide feature blocks
    static constexpr int XROW = 2 * D + 16;             // LDS bytes per row of a raw x tile (16-byte column reads)
    static constexpr int X_BYTES = BT * XROW;
    static constexpr int ROW = 2 * D + 64;              // LDS bytes per row of an operand tile (transposing reads)
    static constexpr int MAT = BT * ROW;
    static constexpr int TST = D / 2 + 2;               // floats per token of a staged table (8-byte reads)
    static constexpr int T_BYTES = BT * TST * 4;
    static constexpr int XCH = BT * CPR / NT;           // chunks per thread per tile of xk (and of xv)
    static constexpr int TCH = BT * (D / 8) / NT;       // chunks per thread per tile of one table
    static constexpr int OFF_XK = 0, OFF_XV = X_BYTES;
    static constexpr int OFF_KP = 2 * X_BYTES;          // K' (bf16), then r V' hi, r V' lo: one stage of the plain commit
    static constexpr int OFF_COS = OFF_KP + 3 * MAT, OFF_SIN = OFF_COS + T_BYTES;
    static constexpr int OFF_NP = OFF_SIN + T_BYTES;    // [feature block][token] partial sums of squares
    static constexpr int SMEM = OFF_NP + EB * BT * 4;
    static constexpr int MAPW = 2 * EB;                 // wavefronts that own a block of the maps
    static constexpr int DH = D / 64;
    static constexpr int WAVES_USED = DH * EB;          // wavefronts that own a 64 x 32 block of the partial
    static constexpr int WST = 32 * XROW;               // staging slice of one wavefront's 32 rows of W
    static_assert(XCH >= 1 && TCH >= 1, "tile too small for the workgroup");
    static_assert(MAPW <= NT / 64 && WAVES_USED <= NT / 64, "more blocks than wavefronts");
    static_assert((NT / 64) * WST <= OFF_COS, "W staging uses the tile buffers");
    static_assert(SMEM <= 160 * 1024, "LDS");
};

template <int D>
__global__ __launch_bounds__(NT, 1) void commit_fm_partial_kernel(CommitFmArgs a)
{
    using C = FmCfg<D>;
    __shared__ __attribute__((aligned(16))) unsigned char smem[C::SMEM];
    float *cosT = (float *)(smem + C::OFF_COS), *sinT = (float *)(smem + C::OFF_SIN);
    float *np = (float *)(smem + C::OFF_NP);

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, hh = lane >> 5, c = lane & 31;
    const int split = blockIdx.x % a.nsplit;
    const int bh = blockIdx.x / a.nsplit;
    const int h = bh % a.H, b = bh / a.H;
    const int L = a.L, H = a.H;
    const bool rope = a.cs != nullptr;
    const uint32_t tok_bytes = (uint32_t)H * D * 2;
    const uint32_t range = (uint32_t)(L - 1) * tok_bytes + 2 * D;      // bytes of this head's slice
    const __amdgpu_buffer_rsrc_t xk_rsrc = make_rsrc((const bf16_t *)a.xk + ((size_t)b * L * H + h) * D, range);
    const __amdgpu_buffer_rsrc_t xv_rsrc = make_rsrc((const bf16_t *)a.xv + ((size_t)b * L * H + h) * D, range);
    const uint32_t tab_bytes = (uint32_t)L * (D / 2) * 4;
    const __amdgpu_buffer_rsrc_t c_rsrc = make_rsrc(rope ? (const void *)a.cs : a.xk, rope ? tab_bytes : 0);
    const __amdgpu_buffer_rsrc_t s_rsrc = make_rsrc(rope ? (const void *)a.sn : a.xk, rope ? tab_bytes : 0);

    const int ntiles = (L + BT - 1) / BT;
    const int t_begin = (int)((long long)split * ntiles / a.nsplit);
    const int t_end = (int)((long long)(split + 1) * ntiles / a.nsplit);

    // ---- rows of a tile: requested into register buffer `buf`, later written to LDS as they are.
    // Rows past the end of the sequence and tiles that are not this workgroup's read as zero (offsets beyond
    // the buffers): a zero row maps to a zero key and a zero value and adds nothing.
    u32x4 xkr[PF][C::XCH], xvr[PF][C::XCH], csr[PF][C::TCH], snr[PF][C::TCH];
    auto fetch = [&](int tile, auto buf_) {
        constexpr int buf = decltype(buf_)::value;
        const bool live = tile < t_end;
#pragma unroll
        for (int i = 0; i < C::XCH; ++i) {
            const int id = tid + NT * i;
            const int tok = tile * BT + id / C::CPR;
            const uint32_t off = live && tok < L ? (uint32_t)tok * tok_bytes + 16 * (id % C::CPR) : 0x80000000u;
            xkr[buf][i] = __builtin_amdgcn_raw_buffer_load_b128(xk_rsrc, off, 0, 0);
            xvr[buf][i] = __builtin_amdgcn_raw_buffer_load_b128(xv_rsrc, off, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < C::TCH; ++i) {
            const int id = tid + NT * i;
            const int tok = tile * BT + id / (D / 8);
            const uint32_t off = live && tok < L ? (uint32_t)tok * (D / 2) * 4 + 16 * (id % (D / 8)) : 0x80000000u;
            csr[buf][i] = __builtin_amdgcn_raw_buffer_load_b128(c_rsrc, off, 0, 0);
            snr[buf][i] = __builtin_amdgcn_raw_buffer_load_b128(s_rsrc, off, 0, 0);
        }
    };
    auto stage_raw = [&](auto buf_) {
        constexpr int buf = decltype(buf_)::value;
#pragma unroll
        for (int i = 0; i < C::XCH; ++i) {
            const int id = tid + NT * i;
            const int o = (id / C::CPR) * C::XROW + 16 * (id % C::CPR);
            *(u32x4 *)(smem + C::OFF_XK + o) = xkr[buf][i];
            *(u32x4 *)(smem + C::OFF_XV + o) = xvr[buf][i];
        }
        if (rope) {
#pragma unroll
            for (int i = 0; i < C::TCH; ++i) {
                const int id = tid + NT * i;
                const int o = (id / (D / 8)) * C::TST + 4 * (id % (D / 8));
                u32x2 *cd = (u32x2 *)(cosT + o), *sd = (u32x2 *)(sinT + o);
                cd[0] = u32x2{csr[buf][i][0], csr[buf][i][1]};
                cd[1] = u32x2{csr[buf][i][2], csr[buf][i][3]};
                sd[0] = u32x2{snr[buf][i][0], snr[buf][i][1]};
                sd[1] = u32x2{snr[buf][i][2], snr[buf][i][3]};
            }
        }
    };
    static_for<0, PF>([&](auto i_) { fetch(t_begin + decltype(i_)::value, i_); });

    // ---- this wavefront's block of the maps: features 32 fb .. + 31 of tokens 32 tb .. + 31 of a tile.
    // A operand: lane (row e = 32 fb + c, hh) holds W[h][e][16 t + 8 hh + 0..7].  The 32 rows come in whole
    // (coalesced) and pass through this wavefront's slice of the still unused tile buffers.
    const bool mapper = wave < C::MAPW;
    const int fb = wave % C::EB, tb = (wave / C::EB) & 1;
    bf16x8 wkf[C::KS], wvf[C::KS];
    if (mapper) {
        constexpr int WCH = 32 * C::CPR / 64;            // 16-byte pieces of 32 rows per lane
        unsigned char *wst = smem + wave * C::WST;
        const bf16_t *Wkg = (const bf16_t *)a.Wk + ((size_t)h * D + 32 * fb) * D;
        const bf16_t *Wvg = (const bf16_t *)a.Wv + ((size_t)h * D + 32 * fb) * D;
        u32x4 wr[2][WCH];
#pragma unroll
        for (int i = 0; i < WCH; ++i) {
            const int id = lane + 64 * i;
            wr[0][i] = *(const u32x4 *)(Wkg + (size_t)(id / C::CPR) * D + 8 * (id % C::CPR));
            wr[1][i] = *(const u32x4 *)(Wvg + (size_t)(id / C::CPR) * D + 8 * (id % C::CPR));
        }
        static_for<0, 2>([&](auto m_) {
            constexpr int m = decltype(m_)::value;
#pragma unroll
            for (int i = 0; i < WCH; ++i) {
                const int id = lane + 64 * i;
                *(u32x4 *)(wst + (id / C::CPR) * C::XROW + 16 * (id % C::CPR)) = wr[m][i];
            }
#pragma unroll
            for (int t = 0; t < C::KS; ++t) {
                const bf16x8 f = *(const bf16x8 *)(wst + c * C::XROW + 32 * t + 16 * hh);
                if constexpr (m == 0) wkf[t] = f;
                else wvf[t] = f;
            }
        });
    }
    __syncthreads();                                     // the tile buffers are free for the first tile

    // ---- this wavefront's 64 x 32 block of the D x D partial: feature blocks d0, d0 + 1 x e0
    const bool compute = wave < C::WAVES_USED;
    const int d0 = 2 * (wave / C::EB), e0 = wave % C::EB;
    // transposing read of tokens R + 0..3 (+ 4 hh), R = 16 t + 8 s: lane l of a group of 16 addresses row
    // R + l / 4 (+ 4 hh), logical piece 4 (l / 16 % 2) + l % 4; its row's swizzle is (4 t + 2 s + hh) % 8
    const int tr_row = (((lane & 15) >> 2) + 4 * hh) * C::ROW;
    const int tr_piece = (4 * ((lane >> 4) & 1) + (lane & 3)) ^ hh;
    f32x16 acc[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;

    const int tok_row = 32 * tb + c;                     // this lane's token within the tile (map phases)
    // byte offset, in an operand tile, of features 32 fb + 8 q + 4 hh + 0..3 of that token: piece 2 q + hh of
    // 64-byte group fb, swizzled with the row
    const int sw = (tok_row >> 2) & 7;
    auto opnd_off = [&](int q) { return tok_row * C::ROW + 64 * fb + 8 * ((2 * q + hh) ^ sw); };

    for (int tile0 = t_begin; tile0 < t_end; tile0 += PF) {
        static_for<0, PF>([&](auto i_) {
            const int tile = tile0 + decltype(i_)::value;
            if (tile >= t_end) return;                   // uniform over the workgroup
            stage_raw(i_);                               // waits for this tile's rows
            lds_barrier();
            fetch(tile + PF, i_);
            f32x16 yv = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
            if (mapper) {
                // B operand: lane (token c, hh) holds x[32 tb + c][16 t + 8 hh + 0..7]
                const unsigned char *xkp = smem + C::OFF_XK + tok_row * C::XROW + 16 * hh;
                const unsigned char *xvp = smem + C::OFF_XV + tok_row * C::XROW + 16 * hh;
                f32x16 yk = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
                for (int t = 0; t < C::KS; ++t) {
                    yk = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wkf[t], *(const bf16x8 *)(xkp + 32 * t), yk, 0, 0, 0);
                    yv = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wvf[t], *(const bf16x8 *)(xvp + 32 * t), yv, 0, 0, 0);
                }
                // registers 4 q .. 4 q + 3 are features e = 32 fb + 8 q + 4 hh + 0..3: rotation pairs e / 2, e / 2 + 1
                float ss = 0.f;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    float y[4] = {yk[4 * q], yk[4 * q + 1], yk[4 * q + 2], yk[4 * q + 3]};
                    if (rope) {
                        const f32x2 c2 = *(const f32x2 *)(cosT + tok_row * C::TST + 16 * fb + 4 * q + 2 * hh);
                        const f32x2 s2 = *(const f32x2 *)(sinT + tok_row * C::TST + 16 * fb + 4 * q + 2 * hh);
#pragma unroll
                        for (int p = 0; p < 2; ++p) {
                            const float y0 = y[2 * p], y1 = y[2 * p + 1];
                            y[2 * p] = y0 * c2[p] - y1 * s2[p];
                            y[2 * p + 1] = fmaf(y0, s2[p], y1 * c2[p]);
                        }
                    }
                    bf16x4 w4;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        w4[i] = to_bf16(y[i]);
                        const float kr = (float)w4[i];   // the norm is that of the operand the contraction reads
                        ss = fmaf(kr, kr, ss);
                    }
                    *(bf16x4 *)(smem + C::OFF_KP + opnd_off(q)) = w4;
                }
                ss = xhalf_sum(ss);
                if (hh == 0) np[fb * BT + tok_row] = ss;
            }
            lds_barrier();
            if (mapper) {
                float tot = 0.f;
#pragma unroll
                for (int f = 0; f < C::EB; ++f) tot += np[f * BT + tok_row];
                const float rn = fast_rsqrt(tot + a.l2_eps);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    u32x2 vh, vl;
#pragma unroll
                    for (int p = 0; p < 2; ++p) {
                        uint32_t h0, h1;
                        float l0, l1;
                        split_bf16_trunc(yv[4 * q + 2 * p] * rn, h0, l0);
                        split_bf16_trunc(yv[4 * q + 2 * p + 1] * rn, h1, l1);
                        vh[p] = (h0 >> 16) | h1;
                        union { bf16x2 v; uint32_t u; } pk;
                        pk.v[0] = to_bf16(l0);
                        pk.v[1] = to_bf16(l1);
                        vl[p] = pk.u;
                    }
                    *(u32x2 *)(smem + C::OFF_KP + C::MAT + opnd_off(q)) = vh;
                    *(u32x2 *)(smem + C::OFF_KP + 2 * C::MAT + opnd_off(q)) = vl;
                }
            }
            lds_barrier();
            if (compute) {
                const unsigned char *sm = smem + C::OFF_KP + tr_row;
                // operand fragments of 16-token step t: tokens 16t + 4hh + 0..3 and 16t + 8 + 4hh + 0..3
                bf16x8 ka[2][2], vh[2], vl[2];
                auto load_step = [&](int t, int buf) {
                    const unsigned char *r0 = sm + 16 * t * C::ROW + 8 * (tr_piece ^ ((4 * t) & 7));
                    const unsigned char *r1 = sm + (16 * t + 8) * C::ROW + 8 * (tr_piece ^ ((4 * t + 2) & 7));
                    auto pair = [&](int off) {
                        return __builtin_shufflevector(lds_read_tr(r0 + off), lds_read_tr(r1 + off), 0, 1, 2, 3, 4, 5, 6, 7);
                    };
#pragma unroll
                    for (int i = 0; i < 2; ++i) ka[buf][i] = pair(64 * (d0 + i));
                    vh[buf] = pair(C::MAT + 64 * e0);
                    vl[buf] = pair(2 * C::MAT + 64 * e0);
                };
                load_step(0, 0);
#pragma unroll
                for (int t = 0; t < BT / 16; ++t) {
                    if (t + 1 < BT / 16) load_step(t + 1, (t + 1) & 1);
#pragma unroll
                    for (int i = 0; i < 2; ++i) {
                        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[t & 1][i], vh[t & 1], acc[i], 0, 0, 0);
                        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[t & 1][i], vl[t & 1], acc[i], 0, 0, 0);
                    }
                }
            }
        });
    }

    // partial[bh][split][d][e]
    if (compute) {
        float *part = (float *)a.workspace + ((size_t)bh * a.nsplit + split) * D * D;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int d = 32 * (d0 + i) + 8 * (r >> 2) + 4 * hh + (r & 3);
                part[(size_t)d * D + 32 * e0 + c] = acc[i][r];
            }
    }
}

}  // namespace

hipError_t launch_commit_fm_bf16(const CommitFmArgs &a, hipStream_t stream)
{
    const long long nwg = (long long)a.B * a.H * a.nsplit;
    if (nwg <= 0 || nwg > 0x7fffffffLL) return hipErrorInvalidValue;
    // one stream's xk (or xv) and a rotation table are addressed with 32-bit byte offsets
    if ((long long)(a.L + 4 * BT) * a.H * a.D * 2 > 0x7fffffffLL) return hipErrorInvalidValue;
    if ((long long)(a.L + 4 * BT) * (a.D / 2) * 4 > 0x7fffffffLL) return hipErrorInvalidValue;
    hipError_t e;
    if (a.D == 128)
        e = launch_kernel(commit_fm_partial_kernel<128>, dim3((unsigned)nwg), dim3(NT), stream, a);
    else if (a.D == 64)
        e = launch_kernel(commit_fm_partial_kernel<64>, dim3((unsigned)nwg), dim3(NT), stream, a);
    else
        return hipErrorInvalidValue;
    if (e != hipSuccess) return e;
    CommitArgs r;
    r.k = nullptr; r.v = nullptr; r.gate = a.gate; r.beta = nullptr; r.S = a.S; r.workspace = a.workspace;
    r.B = a.B; r.H = a.H; r.L = a.L; r.D = a.D; r.nsplit = a.nsplit; r.l2_eps = a.l2_eps;
    return launch_commit_reduce_bf16(r, stream);
}

}  // namespace arl2
