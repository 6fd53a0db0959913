// Post-denoise state commit with the key and value feature maps of the linear branch fused in (gfx950):
//   S <- gate * S + sum_i L2Norm(RoPE_i(Wk[h] xk_i))^T (Wv[h] xv_i)             paper Eq. (3), Eq. (4)
// What arl2_feature_map (twice) followed by the plain commit computes, without the two [B][L][H][D]
// intermediates and their launches: a 64-token tile of xk and xv is mapped on MFMA inside the commit's
// token loop and handed, through LDS, to the contraction over tokens.
//
// One workgroup of eight wavefronts owns a share of the tokens of one (stream, head), as in the plain commit
// (token splits, fp32 D x D partial per split, the same reduce kernel).  The work on a tile:
//   stage     the raw rows of xk, xv and of the rotation tables go from prefetch registers to LDS;
//   map       wavefront (fb, tb) computes the 32-feature x 32-token blocks y_k^T = Wk x^T and y_v^T = Wv x^T (its rows
//             of Wk and Wv stay in registers as A fragments for the whole kernel; a lane holds one token's
//             features, both members of a rotation pair);
//   key       y_k is rotated and rounded to bf16 -- the key operand of the contraction -- and the squares of the
//             rounded values are added up per token (partial sums per feature block, through LDS);
//   value     with the token's norm complete (sum over the feature blocks, fixed order), y_v is scaled by
//             r = 1/sqrt(|k'|^2 + eps) in fp32 and split into bf16 hi (truncated) + lo (rounded remainder): the
//             mapped values are never rounded to bf16 on their own, unlike in the three-call path;
//   contract  every wavefront contracts its 64 x 32 block of K'^T (r V') over the tile's tokens (transposing LDS
//             reads, two MFMAs per step as in the plain commit).
// map and contract run on the matrix cores, key and value on the vector ALU, and a wavefront overlaps the two
// when they are independent.  The loop is therefore a software pipeline with two barrier intervals per tile:
//   interval 1 of tile j:  value(j), key(j) to its operand tile, tables(j+1) staged   |  map(j+1)
//   interval 2 of tile j:  key(j+1) rotated and rounded in registers, x(j+2) staged    |  contract(j)
// with the raw x rows double-buffered in LDS (map(j+1) reads one buffer while x(j+2) lands in the other).
//
// LDS layouts.  Operand tiles (K', r V' hi, r V' lo): token-major rows of 2 D + 64 bytes, which the
// transposing read of the contraction needs (four consecutive rows start 16 banks apart).  key and value write
// them one token per lane, 8 bytes at the same column of 32 rows: only four different bank phases, an 8-way
// conflict.  The 8-byte piece a value goes to is therefore XORed, within its 64-byte group, with bits 2..4 of
// the row: the eight rows that share a bank phase use eight different pieces, and the four rows a
// transposing read takes (one value of bits 2..4) still find their pieces side by side, permuted by a value the
// reader knows.  Raw x tiles: rows of 2 D bytes without padding (two buffers of xk and xv plus the tables and
// the operand tiles fill the 160 KB), the 16-byte chunk index XORed with the row so that the 16 rows a
// B-operand read touches at one column fall on different banks.
#include "arl2_device.h"

#include <type_traits>

namespace arl2 {
namespace {

constexpr int BT = 64;     // tokens per tile
constexpr int NT = 512;    // eight wavefronts

template <int D>
struct FmCfg {
    static constexpr int CPR = D / 8;                   // 16-byte chunks per row of x
    static constexpr int KS = D / 16;                   // k-steps of a D-long contraction
    static constexpr int EB = D / 32;                   // 32-wide feature blocks
    static constexpr int XROW = 2 * D;                  // LDS bytes per row of a raw x tile (chunks swizzled)
    static constexpr int RPB = 256 / XROW;              // rows that share the 64 banks (1 or 2)
    static constexpr int X_BYTES = BT * XROW;           // one tile of xk or xv
    static constexpr int ROW = 2 * D + 64;              // LDS bytes per row of an operand tile (transposing reads)
    static constexpr int MAT = BT * ROW;
    static constexpr int TST = D / 2 + 2;               // floats per token of a staged table (8-byte reads)
    static constexpr int T_BYTES = BT * TST * 4;
    static constexpr int XCH = BT * CPR / NT;           // chunks per thread per tile of xk (and of xv)
    static constexpr int TCH = BT * (D / 8) / NT;       // chunks per thread per tile of one table
    static constexpr int OFF_X = 0;                     // [buffer][xk, xv]
    static constexpr int OFF_KP = 4 * X_BYTES;          // K' (bf16), then r V' hi, r V' lo: one stage of the plain commit
    static constexpr int OFF_COS = OFF_KP + 3 * MAT, OFF_SIN = OFF_COS + T_BYTES;
    static constexpr int OFF_NP = OFF_SIN + T_BYTES;    // [feature block][token] partial sums of squares
    static constexpr int SMEM = OFF_NP + EB * BT * 4;
    static constexpr int MAPW = 2 * EB;                 // wavefronts that own a block of the maps
    static constexpr int DH = D / 64;
    static constexpr int WAVES_USED = DH * EB;          // wavefronts that own a 64 x 32 block of the partial
    static constexpr int WROW = 2 * D + 16;             // row of the staging slice of one wavefront's 32 rows of W
    static constexpr int WST = 32 * WROW;
    static_assert(XCH >= 1 && TCH >= 1, "tile too small for the workgroup");
    static_assert(MAPW <= NT / 64 && WAVES_USED <= NT / 64, "more blocks than wavefronts");
    static_assert(XROW == 256 || XROW == 128, "the chunk swizzle assumes one or two rows per 256 bytes");
    static_assert((NT / 64) * WST <= OFF_COS, "W staging uses the tile buffers");
    static_assert(SMEM <= 160 * 1024, "LDS");
    // byte offset of 16-byte chunk ch of row r in a raw x tile
    __device__ static constexpr int x_off(int r, int ch) { return r * XROW + 16 * (ch ^ ((r / RPB) & (CPR - 1))); }
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
    const int n = t_end - t_begin;

    // ---- rows of a tile: requested into registers, later written to LDS as they are.
    // Rows past the end of the sequence and tiles that are not this workgroup's read as zero (offsets beyond
    // the buffers): a zero row maps to a zero key and a zero value and adds nothing.
    u32x4 xkr[C::XCH], xvr[C::XCH], csr[C::TCH], snr[C::TCH];
    auto fetch_x = [&](int tile) __attribute__((always_inline)) {
        const bool live = tile < t_end;
#pragma unroll
        for (int i = 0; i < C::XCH; ++i) {
            const int id = tid + NT * i;
            const int tok = tile * BT + id / C::CPR;
            const uint32_t off = live && tok < L ? (uint32_t)tok * tok_bytes + 16 * (id % C::CPR) : 0x80000000u;
            xkr[i] = __builtin_amdgcn_raw_buffer_load_b128(xk_rsrc, off, 0, 0);
            xvr[i] = __builtin_amdgcn_raw_buffer_load_b128(xv_rsrc, off, 0, 0);
        }
    };
    auto fetch_tables = [&](int tile) __attribute__((always_inline)) {
        const bool live = tile < t_end;
#pragma unroll
        for (int i = 0; i < C::TCH; ++i) {
            const int id = tid + NT * i;
            const int tok = tile * BT + id / (D / 8);
            const uint32_t off = live && tok < L ? (uint32_t)tok * (D / 2) * 4 + 16 * (id % (D / 8)) : 0x80000000u;
            csr[i] = __builtin_amdgcn_raw_buffer_load_b128(c_rsrc, off, 0, 0);
            snr[i] = __builtin_amdgcn_raw_buffer_load_b128(s_rsrc, off, 0, 0);
        }
    };
    auto stage_x = [&](int buf) __attribute__((always_inline)) {     // waits for the rows
        unsigned char *xb = smem + C::OFF_X + buf * 2 * C::X_BYTES;
#pragma unroll
        for (int i = 0; i < C::XCH; ++i) {
            const int id = tid + NT * i;
            const int o = C::x_off(id / C::CPR, id % C::CPR);
            *(u32x4 *)(xb + o) = xkr[i];
            *(u32x4 *)(xb + C::X_BYTES + o) = xvr[i];
        }
    };
    auto stage_tables = [&]() __attribute__((always_inline)) {
        if (!rope) return;
#pragma unroll
        for (int i = 0; i < C::TCH; ++i) {
            const int id = tid + NT * i;
            const int o = (id / (D / 8)) * C::TST + 4 * (id % (D / 8));
            u32x2 *cd = (u32x2 *)(cosT + o), *sd = (u32x2 *)(sinT + o);
            cd[0] = u32x2{csr[i][0], csr[i][1]};
            cd[1] = u32x2{csr[i][2], csr[i][3]};
            sd[0] = u32x2{snr[i][0], snr[i][1]};
            sd[1] = u32x2{snr[i][2], snr[i][3]};
        }
    };
    fetch_x(t_begin);
    fetch_tables(t_begin);

    // ---- this wavefront's block of the maps: features 32 fb .. + 31 of tokens 32 tb .. + 31 of a tile.
    // A operand: lane (row e = 32 fb + c, hh) holds W[h][e][16 t + 8 hh + 0..7].  The 32 rows come in whole
    // (coalesced) and pass through this wavefront's slice of the still unused tile buffers.
    const bool mapper = C::MAPW == NT / 64 || wave < C::MAPW;   // (D = 128: every wavefront, known at compile time)
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
                *(u32x4 *)(wst + (id / C::CPR) * C::WROW + 16 * (id % C::CPR)) = wr[m][i];
            }
#pragma unroll
            for (int t = 0; t < C::KS; ++t) {
                const bf16x8 f = *(const bf16x8 *)(wst + c * C::WROW + 32 * t + 16 * hh);
                if constexpr (m == 0) wkf[t] = f;
                else wvf[t] = f;
            }
        });
    }
    __syncthreads();                                     // the tile buffers are free for the first tile

    // ---- this wavefront's 64 x 32 block of the D x D partial: feature blocks d0, d0 + 1 x e0
    const bool compute = C::WAVES_USED == NT / 64 || wave < C::WAVES_USED;
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

    const int tok_row = 32 * tb + c;                     // this lane's token within the tile (map, key, value)
    // byte offset, in an operand tile, of features 32 fb + 8 q + 4 hh + 0..3 of that token: piece 2 q + hh of
    // 64-byte group fb, swizzled with the row
    const int sw = (tok_row >> 2) & 7;
    auto opnd_off = [&](int q) { return tok_row * C::ROW + 64 * fb + 8 * ((2 * q + hh) ^ sw); };
    // B operand of k-step t: chunk 2 t + hh of the token's row, at chunk slot (2 t) ^ xsw
    const int x_row = tok_row * C::XROW;
    const int xsw = 16 * (hh ^ ((tok_row / C::RPB) & (C::CPR - 1)));
    const float *cosp = cosT + tok_row * C::TST + 16 * fb + 2 * hh, *sinp = sinT + tok_row * C::TST + 16 * fb + 2 * hh;

    // ---- the pieces of a tile's work.  yk, yv: this wavefront's blocks of the mapped key and value (fp32);
    // kq: the rotated key rounded to bf16, four features per quad.
    f32x16 yk, yv_next, yv;
    bf16x4 kq[4];
    // k-step t of both maps, on the raw rows in x buffer `xb`
    auto map_step = [&](const unsigned char *xb, int t) __attribute__((always_inline)) {
        if (!mapper) return;
        if (t == 0) {
#pragma unroll
            for (int r = 0; r < 16; ++r) yk[r] = yv_next[r] = 0.f;
        }
        const unsigned char *p = xb + x_row + (xsw ^ (32 * t));
        yk = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wkf[t], *(const bf16x8 *)p, yk, 0, 0, 0);
        yv_next = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wvf[t], *(const bf16x8 *)(p + C::X_BYTES), yv_next, 0, 0, 0);
    };
    // quad q of the mapped key: registers 4 q .. 4 q + 3 are features e = 32 fb + 8 q + 4 hh + 0..3, rotation pairs
    // e / 2 and e / 2 + 1; rotate, round, add the squares of the rounded values to ss
    float ss = 0.f;
    auto key_quad = [&](int q) __attribute__((always_inline)) {
        if (!mapper) return;
        float y[4] = {yk[4 * q], yk[4 * q + 1], yk[4 * q + 2], yk[4 * q + 3]};
        if (rope) {
            const f32x2 c2 = *(const f32x2 *)(cosp + 4 * q);
            const f32x2 s2 = *(const f32x2 *)(sinp + 4 * q);
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                const float y0 = y[2 * p], y1 = y[2 * p + 1];
                y[2 * p] = y0 * c2[p] - y1 * s2[p];
                y[2 * p + 1] = fmaf(y0, s2[p], y1 * c2[p]);
            }
        }
        if (q == 0) ss = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            kq[q][i] = to_bf16(y[i]);
            const float kr = (float)kq[q][i];            // the norm is that of the operand the contraction reads
            ss = fmaf(kr, kr, ss);
        }
        if (q == 3) {
            ss = xhalf_sum(ss);
            if (hh == 0) np[fb * BT + tok_row] = ss;
        }
    };
    auto write_key = [&]() __attribute__((always_inline)) {
        if (!mapper) return;
#pragma unroll
        for (int q = 0; q < 4; ++q) *(bf16x4 *)(smem + C::OFF_KP + opnd_off(q)) = kq[q];
    };
    // the token's inverse norm from the partial sums of the feature blocks (fixed order)
    float rn = 0.f;
    auto norm = [&]() __attribute__((always_inline)) {
        if (!mapper) return;
        float tot = 0.f;
#pragma unroll
        for (int f = 0; f < C::EB; ++f) tot += np[f * BT + tok_row];
        rn = fast_rsqrt(tot + a.l2_eps);
    };
    // quad q of the mapped value: scaled, split into bf16 hi + lo, written to the operand tiles
    auto value_quad = [&](int q) __attribute__((always_inline)) {
        if (!mapper) return;
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
    };
    // contraction over the tile in the operand tiles: fragments of 16-token step t are tokens 16t + 4hh + 0..3
    // and 16t + 8 + 4hh + 0..3
    bf16x8 ka[2][2], vhf[2], vlf[2];
    auto load_step = [&](int t, int buf) __attribute__((always_inline)) {
        if (!compute) return;
        const unsigned char *sm = smem + C::OFF_KP + tr_row;
        const unsigned char *r0 = sm + 16 * t * C::ROW + 8 * (tr_piece ^ ((4 * t) & 7));
        const unsigned char *r1 = sm + (16 * t + 8) * C::ROW + 8 * (tr_piece ^ ((4 * t + 2) & 7));
        auto pair = [&](int off) {
            return __builtin_shufflevector(lds_read_tr(r0 + off), lds_read_tr(r1 + off), 0, 1, 2, 3, 4, 5, 6, 7);
        };
#pragma unroll
        for (int i = 0; i < 2; ++i) ka[buf][i] = pair(64 * (d0 + i));
        vhf[buf] = pair(C::MAT + 64 * e0);
        vlf[buf] = pair(2 * C::MAT + 64 * e0);
    };
    auto contract_step = [&](int t) __attribute__((always_inline)) {
        if (!compute) return;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[t & 1][i], vhf[t & 1], acc[i], 0, 0, 0);
            acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[t & 1][i], vlf[t & 1], acc[i], 0, 0, 0);
        }
    };

    // ---- software pipeline over this workgroup's tiles j = 0 .. n - 1 (tile t_begin + j; x buffer j % 2).
    // Work on a tile past the last one runs on zero rows or stale buffers and is never read: the loop body has
    // no branches, and every address stays inside the buffers.
    unsigned char *const xbuf0 = smem + C::OFF_X, *const xbuf1 = xbuf0 + 2 * C::X_BYTES;
    stage_x(0);                                          // tile 0
    stage_tables();
    fetch_x(t_begin + 1);
    fetch_tables(t_begin + 1);
    lds_barrier();
    static_for<0, C::KS>([&](auto t_) { map_step(xbuf0, decltype(t_)::value); });
    static_for<0, 4>([&](auto q_) { key_quad(decltype(q_)::value); });
#pragma unroll
    for (int r = 0; r < 16; ++r) yv[r] = yv_next[r];
    stage_x(1);                                          // tile 1
    fetch_x(t_begin + 2);
    lds_barrier();                                       // tile 0: norms complete, tables consumed; tile 1: rows staged
    for (int j = 0; j < n; ++j) {
        // interval 1: key (to its tile) and value of tile j, tables of tile j + 1   |   maps of tile j + 1
        const unsigned char *xb = (j & 1) ? xbuf0 : xbuf1;            // buffer (j + 1) % 2
        write_key();
        norm();
        static_for<0, 4>([&](auto q_) {
            constexpr int q = decltype(q_)::value;
            if constexpr (2 * q < C::KS) map_step(xb, 2 * q);
            if constexpr (2 * q + 1 < C::KS) map_step(xb, 2 * q + 1);
            value_quad(q);
        });
        stage_tables();                                  // tile j + 1
        fetch_tables(t_begin + j + 2);
        lds_barrier();
        // interval 2: key of tile j + 1 rotated and rounded, rows of tile j + 2   |   contraction of tile j
        load_step(0, 0);
        static_for<0, BT / 16>([&](auto t_) {
            constexpr int t = decltype(t_)::value;
            if constexpr (t + 1 < BT / 16) load_step(t + 1, (t + 1) & 1);
            contract_step(t);
            key_quad(t);
        });
#pragma unroll
        for (int r = 0; r < 16; ++r) yv[r] = yv_next[r];
        stage_x(j & 1);                                  // tile j + 2 into buffer j % 2
        fetch_x(t_begin + j + 3);
        lds_barrier();
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
