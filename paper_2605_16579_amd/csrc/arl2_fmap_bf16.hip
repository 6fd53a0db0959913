// Per-head feature map of the linear branch on bf16 MFMA (gfx950):
//   y[b][l][h][:] = RoPE_l( W[h] x[b][l][h][:] )                       paper Eq. (3) without its L2Norm
// (the readout and the commit kernels normalise the rows they read).  W[h] is the D x D matrix of the
// grouped 1 x 1 map of head h, indexed [out][in]; RoPE rotates the pairs (y[2i], y[2i+1]) by the angle
// whose cosine and sine the caller tabulates per token, [L][D/2]; no table means no rotation (phi_v).
//
// HBM-bound (x read once, y written once, 2 D flop per byte).  Computed transposed,
//   y^T[e][l] = sum_d W[e][d] x[l][d],
// so that a lane ends up with one token's outputs, four consecutive features per register quad: the
// two members of every rotation pair sit in the same lane.
//
// One workgroup owns four consecutive heads (wavefront = head) and one or more tiles of 32 tokens
// (as many as it takes to run the launch as one round of two workgroups per CU, at most 16).  The
// rows of four heads are 4 D contiguous bf16 per token, so the tile moves between HBM and LDS in
// whole 1 KB rows (D = 128); the rotation table of the tile, which all heads share, is staged once per
// tile.  Each wavefront keeps its head's W as MFMA A-operand fragments in registers for all its tiles,
// reads its x fragments (B operand) from the LDS tile, and writes its rotated outputs back into the
// same tile, which then leaves as whole rows.
#include "arl2_device.h"

#include <type_traits>

namespace arl2 {
namespace {

constexpr int NT = 256;    // four wavefronts = four heads
constexpr int HG = 4;      // heads per workgroup
constexpr int TT = 32;     // tokens per tile
constexpr int MAX_NTILE = 16;  // most tiles per workgroup (W stays in registers across them)

// PIPE: the x rows of the next tile are requested while the current one is computed (for workgroups that
// walk several tiles; with a single tile the extra live registers only cost: 8 spill at D = 128).
template <int D, bool PIPE>
__global__ __launch_bounds__(NT, 2) void feature_map_kernel(FmapArgs a, int n_ranges, int n_hg, int ntile)
{
    constexpr int KS = D / 16, EB = D / 32, CPR = D / 8;
    constexpr int HROW = 2 * D + 16;                     // LDS bytes per (token, head) row
    constexpr int TROW = HG * HROW + 16;                 // LDS bytes per token (conflict-free 16-byte column reads)
    constexpr int X_BYTES = TT * TROW;
    constexpr int TST = D / 2 + 2;                       // floats per token of a staged table (conflict-free 8-byte reads)
    constexpr int XCH = TT * HG * CPR / NT;              // 16-byte chunks of the x tile per thread
    constexpr int TCH = TT * (D / 8) / NT;               // 16-byte chunks of one table tile per thread
    static_assert(XCH >= 1 && TCH >= 1, "tile too small for the workgroup");
    __shared__ __attribute__((aligned(16))) unsigned char smem[X_BYTES + 2 * TT * TST * 4];
    float *cosT = (float *)(smem + X_BYTES), *sinT = cosT + TT * TST;

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, hh = lane >> 5, c = lane & 31;
    const int rng = blockIdx.x % n_ranges;
    const int hg = (blockIdx.x / n_ranges) % n_hg;
    const int b = blockIdx.x / (n_ranges * n_hg);
    const int L = a.L, H = a.H;
    const int h = hg * HG + wave;
    const bool active = h < H;
    const bool rope = a.cs != nullptr;

    // the whole x and y arrays as buffers: out-of-range chunks read zero / are dropped
    const uint32_t tok_bytes = (uint32_t)H * D * 2;
    const uint32_t total = (uint32_t)a.B * L * tok_bytes;
    const __amdgpu_buffer_rsrc_t x_rsrc = make_rsrc(a.x, total);
    const __amdgpu_buffer_rsrc_t y_rsrc = make_rsrc(a.y, total);
    const uint32_t tab_bytes = (uint32_t)L * (D / 2) * 4;
    const __amdgpu_buffer_rsrc_t c_rsrc = make_rsrc(rope ? a.cs : a.x, rope ? tab_bytes : 0);
    const __amdgpu_buffer_rsrc_t s_rsrc = make_rsrc(rope ? a.sn : a.x, rope ? tab_bytes : 0);

    // chunk i of this thread in a tile: token tk, 16-byte column col of the token's HG heads
    const uint32_t head0_bytes = (uint32_t)hg * HG * D * 2;
    // Loads of one tile's x rows into registers; a tile past the end of the chunk reads nothing (every
    // offset out of range).  The first tile is requested before the W fragments and every further tile
    // while the one before it is being computed.  (The rotation table rows, small and L2-resident, are
    // read when the tile is staged: holding them in registers too spills.)
    u32x4 xr[XCH];
    auto fetch_tile = [&](int tile) {
        const int l0 = (rng * ntile + tile) * TT;
        const bool live = tile < ntile && l0 < L;
#pragma unroll
        for (int i = 0; i < XCH; ++i) {
            const int id = tid + NT * i;
            const int tk = id / (HG * CPR), col = id % (HG * CPR);
            const bool ok = live && l0 + tk < L && hg * HG + col / CPR < H;
            const uint32_t off = ok ? ((uint32_t)b * L + l0 + tk) * tok_bytes + head0_bytes + 16 * col : total;
            xr[i] = __builtin_amdgcn_raw_buffer_load_b128(x_rsrc, off, 0, 0);
        }
    };
    if constexpr (PIPE) fetch_tile(0);

    // A operand: lane (row e = 32 eb + c, hh) holds W[h][e][16 t + 8 hh + 0..7], kept for all tiles.
    // The rows come in whole (16 lanes per 2 D-byte row) and pass, 32 rows at a time, through this
    // wavefront's quarter of the still empty tile buffer; fragment loads straight from global memory touch
    // 32 cache lines per instruction and are bound by cache-line requests.
    bf16x8 wf[EB][KS];
    static_assert(HG * TT * HROW <= X_BYTES && TT * CPR % 64 == 0, "W staging uses the tile buffer");
    if (active) {
        constexpr int WCH = TT * CPR / 64;               // 16-byte pieces of 32 rows per lane
        const bf16_t *Wg = (const bf16_t *)a.W + (size_t)h * D * D;
        unsigned char *wst = smem + wave * (TT * HROW);
        u32x4 wr[2][WCH];
        auto fetch_w = [&](auto eb_, auto buf_) {
            constexpr int eb = decltype(eb_)::value, buf = decltype(buf_)::value;
#pragma unroll
            for (int i = 0; i < WCH; ++i) {
                const int id = lane + 64 * i;
                wr[buf][i] = *(const u32x4 *)(Wg + (size_t)(32 * eb + id / CPR) * D + 8 * (id % CPR));
            }
        };
        fetch_w(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
        static_for<0, EB>([&](auto eb_) {
            constexpr int eb = decltype(eb_)::value;
            if constexpr (eb + 1 < EB) fetch_w(std::integral_constant<int, eb + 1>{}, std::integral_constant<int, (eb + 1) & 1>{});
#pragma unroll
            for (int i = 0; i < WCH; ++i) {
                const int id = lane + 64 * i;
                *(u32x4 *)(wst + (id / CPR) * HROW + 16 * (id % CPR)) = wr[eb & 1][i];
            }
#pragma unroll
            for (int t = 0; t < KS; ++t) wf[eb][t] = *(const bf16x8 *)(wst + c * HROW + 32 * t + 16 * hh);
        });
    }
    __syncthreads();                                     // the tile buffer is free for the first tile

    for (int tile = 0; tile < ntile; ++tile) {
        const int l0 = (rng * ntile + tile) * TT;
        if (l0 >= L) break;                              // uniform over the workgroup
        // ---- stage the x tile and the table tile
        if constexpr (!PIPE) fetch_tile(tile);
#pragma unroll
        for (int i = 0; i < XCH; ++i) {
            const int id = tid + NT * i;
            const int tk = id / (HG * CPR), col = id % (HG * CPR);
            *(u32x4 *)(smem + tk * TROW + (col / CPR) * HROW + 16 * (col % CPR)) = xr[i];
        }
        if (rope) {
#pragma unroll
            for (int i = 0; i < TCH; ++i) {
                const int id = tid + NT * i;
                const int tk = id / (D / 8), col = id % (D / 8);
                const uint32_t off = l0 + tk < L ? (uint32_t)(l0 + tk) * (D / 2) * 4 + 16 * col : tab_bytes;
                const u32x4 cv = __builtin_amdgcn_raw_buffer_load_b128(c_rsrc, off, 0, 0);
                const u32x4 sv = __builtin_amdgcn_raw_buffer_load_b128(s_rsrc, off, 0, 0);
                u32x2 *cd = (u32x2 *)(cosT + tk * TST + 4 * col), *sd = (u32x2 *)(sinT + tk * TST + 4 * col);
                cd[0] = u32x2{cv[0], cv[1]};
                cd[1] = u32x2{cv[2], cv[3]};
                sd[0] = u32x2{sv[0], sv[1]};
                sd[1] = u32x2{sv[2], sv[3]};
            }
        }
        __syncthreads();
        if constexpr (PIPE) fetch_tile(tile + 1);        // in flight during this tile's arithmetic
        // ---- B operand: lane (token c, hh) holds x[l0 + c][h][16 t + 8 hh + 0..7]
        bf16x8 xf[KS];
        unsigned char *mine = smem + c * TROW + wave * HROW;
#pragma unroll
        for (int t = 0; t < KS; ++t) xf[t] = *(const bf16x8 *)(mine + 32 * t + 16 * hh);
        __syncthreads();                                 // every wavefront holds its fragments: the tile may be overwritten
        if (active) {
#pragma unroll
            for (int eb = 0; eb < EB; ++eb) {
                f32x16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
                for (int t = 0; t < KS; ++t) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[eb][t], xf[t], acc, 0, 0, 0);
                // registers 4 q .. 4 q + 3 are features e0 .. e0 + 3, e0 = 32 eb + 8 q + 4 hh: pairs e0 / 2, e0 / 2 + 1
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    float y[4] = {acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
                    if (rope) {
                        const f32x2 c2 = *(const f32x2 *)(cosT + c * TST + 16 * eb + 4 * q + 2 * hh);
                        const f32x2 s2 = *(const f32x2 *)(sinT + c * TST + 16 * eb + 4 * q + 2 * hh);
#pragma unroll
                        for (int p = 0; p < 2; ++p) {
                            const float y0 = y[2 * p], y1 = y[2 * p + 1];
                            y[2 * p] = y0 * c2[p] - y1 * s2[p];
                            y[2 * p + 1] = fmaf(y0, s2[p], y1 * c2[p]);
                        }
                    }
                    bf16x4 w4;
#pragma unroll
                    for (int i = 0; i < 4; ++i) w4[i] = to_bf16(y[i]);
                    *(bf16x4 *)(mine + 2 * (32 * eb + 8 * q + 4 * hh)) = w4;
                }
            }
        }
        __syncthreads();
        // ---- the tile leaves as whole rows
#pragma unroll
        for (int i = 0; i < XCH; ++i) {
            const int id = tid + NT * i;
            const int tk = id / (HG * CPR), col = id % (HG * CPR);
            const bool ok = l0 + tk < L && hg * HG + col / CPR < H;
            const u32x4 v = *(const u32x4 *)(smem + tk * TROW + (col / CPR) * HROW + 16 * (col % CPR));
            const uint32_t off = ok ? ((uint32_t)b * L + l0 + tk) * tok_bytes + head0_bytes + 16 * col : total;
            __builtin_amdgcn_raw_buffer_store_b128(v, y_rsrc, off, 0, 0);
        }
        __syncthreads();                                 // the next tile's rows may be written
    }
}

}  // namespace

hipError_t launch_feature_map_bf16(const FmapArgs &a, hipStream_t stream)
{
    const int n_hg = (a.H + HG - 1) / HG;
    const int tiles = (a.L + TT - 1) / TT;
    // Two workgroups fit a CU (registers: W stays in them).  Up to that many workgroups run as one round,
    // each walking as many tiles as that takes; beyond MAX_NTILE tiles per workgroup there are enough
    // rounds for the last, partly filled one not to matter.
    const long long slots = 2 * kNumCu;
    long long ntile = ((long long)a.B * n_hg * tiles + slots - 1) / slots;
    if (ntile < 1) ntile = 1;
    if (ntile > MAX_NTILE) ntile = MAX_NTILE;
    const int n_ranges = (tiles + (int)ntile - 1) / (int)ntile;
    const long long nwg = (long long)a.B * n_hg * n_ranges;
    if (nwg <= 0 || nwg > 0x7fffffffLL) return hipErrorInvalidValue;
    // x and y are addressed with 32-bit byte offsets
    if ((long long)a.B * a.L * a.H * a.D * 2 > 0x7fffffffLL) return hipErrorInvalidValue;
    const dim3 grid((unsigned)nwg), block(NT);
    if (a.D == 128 && ntile > 1) return launch_kernel(feature_map_kernel<128, true>, grid, block, stream, a, n_ranges, n_hg, (int)ntile);
    if (a.D == 128) return launch_kernel(feature_map_kernel<128, false>, grid, block, stream, a, n_ranges, n_hg, (int)ntile);
    if (a.D == 64 && ntile > 1) return launch_kernel(feature_map_kernel<64, true>, grid, block, stream, a, n_ranges, n_hg, (int)ntile);
    if (a.D == 64) return launch_kernel(feature_map_kernel<64, false>, grid, block, stream, a, n_ranges, n_hg, (int)ntile);
    return hipErrorInvalidValue;
}

}  // namespace arl2
