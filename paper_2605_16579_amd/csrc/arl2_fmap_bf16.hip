// Per-head feature map of the linear branch on bf16 MFMA (gfx950):
//   y[b][l][h][:] = RoPE_l( W[h] x[b][l][h][:] )                       paper Eq. (3) without its L2Norm
// (the readout and the commit kernels normalise the rows they read).  W[h] is the D x D matrix of the
// grouped 1 x 1 map of head h, indexed [out][in]; RoPE rotates the pairs (y[2i], y[2i+1]) by the angle
// whose cosine and sine the caller tabulates per token, [L][D/2]; no table means no rotation (phi_v).
//
// HBM-bound (x read once, y written once, 2 D flop per byte).  Computed transposed,
//   y^T[e][l] = sum_d W[e][d] x[l][d],
// so that both operands are read as rows (A = rows of W, B = rows of x, 16 bytes per lane straight
// from global memory) and a lane ends up with one token's outputs, four consecutive features per
// register quad: the two members of every rotation pair sit in the same lane.  One wavefront owns 32
// tokens of one head; results are transposed through LDS so that every output row is written as
// contiguous 16-byte pieces.
#include "arl2_device.h"

namespace arl2 {
namespace {

constexpr int NT = 256;    // four wavefronts, 32 tokens each

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}

template <int D>
__global__ __launch_bounds__(NT, 2) void feature_map_kernel(FmapArgs a, int n_tiles)
{
    constexpr int KS = D / 16, EB = D / 32, CPR = D / 8;
    constexpr int OROW = 2 * D + 16;                     // LDS bytes per staged output row
    __shared__ __attribute__((aligned(16))) unsigned char smem[4 * 32 * OROW];

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, hh = lane >> 5, c = lane & 31;
    const int tile = blockIdx.x % n_tiles;
    const int bh = blockIdx.x / n_tiles;
    const int h = bh % a.H, b = bh / a.H;
    const int L = a.L, H = a.H;
    const int l0 = tile * 128 + wave * 32;               // this wavefront's first token
    const int l = l0 + c;                                // this lane's token
    const uint32_t tok_bytes = (uint32_t)H * D * 2;
    const bf16_t *xg = (const bf16_t *)a.x + ((size_t)b * L * H + h) * D;
    const __amdgpu_buffer_rsrc_t x_rsrc = make_rsrc(xg, (uint32_t)(L - 1) * tok_bytes + 2 * D);

    // B operand: lane (token c, hh) holds x[l][16 t + 8 hh + 0..7]; tokens past the end read as zero
    bf16x8 xf[KS];
#pragma unroll
    for (int t = 0; t < KS; ++t) {
        union { u32x4 u; bf16x8 v; } cv;
        cv.u = __builtin_amdgcn_raw_buffer_load_b128(x_rsrc, (uint32_t)l * tok_bytes + 32 * t + 16 * hh, 0, 0);
        xf[t] = cv.v;
    }

    // A operand: lane (row e = 32 eb + c, hh) holds W[h][e][16 t + 8 hh + 0..7]
    const bf16_t *Wg = (const bf16_t *)a.W + (size_t)h * D * D + (size_t)c * D + 8 * hh;
    f32x16 acc[EB];
#pragma unroll
    for (int eb = 0; eb < EB; ++eb) {
        bf16x8 wf[KS];
#pragma unroll
        for (int t = 0; t < KS; ++t) wf[t] = *(const bf16x8 *)(Wg + (size_t)32 * eb * D + 16 * t);
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[eb][r] = 0.f;
#pragma unroll
        for (int t = 0; t < KS; ++t) acc[eb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[t], xf[t], acc[eb], 0, 0, 0);
    }

    // rotation: registers 4 q .. 4 q + 3 of block eb are features e0 .. e0 + 3, e0 = 32 eb + 8 q + 4 hh,
    // i.e. the pairs e0 / 2 and e0 / 2 + 1
    if (a.cs != nullptr) {
        const int lc = l < L ? l : L - 1;
        const float *cs = a.cs + (size_t)lc * (D / 2) + 2 * hh;
        const float *sn = a.sn + (size_t)lc * (D / 2) + 2 * hh;
#pragma unroll
        for (int eb = 0; eb < EB; ++eb)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f32x2 c2 = *(const f32x2 *)(cs + 16 * eb + 4 * q);
                const f32x2 s2 = *(const f32x2 *)(sn + 16 * eb + 4 * q);
#pragma unroll
                for (int p = 0; p < 2; ++p) {
                    const float y0 = acc[eb][4 * q + 2 * p], y1 = acc[eb][4 * q + 2 * p + 1];
                    acc[eb][4 * q + 2 * p] = y0 * c2[p] - y1 * s2[p];
                    acc[eb][4 * q + 2 * p + 1] = fmaf(y0, s2[p], y1 * c2[p]);
                }
            }
    }

    // transpose through this wavefront's LDS region, then whole rows go out as 16-byte pieces
    unsigned char *region = smem + wave * 32 * OROW;
#pragma unroll
    for (int eb = 0; eb < EB; ++eb)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            bf16x4 w4;
#pragma unroll
            for (int i = 0; i < 4; ++i) w4[i] = to_bf16(acc[eb][4 * q + i]);
            *(bf16x4 *)(region + c * OROW + 2 * (32 * eb + 8 * q + 4 * hh)) = w4;
        }
    __builtin_amdgcn_wave_barrier();
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the region is private to this wavefront
    bf16_t *yg = (bf16_t *)a.y + ((size_t)b * L * H + h) * D;
#pragma unroll
    for (int i = 0; i < CPR / 2; ++i) {
        const int idx = lane + 64 * i;
        const int row = idx / CPR, col = idx % CPR;
        if (l0 + row < L) {
            const u32x4 v = *(const u32x4 *)(region + row * OROW + 16 * col);
            *(u32x4 *)(yg + (size_t)(l0 + row) * H * D + 8 * col) = v;
        }
    }
}

}  // namespace

hipError_t launch_feature_map_bf16(const FmapArgs &a, hipStream_t stream)
{
    const int n_tiles = (a.L + 127) / 128;
    const long long nwg = (long long)a.B * a.H * n_tiles;
    if (nwg <= 0 || nwg > 0x7fffffffLL) return hipErrorInvalidValue;
    // one stream's x is addressed with 32-bit byte offsets
    if ((long long)(a.L + 128) * a.H * a.D * 2 > 0x7fffffffLL) return hipErrorInvalidValue;
    if (a.D == 128)
        hipLaunchKernelGGL(feature_map_kernel<128>, dim3((unsigned)nwg), dim3(NT), 0, stream, a, n_tiles);
    else if (a.D == 64)
        hipLaunchKernelGGL(feature_map_kernel<64>, dim3((unsigned)nwg), dim3(NT), 0, stream, a, n_tiles);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace arl2
