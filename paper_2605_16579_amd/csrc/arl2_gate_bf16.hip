// Branch-mix gate on bf16 MFMA (gfx950):
//   G[b][l][n] = sigmoid( sum_j x[b][l][j] Wg[n][j] )                        paper Eq. (6)
// x is the layer's hidden state [B][L][dm], dm = H D; Wg holds one row of dm weights per gate output:
// one per head (the paper's headwise gate) or a single one (the scalar gate of its gate ablation, Tab. 4).
// HBM-bound: x is read once (2 H flop per byte).  Computed transposed, G^T[h][l] = Wg x^T, so that both
// operands are read as rows; the H <= 32 heads occupy the rows of one 32 x 32 MFMA tile (rows >= H are
// zero).  One workgroup owns 32 tokens; its four wavefronts split dm and add their partial sums in LDS.
#include "arl2_device.h"

namespace arl2 {
namespace {

constexpr int NT = 256;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}

__global__ __launch_bounds__(NT) void gate_proj_kernel(GateArgs a)
{
    __shared__ float part[4][16][64];                    // [wavefront][register][lane]
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, hh = lane >> 5, c = lane & 31;
    const int dm = a.dm, H = a.n_out;                    // rows of Wg = gate outputs per token
    const long long tok0 = (long long)blockIdx.x * 32;   // first token (over streams and chunk positions)
    const long long ntok = (long long)a.B * a.L;

    const uint32_t x_bytes = (uint32_t)(ntok * dm * 2), w_bytes = (uint32_t)H * dm * 2;
    const __amdgpu_buffer_rsrc_t x_rsrc = make_rsrc(a.x, x_bytes);
    const __amdgpu_buffer_rsrc_t w_rsrc = make_rsrc(a.Wg, w_bytes);
    // lanes whose token or head does not exist read zeros
    const uint32_t x_row = tok0 + c < ntok ? (uint32_t)((tok0 + c) * dm * 2) : x_bytes;
    const uint32_t w_row = c < H ? (uint32_t)c * dm * 2 : w_bytes;

    // k-steps of 16 features, dealt to the wavefronts in contiguous quarters
    const int ksteps = dm / 16;
    const int t0 = ksteps * wave / 4, t1 = ksteps * (wave + 1) / 4;
    f32x16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    for (int t = t0; t < t1; ++t) {
        union { u32x4 u; bf16x8 v; } wa, xb;
        const uint32_t col = 32 * t + 16 * hh;
        wa.u = __builtin_amdgcn_raw_buffer_load_b128(w_rsrc, w_row < w_bytes ? w_row + col : w_bytes, 0, 0);
        xb.u = __builtin_amdgcn_raw_buffer_load_b128(x_rsrc, x_row < x_bytes ? x_row + col : x_bytes, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa.v, xb.v, acc, 0, 0, 0);
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) part[wave][r][lane] = acc[r];
    __syncthreads();
    // thread (register r, lane) of the first 1024 elements: head n = 8 (r / 4) + 4 hh + r % 4, token tok0 + c
    for (int i = tid; i < 16 * 64; i += NT) {
        const int r = i >> 6, ln = i & 63;
        const int n = 8 * (r >> 2) + 4 * (ln >> 5) + (r & 3);
        const long long tok = tok0 + (ln & 31);
        if (n < H && tok < ntok) {
            const float s = (part[0][r][ln] + part[1][r][ln]) + (part[2][r][ln] + part[3][r][ln]);
            const float g = 1.0f / (1.0f + __expf(-s));
            if (a.g_is_bf16) ((bf16_t *)a.g)[tok * H + n] = to_bf16(g);
            else ((float *)a.g)[tok * H + n] = g;
        }
    }
}

}  // namespace

hipError_t launch_gate_proj_bf16(const GateArgs &a, hipStream_t stream)
{
    const long long ntok = (long long)a.B * a.L;
    const long long nwg = (ntok + 31) / 32;
    if (nwg <= 0 || nwg > 0x7fffffffLL) return hipErrorInvalidValue;
    if (a.n_out < 1 || a.n_out > 32 || a.dm % 16 != 0) return hipErrorInvalidValue;
    // x is addressed with 32-bit byte offsets
    if (ntok * a.dm * 2 > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(gate_proj_kernel, dim3((unsigned)nwg), dim3(NT), 0, stream, a);
    return hipGetLastError();
}

}  // namespace arl2
