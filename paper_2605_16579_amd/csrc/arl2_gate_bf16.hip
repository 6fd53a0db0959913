// Branch-mix gate on bf16 MFMA (gfx950):
//   G[b][l][n] = sigmoid( sum_j x[b][l][j] Wg[n][j] )                        paper Eq. (6)
// x is the layer's hidden state [B][L][dm], dm = H D; Wg holds one row of dm weights per gate output:
// one per head (the paper's headwise gate) or a single one (the scalar gate of its gate ablation, Tab. 4).
// HBM-bound: x is read once (2 H flop per byte).  Computed transposed, G^T[h][l] = Wg x^T, so that both
// operands are read as rows; the H <= 32 heads occupy the rows of one 32 x 32 MFMA tile (rows >= H are
// zero).  One workgroup owns 32 tokens and walks the hidden dimension in chunks of 512 columns: the chunk
// of x travels HBM -> registers -> LDS as whole 1 KB row pieces (fragment loads straight from global
// memory touch 32 cache lines per instruction and made the kernel request-bound), two LDS buffers, the
// next chunk in flight while the four wavefronts each contract a quarter of the current one; their
// partial sums are added in LDS.
#include "arl2_device.h"

#include <type_traits>

namespace arl2 {
namespace {

constexpr int NT = 256;
constexpr int CW = 512;                  // columns of x per chunk
constexpr int XROW = 2 * CW + 16;        // LDS bytes per token row of a chunk (conflict-free 16-byte reads)
constexpr int XCH = 32 * (2 * CW / 16) / NT;   // 16-byte pieces of a chunk per thread

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}

__global__ __launch_bounds__(NT) void gate_proj_kernel(GateArgs a)
{
    __shared__ __attribute__((aligned(16))) unsigned char xs[2][32 * XROW];
    static_assert(sizeof(float) * 4 * 16 * 64 <= 32 * XROW, "the partial sums reuse the first chunk buffer");
    float (*part)[16][64] = reinterpret_cast<float (*)[16][64]>(&xs[0][0]);   // [wavefront][register][lane], after the last chunk
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, hh = lane >> 5, c = lane & 31;
    const int dm = a.dm, H = a.n_out;                    // rows of Wg = gate outputs per token
    const long long tok0 = (long long)blockIdx.x * 32;   // first token (over streams and chunk positions)
    const long long ntok = (long long)a.B * a.L;

    const uint32_t x_bytes = (uint32_t)(ntok * dm * 2), w_bytes = (uint32_t)H * dm * 2;
    const __amdgpu_buffer_rsrc_t x_rsrc = make_rsrc(a.x, x_bytes);
    const __amdgpu_buffer_rsrc_t w_rsrc = make_rsrc(a.Wg, w_bytes);
    // lanes whose head does not exist read zeros
    const uint32_t w_row = c < H ? (uint32_t)c * dm * 2 : w_bytes;

    // piece i of this thread in a chunk: token row (tid + NT i) / 64, 16-byte column (tid + NT i) % 64
    const int nchunk = (dm + CW - 1) / CW;
    // Three chunks are requested at once (one memory latency for 1536 columns, the hidden size of the
    // paper's model), then staged and contracted one after the other.
    constexpr int GRP = 3;
    u32x4 xr[GRP][XCH];
    auto fetch = [&](int ch, auto j_) {                  // chunk ch of the 32 token rows into register set j
        constexpr int j = decltype(j_)::value;
#pragma unroll
        for (int i = 0; i < XCH; ++i) {
            const int id = tid + NT * i, row = id / (2 * CW / 16), col = id % (2 * CW / 16);
            const int colb = 2 * CW * ch + 16 * col;                       // byte column in the row of x
            const bool ok = tok0 + row < ntok && colb < 2 * dm;
            xr[j][i] = __builtin_amdgcn_raw_buffer_load_b128(x_rsrc, ok ? (uint32_t)((tok0 + row) * dm * 2 + colb) : x_bytes, 0, 0);
        }
    };
    f32x16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    constexpr int KS = CW / 16 / 4;                      // k-steps of a chunk per wavefront
    auto contract = [&](int ch, auto j_) {               // stage register set j as chunk ch, then this wavefront's quarter of it
        constexpr int j = decltype(j_)::value;
        unsigned char *buf = xs[ch & 1];
#pragma unroll
        for (int i = 0; i < XCH; ++i) {
            const int id = tid + NT * i, row = id / (2 * CW / 16), col = id % (2 * CW / 16);
            *(u32x4 *)(buf + row * XROW + 16 * col) = xr[j][i];
        }
        // A = Wg rows from global memory (few rows, L2-resident)
        union { u32x4 u; bf16x8 v; } wa[KS];
#pragma unroll
        for (int i = 0; i < KS; ++i) {
            const uint32_t colb = 2 * CW * ch + 32 * (KS * wave + i) + 16 * hh;
            wa[i].u = __builtin_amdgcn_raw_buffer_load_b128(w_rsrc, (w_row < w_bytes && colb < (uint32_t)(2 * dm)) ? w_row + colb : w_bytes, 0, 0);
        }
        __syncthreads();                                 // the chunk is in LDS (the other buffer was last read a barrier ago)
#pragma unroll
        for (int i = 0; i < KS; ++i) {
            const bf16x8 xb = *(const bf16x8 *)(buf + c * XROW + 32 * (KS * wave + i) + 16 * hh);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa[i].v, xb, acc, 0, 0, 0);
        }
    };
    const std::integral_constant<int, 0> J0{};
    const std::integral_constant<int, 1> J1{};
    const std::integral_constant<int, 2> J2{};
    for (int ch = 0; ch < nchunk; ch += GRP) {           // chunks past the last one read zeros and are skipped
        fetch(ch, J0);
        if (ch + 1 < nchunk) fetch(ch + 1, J1);
        if (ch + 2 < nchunk) fetch(ch + 2, J2);
        contract(ch, J0);
        if (ch + 1 < nchunk) contract(ch + 1, J1);
        if (ch + 2 < nchunk) contract(ch + 2, J2);
    }
    __syncthreads();                                     // every wavefront has read its last chunk
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
