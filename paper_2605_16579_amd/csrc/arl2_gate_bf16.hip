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
//
// More than 32 gate outputs per token (the element-wise gate of the same ablation, one per feature: Wg is
// dm x dm) make the projection a dense matrix product and MFMA-bound: gate_dense_kernel below.
#include "arl2_device.h"

#include <type_traits>

namespace arl2 {
namespace {

constexpr int NT = 256;
constexpr int CW = 512;                  // columns of x per chunk
constexpr int XROW = 2 * CW + 16;        // LDS bytes per token row of a chunk (conflict-free 16-byte reads)
constexpr int XCH = 32 * (2 * CW / 16) / NT;   // 16-byte pieces of a chunk per thread

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

// ---- dense projection: G[tok][n] = sigmoid( sum_j x[tok][j] Wg[n][j] ) for any number of outputs n ----
// One workgroup owns TM tokens x TN outputs, each wavefront 64 tokens x TN / WN outputs (2 x NB MFMA
// blocks).  The hidden dimension is walked in steps of 64 columns: the 128-byte row pieces of x and Wg
// travel HBM/L2 -> registers -> LDS (padded rows: conflict-free 16-byte fragment reads), two LDS stages,
// two steps of loads in flight in two register sets, one LDS-only barrier per step so that the loads
// stay in flight across it.  With 2 x 2 blocks per wavefront every MFMA needs one 1 KB fragment from LDS
// and the LDS pipe is as busy as the matrix pipe; 2 x 4 blocks need 0.75.  Two shapes:
//   128 x 128, four wavefronts, two workgroups per CU    small problems: twice as many workgroups
//   256 x 256, eight wavefronts of 64 x 128              large problems: half the LDS and L2 traffic per flop
constexpr int GK = 64;                        // hidden columns per step
constexpr int GROW = 2 * GK + 16;             // LDS bytes per staged row piece

template <int TM, int TN, int NTH>
__global__ __launch_bounds__(NTH, 512 / NTH) void gate_dense_kernel(GateArgs a, int n_ntile)
{
    constexpr int WM = TM / 64, WN = NTH / 64 / WM;      // wavefronts along tokens, along outputs
    constexpr int NB = TN / WN / 32;                     // 32-output blocks per wavefront
    constexpr int PR = NTH / 8;                          // rows covered by one round of 16-byte pieces
    constexpr int XCHD = TM / PR, WCHD = TN / PR;        // pieces per thread and step: x, Wg
    constexpr int OROW = TN + 4;                         // floats per row of the output tile staged in LDS
    constexpr int STG = (TM + TN) * GROW;
    static_assert(WM * WN * 64 == NTH && NB * 32 * WN == TN && XCHD * PR == TM && WCHD * PR == TN, "tile shape");
    static_assert(32 * WM * OROW * 4 <= 2 * STG, "half of the output tile reuses the operand stages");
    __shared__ __attribute__((aligned(16))) unsigned char sm[2 * STG];   // [stage][x rows, Wg rows]
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, hh = lane >> 5, c = lane & 31;
    const int wm = wave % WM, wn = wave / WM;
    const int dm = a.dm, N = a.n_out;
    const long long ntok = (long long)a.B * a.L;
    // consecutive workgroups of an XCD share a token tile and walk over the outputs: x is fetched once
    const int work = xcd_contiguous_id(blockIdx.x, gridDim.x);
    const long long tok0 = (long long)(work / n_ntile) * TM;
    const int n0 = (work % n_ntile) * TN;

    const uint32_t x_bytes = (uint32_t)(ntok * dm * 2), w_bytes = (uint32_t)((long long)N * dm * 2);
    const __amdgpu_buffer_rsrc_t x_rsrc = make_rsrc(a.x, x_bytes);
    const __amdgpu_buffer_rsrc_t w_rsrc = make_rsrc(a.Wg, w_bytes);
    const int prow = tid >> 3, pcol = tid & 7;           // piece i of this thread: row prow + PR i, 16-byte column pcol
    const int nk = (dm + GK - 1) / GK;

    // byte offsets of this thread's pieces at step 0; rows past the end point past the buffer (reads return zero)
    uint32_t xoff[XCHD], woff[WCHD];
#pragma unroll
    for (int i = 0; i < XCHD; ++i) {
        const int row = prow + PR * i;
        xoff[i] = tok0 + row < ntok ? (uint32_t)((tok0 + row) * dm * 2 + 16 * pcol) : x_bytes;
    }
#pragma unroll
    for (int i = 0; i < WCHD; ++i) {
        const int row = prow + PR * i;
        woff[i] = n0 + row < N ? (uint32_t)((long long)(n0 + row) * dm * 2 + 16 * pcol) : w_bytes;
    }
    u32x4 xr[2][XCHD], wr[2][WCHD];
    auto fetch = [&](int kc, auto j_) __attribute__((always_inline)) {   // step kc into register set j; rows and columns past the end read zeros
        constexpr int j = decltype(j_)::value;
        const uint32_t colb = 2 * GK * kc;
        const bool okc = kc < nk && (int)colb + 16 * pcol < 2 * dm;
#pragma unroll
        for (int i = 0; i < XCHD; ++i)
            xr[j][i] = __builtin_amdgcn_raw_buffer_load_b128(x_rsrc, okc && xoff[i] != x_bytes ? xoff[i] + colb : x_bytes, 0, 0);
#pragma unroll
        for (int i = 0; i < WCHD; ++i)
            wr[j][i] = __builtin_amdgcn_raw_buffer_load_b128(w_rsrc, okc && woff[i] != w_bytes ? woff[i] + colb : w_bytes, 0, 0);
    };
    auto stage = [&](int st, auto j_) __attribute__((always_inline)) {
        constexpr int j = decltype(j_)::value;
        unsigned char *p = sm + st * STG + prow * GROW + 16 * pcol;
#pragma unroll
        for (int i = 0; i < XCHD; ++i) *(u32x4 *)(p + PR * i * GROW) = xr[j][i];
#pragma unroll
        for (int i = 0; i < WCHD; ++i) *(u32x4 *)(p + (TM + PR * i) * GROW) = wr[j][i];
    };
    f32x16 acc[2][NB];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    auto contract = [&](int st) __attribute__((always_inline)) {
        const unsigned char *xs = sm + st * STG + (64 * wm + c) * GROW + 16 * hh;
        const unsigned char *ws = sm + st * STG + (TM + 32 * NB * wn + c) * GROW + 16 * hh;
#pragma unroll
        for (int t = 0; t < GK / 16; ++t) {
            bf16x8 xa[2], wb[NB];
#pragma unroll
            for (int i = 0; i < 2; ++i) xa[i] = *(const bf16x8 *)(xs + 32 * i * GROW + 32 * t);
#pragma unroll
            for (int j = 0; j < NB; ++j) wb[j] = *(const bf16x8 *)(ws + 32 * j * GROW + 32 * t);
#pragma unroll
            for (int j = 0; j < NB; ++j)
#pragma unroll
                for (int i = 0; i < 2; ++i)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa[i], wb[j], acc[i][j], 0, 0, 0);
        }
    };

    const std::integral_constant<int, 0> J0{};
    const std::integral_constant<int, 1> J1{};
    // Step kc lives in register set kc % 2 and LDS stage kc % 2.  A step requests the loads of step kc + 2
    // first (its register set was staged in the previous step), contracts stage kc % 2 and then stages step
    // kc + 1, whose loads were requested a whole step earlier.
    fetch(0, J0);
    fetch(1, J1);
    stage(0, J0);
    lds_barrier();
    for (int kc = 0; kc < nk; kc += 2) {
        fetch(kc + 2, J0);
        contract(0);
        stage(1, J1);                 // step kc + 1 (zeros past the end); stage 1 was last read before the previous barrier
        lds_barrier();
        fetch(kc + 3, J1);
        if (kc + 1 < nk) contract(1);
        stage(0, J0);
        lds_barrier();
    }

    // Epilogue through LDS (free after the last barrier), one 32-token block of every wavefront at a time:
    // accumulator register r of block (i, j) is token 64 wm + 32 i + 8 (r / 4) + 4 hh + r % 4, output
    // 32 (NB wn + j) + c; the 32 WM staged rows are then read back by rows, 16 bytes of fp32 per lane, so
    // that a store instruction writes whole row pieces of up to 1 KB.
    float *ot = reinterpret_cast<float *>(sm);
    const bool vec = (N & 3) == 0 && (reinterpret_cast<uintptr_t>(a.g) & 15) == 0;   // every row of g starts 16-byte (bf16: 8-byte) aligned
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        if (i) lds_barrier();                            // the first block has been read back
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                ot[(32 * wm + 8 * (r >> 2) + 4 * hh + (r & 3)) * OROW + 32 * (NB * wn + j) + c] = acc[i][j][r];
        lds_barrier();
#pragma unroll 4
        for (int id = tid; id < 32 * WM * (TN / 4); id += NTH) {
            const int row = id / (TN / 4), col = 4 * (id % (TN / 4)), n = n0 + col;
            const long long tok = tok0 + 64 * (row >> 5) + 32 * i + (row & 31);
            if (tok >= ntok || n >= N) continue;
            f32x4 s = *(const f32x4 *)(ot + row * OROW + col);
#pragma unroll
            for (int e = 0; e < 4; ++e) s[e] = 1.0f / (1.0f + __expf(-s[e]));
            if (vec) {
                if (a.g_is_bf16) {
                    bf16x4 o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = to_bf16(s[e]);
                    *(bf16x4 *)((bf16_t *)a.g + tok * N + n) = o;
                } else {
                    *(f32x4 *)((float *)a.g + tok * N + n) = s;
                }
            } else {
                for (int e = 0; e < 4 && n + e < N; ++e) {
                    if (a.g_is_bf16) ((bf16_t *)a.g)[tok * N + n + e] = to_bf16(s[e]);
                    else ((float *)a.g)[tok * N + n + e] = s[e];
                }
            }
        }
    }
}

template <int TM, int TN, int NTH>
hipError_t launch_gate_dense(const GateArgs &a, long long ntok, hipStream_t stream)
{
    const long long n_ntile = (a.n_out + TN - 1) / TN, n_mtile = (ntok + TM - 1) / TM;
    if (n_mtile * n_ntile > 0x7fffffffLL) return hipErrorInvalidValue;
    return launch_kernel(gate_dense_kernel<TM, TN, NTH>, dim3((unsigned)(n_mtile * n_ntile)), dim3(NTH), stream, a, (int)n_ntile);
}

}  // namespace

hipError_t launch_gate_proj_bf16(const GateArgs &a, hipStream_t stream)
{
    const long long ntok = (long long)a.B * a.L;
    const long long nwg = (ntok + 31) / 32;
    if (nwg <= 0 || nwg > 0x7fffffffLL) return hipErrorInvalidValue;
    if (a.n_out < 1 || a.dm % 16 != 0) return hipErrorInvalidValue;
    // x and Wg are addressed with 32-bit byte offsets
    if (ntok * a.dm * 2 > 0x7fffffffLL || (long long)a.n_out * a.dm * 2 > 0x7fffffffLL) return hipErrorInvalidValue;
    if (a.n_out > 32) {
        // the large tiles once they fill the chip at least twice
        const long long big = ((ntok + 255) / 256) * ((a.n_out + 255) / 256);
        return big >= 2 * kNumCu ? launch_gate_dense<256, 256, 512>(a, ntok, stream) : launch_gate_dense<128, 128, 256>(a, ntok, stream);
    }
    return launch_kernel(gate_proj_kernel, dim3((unsigned)nwg), dim3(NT), stream, a);
}

}  // namespace arl2
