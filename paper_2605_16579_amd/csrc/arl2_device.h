// Internal declarations shared by the gfx950 kernels of the ARL^2 hybrid attention library.
// Not part of the public interface (that is include/arl2.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <tuple>
#include <type_traits>
#include <utility>

namespace arl2 {

typedef __bf16 bf16_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

// MI355X has 8 accelerator dies (XCDs), each with its own L2; the hardware deals
// consecutive workgroup ids to the XCDs round-robin.
constexpr int kNumXcd = 8;
constexpr int kNumCu = 256;
constexpr int kWave = 64;

template <class Tuple, size_t... I>
inline void fill_arg_pointers(void **ptrs, Tuple &vals, std::index_sequence<I...>)
{
    ((ptrs[I] = (void *)&std::get<I>(vals)), ...);
}

struct FwdArgs {
    const void *q, *k, *v;
    const void *q_lin;     // row the linear branch normalises; nullptr: q itself
    // or, fused: q_lin = RoPE(Wq[h] xq) computed in the kernel (all nullptr when not used)
    const void *xq;        // [B][Lq][H][D] bf16, the projection the feature map acts on
    const void *Wq;        // [H][D][D] bf16, [head][out][in]
    const float *cs, *sn;  // [Lq][D/2] rotation tables, or both nullptr
    const float *S;        // may be nullptr
    const void *g;         // may be nullptr
    void *out;
    int B, H, Lq, Lkv, D;
    int g_is_bf16;
    int g_per_element;     // g is [B][Lq][H][D] instead of [B][Lq][H]
    int g_per_token;       // g is [B][Lq]: one gate per token, shared by the heads
    float sm_scale;        // already resolved (never 0)
    float l2_eps;          // already resolved
};

struct CommitArgs {
    const void *k, *v;
    const float *gate;     // forget gate alpha
    const float *beta;     // nullptr: plain commit; else the delta rule's learning rate
    float *S;
    void *workspace;
    int B, H, L, D;
    int nsplit;            // token splits per (stream, head) for the bf16 path
    float l2_eps;
};

struct CommitFmArgs {
    const void *xk, *xv;   // [B][L][H][D] bf16, the projections the key and value maps act on
    const void *Wk, *Wv;   // [H][D][D] bf16, [head][out][in]
    const float *cs, *sn;  // [L][D/2] rotation tables of the key map, or both nullptr
    const float *gate;
    float *S;
    void *workspace;
    int B, H, L, D;
    int nsplit;
    float l2_eps;
};

struct FmapArgs {
    const void *x;         // [B][L][H][D] bf16
    const void *W;         // [H][D][D] bf16, indexed [head][out][in]
    const float *cs, *sn;  // [L][D/2] cosines and sines of the rotation, or both nullptr
    void *y;               // [B][L][H][D] bf16
    int B, H, L, D;
};

struct GateArgs {
    const void *x;         // [B][L][dm] bf16, dm = H * D
    const void *Wg;        // [n_out][dm] bf16
    void *g;               // [B][L][n_out], fp32 or bf16
    int B, H, L, dm;
    int n_out;             // gate outputs per token: H (headwise), 1 (scalar) or H * D (element-wise)
    int g_is_bf16;
};

struct GdnArgs {
    const void *k, *v;
    const float *alpha;    // per-token forget gate  [B][L][H]
    const float *beta;     // per-token learning rate [B][L][H]
    float *S;
    void *workspace;
    int B, H, L, D;
    float l2_eps;
};

// Token splits used by the bf16 commit for a problem size (also sizes the workspace).
int commit_nsplit(int B, int H, int L);

// Launchers: enqueue on `stream`, return the HIP error of the launch.
hipError_t launch_fwd_bf16(const FwdArgs &a, hipStream_t stream);
hipError_t launch_fwd_f32(const FwdArgs &a, hipStream_t stream);
hipError_t launch_commit_bf16(const CommitArgs &a, hipStream_t stream);
hipError_t launch_commit_f32(const CommitArgs &a, hipStream_t stream);
hipError_t launch_commit_fm_bf16(const CommitFmArgs &a, hipStream_t stream);
// S = gate * S + the token-split partial sums in a.workspace ([B*H][nsplit][D][D] fp32), added in split order.
hipError_t launch_commit_reduce_bf16(const CommitArgs &a, hipStream_t stream);
hipError_t launch_commit_gdn_bf16(const GdnArgs &a, hipStream_t stream);
hipError_t launch_feature_map_bf16(const FmapArgs &a, hipStream_t stream);
hipError_t launch_gate_proj_bf16(const GateArgs &a, hipStream_t stream);

// Workspace of the token-sequential commit (per-block transition maps).
size_t gdn_workspace_bytes(int B, int H, int L, int D);

// ---- launching ------------------------------------------------------------------------
// Enqueues `kernel` and returns the status of this launch alone (an error that an earlier, unrelated HIP call
// of the caller left behind is neither reported nor cleared).
template <class... Params, class... Args>
inline hipError_t launch_kernel(void (*kernel)(Params...), dim3 grid, dim3 block, hipStream_t stream, Args... args)
{
    std::tuple<Params...> vals{static_cast<Params>(args)...};
    void *ptrs[sizeof...(Params) > 0 ? sizeof...(Params) : 1];
    fill_arg_pointers(ptrs, vals, std::index_sequence_for<Params...>{});
    return hipLaunchKernel(reinterpret_cast<const void *>(kernel), grid, block, ptrs, 0, stream);
}

// ---- small device helpers -------------------------------------------------------------

// Raw buffer descriptor over [base, base + bytes): loads beyond the range return zero, stores are dropped.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}

// Compile-time loop: f(integral_constant<int, I>) for I = First .. N - 1.
template <int I, int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// Transposing LDS read (ds_read_b64_tr_b16): within each group of 16 lanes, lane i receives element i of the
// four 16-element rows whose 8-byte pieces are addressed by lanes 4j..4j+3 (j = 0..3).
typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;
__device__ __forceinline__ bf16x4 lds_read_tr(const unsigned char *p)
{
    return __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4 *)(p));
}
// Two such reads, `second_row_bytes` apart, as one 8-element MFMA operand fragment.
__device__ __forceinline__ bf16x8 lds_read_tr_pair(const unsigned char *p, int second_row_bytes)
{
    return __builtin_shufflevector(lds_read_tr(p), lds_read_tr(p + second_row_bytes), 0, 1, 2, 3, 4, 5, 6, 7);
}

// Sum / max of a value held by lane l and lane l^32 (the two half-waves).
__device__ __forceinline__ float xhalf_sum(float x)
{
    return x + __shfl_xor(x, 32, kWave);
}
__device__ __forceinline__ float xhalf_max(float x)
{
    return fmaxf(x, __shfl_xor(x, 32, kWave));
}

// Sum over aligned groups of N = 8 or 16 consecutive lanes, every lane of the group receiving it, in
// data-parallel-primitive adds (no LDS crossbar): pairs and quads by quad permutation, then the other
// quad of the 8 (row_half_mirror) and the other half of the 16 (row_mirror), whose lanes already agree.
template <int CTRL>
__device__ __forceinline__ float dpp_peek(float x)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true));
}
template <int N>
__device__ __forceinline__ float lane_group_sum(float x)
{
    static_assert(N == 8 || N == 16, "groups of 8 or 16 lanes");
    x += dpp_peek<0xB1>(x);                  // quad_perm [1,0,3,2]
    x += dpp_peek<0x4E>(x);                  // quad_perm [2,3,0,1]
    x += dpp_peek<0x141>(x);                 // row_half_mirror
    if constexpr (N == 16) x += dpp_peek<0x140>(x);   // row_mirror
    return x;
}

// Workgroup barrier that orders LDS traffic only: global loads and stores issued before it stay in
// flight (__syncthreads would first wait for all of them to complete, which cancels a register prefetch
// that runs several tiles ahead).
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Workgroup barrier that waits only until at most N of this wavefront's LDS operations are outstanding:
// LDS operations complete in order, so everything issued before the last N is done (writes published),
// while the last N (reads of data that stays valid) remain in flight across the barrier.
template <int N>
__device__ __forceinline__ void lds_barrier_keep()
{
    static_assert(N >= 0 && N <= 15, "lgkmcnt is a 4-bit counter");
    asm volatile("s_waitcnt lgkmcnt(%0)\n\ts_barrier" ::"n"(N) : "memory");
}

// 1 / sqrt(x) in one hardware instruction (about 1 ulp); x > 0.
__device__ __forceinline__ float fast_rsqrt(float x) { return __builtin_amdgcn_rsqf(x); }

// x as the sum of two bf16 values: hi is x truncated to bf16 (exact bit mask), lo the rounded remainder;
// the remainder of a truncation has at most 16 significant bits, so hi + lo misses x by 2^-16 |x| at most.
// Returns hi and lo as the upper halves of two 32-bit words (bf16 bit patterns).
__device__ __forceinline__ void split_bf16_trunc(float x, uint32_t &hi_bits, float &lo)
{
    hi_bits = __float_as_uint(x) & 0xffff0000u;
    lo = x - __uint_as_float(hi_bits);
}

// Round-to-nearest-even fp32 -> bf16 (hardware conversion on gfx950).
__device__ __forceinline__ bf16_t to_bf16(float x) { return (bf16_t)x; }

// Map the hardware workgroup id to a logical work index such that consecutive logical
// indices run on the same XCD (and so share that XCD's L2).
__device__ __forceinline__ int xcd_contiguous_id(int id, int n)
{
    const int per = n / kNumXcd, rem = n % kNumXcd;
    const int x = id % kNumXcd, loc = id / kNumXcd;
    return x * per + (x < rem ? x : rem) + loc;
}

}  // namespace arl2
