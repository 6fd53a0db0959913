/*
 * arl2.h -- C ABI of the MI355X (gfx950) library for the ARL^2 hybrid attention step
 * of "Attend Locally, Remember Linearly" (paper Sec. 3.2, Sec. 3.3, Alg. 1).
 *
 * Two operations make up the step:
 *
 *   arl2_hybrid_attn_fwd   one read-only denoising pass:
 *                            out = softmax(q k^T * sm_scale) v  +  g * L2Norm(q) S
 *                          (intra-chunk softmax branch Eq. (2); feature map Eq. (3);
 *                           linear readout of the shared pre-update state Eq. (5), (7);
 *                           headwise gate broadcast over the head dimension Eq. (6)).
 *                          S is never written by this call (Sec. 3.3, clean-pass update).
 *
 *   arl2_state_commit      once per chunk, after the last denoising pass:
 *                            S <- gate * S + sum_i L2Norm(k_i)^T v_i
 *                          (Eq. (4) with beta = 1 and without the delta-correction term;
 *                           the gate multiplies the old state only).
 *
 *   arl2_state_commit_delta the same update with Eq. (4)'s delta-correction term and learning rate.
 *
 *   arl2_state_commit_gdn  Eq. (4) applied token by token in order, with per-token gates.
 *
 *   arl2_feature_map       the learned per-head maps and RoPE of Eq. (3) for the linear branch;
 *   arl2_hybrid_attn_fwd_ex  the readout pass with the linear branch's own query;
 *   arl2_hybrid_attn_fwd_fm  the readout pass that computes that query itself (fused feature map);
 *   arl2_gate_proj         the gate G = sigmoid(x W_g) of Eq. (6): headwise, one per token or element-wise.
 *
 * Reading of the feature map: q and k arrive after RoPE, the learned 1x1 maps are
 * the identity, so phi is the L2 normalisation over the head dimension,
 * x / sqrt(sum x^2 + l2_eps), and V' = v.
 *
 * All data pointers are DEVICE pointers owned by the caller, 16-byte aligned and
 * contiguous in the layouts below.  The library never allocates, frees or
 * synchronises: every call validates its arguments on the host (sizes, alignment, overlapping
 * buffers, limits of the kernels), enqueues its kernels on desc->stream and returns.  A call that
 * returns ARL2_ERR_INVALID_ARG, ARL2_ERR_UNSUPPORTED or ARL2_ERR_WORKSPACE has launched nothing.
 * ARL2_ERR_DEVICE reports that the runtime refused a launch: a call made of several kernels
 * (the state commits) may then have enqueued the earlier ones, and S is undefined.
 * The kernels address one stream's k, v (the whole x for arl2_feature_map and arl2_gate_proj) with
 * 32-bit byte offsets: such an array must stay below 2 GiB, larger problems return ARL2_ERR_UNSUPPORTED.
 *
 * Layouts (row-major):
 *   q, out      [B][Lq ][H][D]   io_dtype
 *   k, v        [B][Lkv][H][D]   io_dtype
 *   g           [B][Lq ][H]      g_dtype, values in [0,1]      (branch-mix gate, Eq. (6); other
 *                                granularities: see arl2_gate_mode)
 *   S           [B][H][D][D]     fp32, S[d_k][d_v]; readout contracts d_k
 *   gate        [B][H]           fp32                          (forget gate alpha, Eq. (4))
 */
#ifndef ARL2_H
#define ARL2_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ARL2_OK = 0,
    ARL2_ERR_INVALID_ARG = 1,   /* NULL/misaligned pointer, non-positive size, bad enum    */
    ARL2_ERR_UNSUPPORTED = 2,   /* valid request outside what the kernels implement        */
    ARL2_ERR_WORKSPACE = 3,     /* workspace missing or smaller than arl2_workspace_bytes  */
    ARL2_ERR_DEVICE = 4         /* a HIP launch failed; see arl2_last_error()              */
} arl2_status;

typedef enum { ARL2_F32 = 0, ARL2_BF16 = 1 } arl2_dtype;

/* Granularity of the branch-mix gate g of the readout pass.  The paper's gate is headwise (Eq. (6),
 * g of shape [B][Lq][H]); its gate ablation (Tab. 4) also has one gate per output feature
 * (ARL2_GATE_PER_ELEMENT, g of shape [B][Lq][H][D], 16-byte aligned) and a scalar gate, one per token
 * shared by the heads (ARL2_GATE_PER_TOKEN, g of shape [B][Lq]). */
typedef enum { ARL2_GATE_PER_HEAD = 0, ARL2_GATE_PER_ELEMENT = 1, ARL2_GATE_PER_TOKEN = 2 } arl2_gate_mode;

typedef struct {
    int32_t B;            /* independent streams, >= 1                                      */
    int32_t H;            /* heads, >= 1                                                    */
    int32_t Lq;           /* query tokens of the chunk, >= 1                                */
    int32_t Lkv;          /* key/value tokens; must equal Lq when S != NULL or in commit.   */
                          /* Lkv != Lq (any value >= 1) is allowed for pure softmax, S NULL */
    int32_t D;            /* head dimension d_k = d_v: 64 or 128                            */
    int32_t io_dtype;     /* arl2_dtype of q, k, v, out                                     */
    int32_t g_dtype;      /* arl2_dtype of g (ignored when g == NULL)                       */
    float sm_scale;       /* softmax logit scale; 0 selects 1/sqrt(D)   (Eq. (1))           */
    float l2_eps;         /* epsilon inside L2Norm's square root; 0 selects 1e-6            */
    int32_t g_mode;       /* arl2_gate_mode of g; 0 (zero-initialised descriptor) is headwise */
    void *workspace;      /* device scratch for arl2_state_commit, >= arl2_workspace_bytes  */
    size_t workspace_bytes;
    void *stream;         /* hipStream_t; NULL is the default stream                        */
} arl2_desc;

/* Device scratch that arl2_state_commit / arl2_state_commit_delta need for this descriptor
 * (token-split partial sums, state snapshot).  arl2_hybrid_attn_fwd needs none.  Returns 0 for
 * an invalid descriptor.                                                                     */
size_t arl2_workspace_bytes(const arl2_desc *desc);

/*
 * Read-only denoising pass (paper Eq. (2), (3), (5), (6), (7); Alg. 1 inner loop).
 *   q, k, v   device, io_dtype, layouts above; not modified.
 *   S         device fp32 [B][H][D][D], READ-ONLY; NULL means a zero state (pure softmax,
 *             used for layers that keep softmax over a KV cache, Eq. (1) with every cached
 *             token visible).
 *   g         device [B][Lq][H]; NULL means a gate of one.
 *   out       device, io_dtype [B][Lq][H][D]; fully overwritten; must not alias an input.
 * bf16 I/O runs on bf16 MFMA with fp32 accumulation and fp32 softmax statistics;
 * fp32 I/O runs in fp32 throughout.
 */
arl2_status arl2_hybrid_attn_fwd(const arl2_desc *desc,
                                 const void *q, const void *k, const void *v,
                                 const float *S, const void *g, void *out);

/*
 * The same pass with a query of its own for the linear branch (paper Eq. (3), (5)): the inter branch
 * normalises and multiplies with S the rows of q_lin, e.g. RoPE(phi_q(Q)) written by arl2_feature_map,
 * while the softmax branch keeps q (Eq. (2)).
 *   q_lin     device, io_dtype [B][Lq][H][D]; NULL means q (then this is arl2_hybrid_attn_fwd).
 *             Not read when S is NULL.
 */
arl2_status arl2_hybrid_attn_fwd_ex(const arl2_desc *desc,
                                    const void *q, const void *k, const void *v, const void *q_lin,
                                    const float *S, const void *g, void *out);

/*
 * The readout pass with the query feature map of the linear branch fused in (paper Eq. (2), (3), (5),
 * (6)): the inter branch reads L2Norm(RoPE(Wq[h] xq)), computed inside the kernel and never stored;
 * equal to arl2_feature_map(xq, Wq, ...) followed by arl2_hybrid_attn_fwd_ex, without the intermediate
 * array and the second launch.
 *   q, k, v   as in arl2_hybrid_attn_fwd (the softmax branch's inputs), bf16 only.
 *   xq        device bf16 [B][Lq][H][D]: the projection the feature map acts on (before RoPE).
 *   Wq, rope_cos, rope_sin   as in arl2_feature_map.
 *   S         device fp32 [B][H][D][D], READ-ONLY, must not be NULL (without a state there is no
 *             linear branch: use arl2_hybrid_attn_fwd).
 */
arl2_status arl2_hybrid_attn_fwd_fm(const arl2_desc *desc,
                                    const void *q, const void *k, const void *v,
                                    const void *xq, const void *Wq,
                                    const float *rope_cos, const float *rope_sin,
                                    const float *S, const void *g, void *out);

/*
 * Per-head feature map of the linear branch, paper Eq. (3) without its L2Norm (the readout and the
 * commits normalise the rows they are given):
 *     y[b][l][h][:] = RoPE_l( W[h] x[b][l][h][:] )
 *   x         device bf16 [B][Lq][H][D] (desc->io_dtype must be ARL2_BF16; Lkv is not used).
 *   W         device bf16 [H][D][D], per head the D x D matrix of the grouped 1 x 1 map, indexed
 *             [head][out][in].
 *   rope_cos, rope_sin   device fp32 [Lq][D/2], 8-byte aligned: cosine and sine of the angle by which
 *             the pair (y[2i], y[2i+1]) of token l is rotated, shared by all streams and heads; which
 *             positions and frequencies they encode is the caller's choice.  Both NULL: no rotation
 *             (the value map phi_v).
 *   y         device bf16 [B][Lq][H][D], fully overwritten; must not alias x or W.
 * fp32 accumulation and rotation, one rounding to bf16 on output.
 */
arl2_status arl2_feature_map(const arl2_desc *desc, const void *x, const void *W,
                             const float *rope_cos, const float *rope_sin, void *y);

/*
 * Branch-mix gate, paper Eq. (6): G = sigmoid(x W_g), the g argument of the readout pass.
 *   x         device bf16 [B][Lq][H*D], the layer's hidden state (desc->io_dtype must be ARL2_BF16).
 *   Wg        device bf16 [n][H*D], one row per gate output: n = H for desc->g_mode == ARL2_GATE_PER_HEAD
 *             (row h is column h of the paper's (H*D) x H matrix W_g), n = 1 for ARL2_GATE_PER_TOKEN and
 *             n = H*D for ARL2_GATE_PER_ELEMENT (the scalar and the element-wise gate of the paper's gate
 *             ablation, Tab. 4; row h*D + e is the gate of feature e of head h).  Below 2 GiB.
 *   g         device [B][Lq][n] in desc->g_dtype ([B][Lq][H][D] element-wise), fully overwritten; must
 *             not alias an input.
 * fp32 accumulation and sigmoid.  Up to 32 outputs per token the call is bound by reading x once; beyond
 * that it is a dense matrix product on the matrix cores.
 */
arl2_status arl2_gate_proj(const arl2_desc *desc, const void *x, const void *Wg, void *g);

/*
 * Post-denoise state update (paper Eq. (3), Eq. (4); Alg. 1 clean pass).
 *   k, v      device, io_dtype [B][Lq][H][D] of the clean pass (desc->Lkv must equal Lq).
 *   gate      device fp32 [B][H].
 *   S         device fp32 [B][H][D][D], updated IN PLACE.
 * The token-split partial sums are reduced in a fixed order: results are bit-identical
 * from run to run.  Uses desc->workspace.
 */
arl2_status arl2_state_commit(const arl2_desc *desc,
                              const void *k, const void *v,
                              const float *gate, float *S);

/*
 * arl2_state_commit for callers that can neither allocate device memory nor bring a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels
 * and bit-identical results; desc->workspace and desc->workspace_bytes are ignored, the token-split
 * partial sums go to a fixed array in device memory that the library holds on every GPU it runs on
 * (arl2_static_scratch_bytes(), 16 MiB).  A problem that needs more returns ARL2_ERR_UNSUPPORTED
 * (bf16: B * H * splits * D * D * 4 bytes, 12 MiB at B = 1, H = 12, Lq = 4680, D = 128; fp32: B * Lq * H * 4
 * bytes).  The call allocates and frees nothing and does not synchronise.  All calls on one GPU share that
 * GPU's array: two calls that overlap in time on one GPU (different streams, or threads) race; calls on
 * one stream, or ordered by events, do not.  Nothing in the array has to survive between calls or to be
 * cleared: every call writes each partial sum before it reads it.
 */
size_t arl2_static_scratch_bytes(void);
arl2_status arl2_state_commit_static(const arl2_desc *desc,
                                     const void *k, const void *v,
                                     const float *gate, float *S);

/*
 * arl2_state_commit with the key and value feature maps of the linear branch fused in (paper Eq. (3),
 * Eq. (4); Alg. 1 clean pass):
 *     S <- gate * S + sum_i L2Norm(RoPE_i(Wk[h] xk_i))^T (Wv[h] xv_i)
 * equal to arl2_feature_map(xk, Wk, rope_cos, rope_sin), arl2_feature_map(xv, Wv, NULL, NULL) and
 * arl2_state_commit on their outputs, without the two intermediate arrays and their launches.  The mapped
 * key is rounded to bf16 once, as arl2_feature_map would store it, and normalised as rounded; the mapped
 * value stays in fp32 until it is scaled by the key's inverse norm (it is not rounded to bf16 on its own,
 * so the result is closer to exact arithmetic than the three calls, not bit-identical to them).
 *   xk, xv    device bf16 [B][Lq][H][D]: the clean pass's projections the maps act on (desc->io_dtype must
 *             be ARL2_BF16, desc->Lkv must equal Lq).
 *   Wk, Wv    device bf16 [H][D][D], indexed [head][out][in], as in arl2_feature_map.
 *   rope_cos, rope_sin   device fp32 [Lq][D/2], 8-byte aligned: the key map's rotation, as in
 *             arl2_feature_map; both NULL: no rotation.  The value map is never rotated.
 *   gate      device fp32 [B][H].
 *   S         device fp32 [B][H][D][D], updated IN PLACE.
 * Deterministic.  Uses desc->workspace (arl2_workspace_bytes covers it).
 */
arl2_status arl2_state_commit_fm(const arl2_desc *desc,
                                 const void *xk, const void *Wk,
                                 const float *rope_cos, const float *rope_sin,
                                 const void *xv, const void *Wv,
                                 const float *gate, float *S);

/*
 * Post-denoise state update with the delta-correction term: paper Eq. (4) taken literally at
 * frame level,
 *     S <- alpha * S + beta * K'^T (V - K' S),      K' = L2Norm(k) per token (Eq. (3)),
 * every token's correction using the same pre-update S (frame-level access, Sec. 3.3).
 *   k, v      device bf16 [B][Lq][H][D] of the clean pass (desc->io_dtype must be ARL2_BF16,
 *             desc->Lkv must equal Lq); fp32 inputs return ARL2_ERR_UNSUPPORTED.
 *   gate      device fp32 [B][H], the forget gate alpha.
 *   beta      device fp32 [B][H], the learning rate.  With all L tokens written at once the update
 *             is a contraction only for beta below about 2 D / L; that is the caller's choice.
 *   S         device fp32 [B][H][D][D], updated IN PLACE.
 * Deterministic like arl2_state_commit.  Uses desc->workspace (arl2_workspace_bytes covers it).
 */
arl2_status arl2_state_commit_delta(const arl2_desc *desc,
                                    const void *k, const void *v,
                                    const float *gate, const float *beta, float *S);

/*
 * Token-sequential gated delta rule: paper Eq. (4) applied to one token at a time, in token order,
 * with per-token gates (Sec. 3.2, remark after Eq. (4); Alg. 1, clean pass).  For j = 1..Lq
 *     S <- alpha_j * S + beta_j * k'_j^T (v_j - k'_j S),      k'_j = L2Norm(k_j)  (Eq. (3)),
 * the correction of token j reading the state as token j-1 left it.
 *   k, v      device bf16 [B][Lq][H][D] of the clean pass (desc->io_dtype must be ARL2_BF16,
 *             desc->Lkv must equal Lq); fp32 inputs return ARL2_ERR_UNSUPPORTED.
 *   alpha     device fp32 [B][Lq][H], per-token forget gates.
 *   beta      device fp32 [B][Lq][H], per-token learning rates; each step is a contraction for
 *             0 <= beta_j <= 1 and 0 <= alpha_j <= 1.
 *   S         device fp32 [B][H][D][D], updated IN PLACE.
 * desc->workspace must hold arl2_gdn_workspace_bytes(desc) bytes (per block of 64 tokens and head the
 * operands of its transition, 65 KiB at D = 128, plus up to 7 composed D x D maps of 128 KiB per head).
 * Deterministic.
 */
size_t arl2_gdn_workspace_bytes(const arl2_desc *desc);
arl2_status arl2_state_commit_gdn(const arl2_desc *desc,
                                  const void *k, const void *v,
                                  const float *alpha, const float *beta, float *S);

const char *arl2_status_string(arl2_status s);

/* Thread-local detail of the last call that failed on this thread ("" if none has failed yet); a later
 * successful call does not clear it: read it right after a call that returned an error. */
const char *arl2_last_error(void);

/* Library version, major * 10000 + minor * 100 + patch. */
int arl2_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ARL2_H */
