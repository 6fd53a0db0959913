// Host side of the C ABI declared in include/arl2.h: argument validation, dispatch to the
// gfx950 kernels, error reporting.  Nothing here allocates device memory or synchronises.
#include "../../include/arl2.h"
#include "arl2_device.h"

#include <atomic>
#include <cstdio>
#include <cstring>

namespace {

thread_local char g_err[256] = "";

arl2_status fail(arl2_status s, const char *fmt, const char *detail = "")
{
    std::snprintf(g_err, sizeof(g_err), fmt, detail);
    return s;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Do the byte ranges [a, a + na) and [b, b + nb) share a byte?  (NULL pointers overlap nothing.)
bool overlaps(const void *a, size_t na, const void *b, size_t nb)
{
    if (a == nullptr || b == nullptr || na == 0 || nb == 0) return false;
    const uintptr_t pa = reinterpret_cast<uintptr_t>(a), pb = reinterpret_cast<uintptr_t>(b);
    return pa < pb + nb && pb < pa + na;
}

size_t elem_bytes(int dtype) { return dtype == ARL2_BF16 ? 2 : 4; }
size_t q_bytes(const arl2_desc *d) { return (size_t)d->B * d->Lq * d->H * d->D * elem_bytes(d->io_dtype); }
size_t kv_bytes(const arl2_desc *d) { return (size_t)d->B * d->Lkv * d->H * d->D * elem_bytes(d->io_dtype); }
size_t state_bytes(const arl2_desc *d) { return (size_t)d->B * d->H * d->D * d->D * sizeof(float); }
size_t g_bytes(const arl2_desc *d)
{
    const size_t per_token = d->g_mode == ARL2_GATE_PER_TOKEN ? 1 : d->g_mode == ARL2_GATE_PER_ELEMENT ? (size_t)d->H * d->D : (size_t)d->H;
    return (size_t)d->B * d->Lq * per_token * elem_bytes(d->g_dtype);
}
size_t table_bytes(const arl2_desc *d) { return (size_t)d->Lq * (d->D / 2) * sizeof(float); }
size_t wmap_bytes(const arl2_desc *d) { return (size_t)d->H * d->D * d->D * 2; }

// The fp32 kernels put heads and streams on the grid's y and z axes.
bool f32_grid_ok(const arl2_desc *d) { return d->io_dtype != ARL2_F32 || (d->H <= 65535 && d->B <= 65535); }

// Checks everything that does not depend on which call is made.
arl2_status check_desc(const arl2_desc *d)
{
    if (d == nullptr) return fail(ARL2_ERR_INVALID_ARG, "desc is NULL");
    if (d->B < 1 || d->H < 1 || d->Lq < 1 || d->Lkv < 1)
        return fail(ARL2_ERR_INVALID_ARG, "B, H, Lq, Lkv must all be >= 1");
    if (d->io_dtype != ARL2_F32 && d->io_dtype != ARL2_BF16)
        return fail(ARL2_ERR_INVALID_ARG, "io_dtype is not an arl2_dtype");
    if (d->g_dtype != ARL2_F32 && d->g_dtype != ARL2_BF16)
        return fail(ARL2_ERR_INVALID_ARG, "g_dtype is not an arl2_dtype");
    if (d->g_mode != ARL2_GATE_PER_HEAD && d->g_mode != ARL2_GATE_PER_ELEMENT && d->g_mode != ARL2_GATE_PER_TOKEN)
        return fail(ARL2_ERR_INVALID_ARG, "g_mode is not an arl2_gate_mode");
    if (d->D != 64 && d->D != 128) return fail(ARL2_ERR_UNSUPPORTED, "D must be 64 or 128");
    if (!(d->sm_scale >= 0.f) || !(d->l2_eps >= 0.f))
        return fail(ARL2_ERR_INVALID_ARG, "sm_scale and l2_eps must be >= 0 (0 selects the default)");
    // element counts must stay addressable with the kernels' index arithmetic
    const double tokens = (double)d->B * (double)(d->Lq > d->Lkv ? d->Lq : d->Lkv);
    if (tokens > 2.0e9 || (double)d->B * d->H > 1.0e6)
        return fail(ARL2_ERR_UNSUPPORTED, "problem too large (B*L must stay below 2e9, B*H below 1e6)");
    return ARL2_OK;
}

// The kernels address one stream's [L][H][D] slice (and the feature map / gate projection the whole
// [B][L][H][D] array) with 32-bit byte offsets.
bool fits_32bit(double elems, int elem_bytes) { return elems * elem_bytes <= 2147483647.0; }

float resolved_eps(const arl2_desc *d) { return d->l2_eps > 0.f ? d->l2_eps : 1e-6f; }

size_t commit_workspace(const arl2_desc *d)
{
    if (d->io_dtype == ARL2_BF16)   // two partial matrices per split (delta rule) plus one state snapshot
        return (size_t)d->B * d->H * (2 * arl2::commit_nsplit(d->B, d->H, d->Lq) + 1) * d->D * d->D * sizeof(float);
    return (size_t)d->B * d->Lq * d->H * sizeof(float);
}

// What the plain commit alone needs (no delta-rule matrices, no state snapshot).
size_t commit_workspace_plain(const arl2_desc *d)
{
    if (d->io_dtype == ARL2_BF16)
        return (size_t)d->B * d->H * arl2::commit_nsplit(d->B, d->H, d->Lq) * d->D * d->D * sizeof(float);
    return (size_t)d->B * d->Lq * d->H * sizeof(float);
}

}  // namespace

extern "C" {

size_t arl2_workspace_bytes(const arl2_desc *desc)
{
    if (check_desc(desc) != ARL2_OK) return 0;
    return commit_workspace(desc);
}

arl2_status arl2_hybrid_attn_fwd_ex(const arl2_desc *desc, const void *q, const void *k, const void *v,
                                    const void *q_lin, const float *S, const void *g, void *out)
{
    arl2_status st = check_desc(desc);
    if (st != ARL2_OK) return st;
    if (!q || !k || !v || !out) return fail(ARL2_ERR_INVALID_ARG, "q, k, v and out must not be NULL");
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || !aligned16(S) || !aligned16(q_lin))
        return fail(ARL2_ERR_INVALID_ARG, "q, k, v, q_lin, S and out must be 16-byte aligned");
    if (g && (reinterpret_cast<uintptr_t>(g) & 3u))
        return fail(ARL2_ERR_INVALID_ARG, "g must be 4-byte aligned");
    if (g && desc->g_mode == ARL2_GATE_PER_ELEMENT && !aligned16(g))
        return fail(ARL2_ERR_INVALID_ARG, "an element-wise g must be 16-byte aligned");
    if (S != nullptr && desc->Lkv != desc->Lq)
        return fail(ARL2_ERR_INVALID_ARG, "Lkv must equal Lq when a state is given");
    if (!f32_grid_ok(desc)) return fail(ARL2_ERR_UNSUPPORTED, "fp32 inputs: H and B must stay below 65536");
    if (desc->io_dtype == ARL2_BF16 && !fits_32bit(((double)desc->Lkv + 256.0) * desc->H * desc->D, 2))
        return fail(ARL2_ERR_UNSUPPORTED, "one stream's k (or v) must stay below 2 GiB");
    {
        const size_t nq = q_bytes(desc), nkv = kv_bytes(desc);
        if (overlaps(out, nq, q, nq) || overlaps(out, nq, k, nkv) || overlaps(out, nq, v, nkv) || overlaps(out, nq, q_lin, nq) ||
            overlaps(out, nq, S, state_bytes(desc)) || overlaps(out, nq, g, g_bytes(desc)))
            return fail(ARL2_ERR_INVALID_ARG, "out must not overlap an input");
    }

    arl2::FwdArgs a;
    a.q = q; a.k = k; a.v = v; a.S = S; a.g = (S != nullptr) ? g : nullptr; a.out = out;
    a.q_lin = (S != nullptr) ? q_lin : nullptr;
    a.xq = nullptr; a.Wq = nullptr; a.cs = nullptr; a.sn = nullptr;
    a.B = desc->B; a.H = desc->H; a.Lq = desc->Lq; a.Lkv = desc->Lkv; a.D = desc->D;
    a.g_is_bf16 = desc->g_dtype == ARL2_BF16;
    a.g_per_element = desc->g_mode == ARL2_GATE_PER_ELEMENT;
    a.g_per_token = desc->g_mode == ARL2_GATE_PER_TOKEN;
    a.sm_scale = desc->sm_scale > 0.f ? desc->sm_scale : 1.0f / sqrtf((float)desc->D);
    a.l2_eps = resolved_eps(desc);
    hipStream_t stream = reinterpret_cast<hipStream_t>(desc->stream);
    const hipError_t e = desc->io_dtype == ARL2_BF16 ? arl2::launch_fwd_bf16(a, stream)
                                                     : arl2::launch_fwd_f32(a, stream);
    if (e != hipSuccess) return fail(ARL2_ERR_DEVICE, "fwd launch failed: %s", hipGetErrorString(e));
    return ARL2_OK;
}

arl2_status arl2_hybrid_attn_fwd(const arl2_desc *desc, const void *q, const void *k, const void *v,
                                 const float *S, const void *g, void *out)
{
    return arl2_hybrid_attn_fwd_ex(desc, q, k, v, nullptr, S, g, out);
}

arl2_status arl2_hybrid_attn_fwd_fm(const arl2_desc *desc, const void *q, const void *k, const void *v,
                                    const void *xq, const void *Wq, const float *rope_cos, const float *rope_sin,
                                    const float *S, const void *g, void *out)
{
    arl2_status st = check_desc(desc);
    if (st != ARL2_OK) return st;
    if (!q || !k || !v || !out || !xq || !Wq || !S)
        return fail(ARL2_ERR_INVALID_ARG, "q, k, v, xq, Wq, S and out must not be NULL");
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || !aligned16(S) || !aligned16(xq) || !aligned16(Wq))
        return fail(ARL2_ERR_INVALID_ARG, "q, k, v, xq, Wq, S and out must be 16-byte aligned");
    if ((rope_cos == nullptr) != (rope_sin == nullptr))
        return fail(ARL2_ERR_INVALID_ARG, "rope_cos and rope_sin must be given together");
    if ((reinterpret_cast<uintptr_t>(rope_cos) & 7u) || (reinterpret_cast<uintptr_t>(rope_sin) & 7u))
        return fail(ARL2_ERR_INVALID_ARG, "rope_cos and rope_sin must be 8-byte aligned");
    if (g && (reinterpret_cast<uintptr_t>(g) & 3u)) return fail(ARL2_ERR_INVALID_ARG, "g must be 4-byte aligned");
    if (g && desc->g_mode == ARL2_GATE_PER_ELEMENT && !aligned16(g))
        return fail(ARL2_ERR_INVALID_ARG, "an element-wise g must be 16-byte aligned");
    if (desc->Lkv != desc->Lq) return fail(ARL2_ERR_INVALID_ARG, "Lkv must equal Lq when a state is given");
    if (desc->io_dtype != ARL2_BF16) return fail(ARL2_ERR_UNSUPPORTED, "arl2_hybrid_attn_fwd_fm takes bf16 inputs only");
    if (!fits_32bit(((double)desc->Lkv + 256.0) * desc->H * desc->D, 2))
        return fail(ARL2_ERR_UNSUPPORTED, "one stream's k (or v) must stay below 2 GiB");
    {
        const size_t nq = q_bytes(desc), nkv = kv_bytes(desc);
        if (overlaps(out, nq, q, nq) || overlaps(out, nq, k, nkv) || overlaps(out, nq, v, nkv) || overlaps(out, nq, xq, nq) ||
            overlaps(out, nq, Wq, wmap_bytes(desc)) || overlaps(out, nq, S, state_bytes(desc)) || overlaps(out, nq, g, g_bytes(desc)) ||
            overlaps(out, nq, rope_cos, table_bytes(desc)) || overlaps(out, nq, rope_sin, table_bytes(desc)))
            return fail(ARL2_ERR_INVALID_ARG, "out must not overlap an input");
    }

    arl2::FwdArgs a;
    a.q = q; a.k = k; a.v = v; a.S = S; a.g = g; a.out = out; a.q_lin = nullptr;
    a.xq = xq; a.Wq = Wq; a.cs = rope_cos; a.sn = rope_sin;
    a.B = desc->B; a.H = desc->H; a.Lq = desc->Lq; a.Lkv = desc->Lkv; a.D = desc->D;
    a.g_is_bf16 = desc->g_dtype == ARL2_BF16;
    a.g_per_element = desc->g_mode == ARL2_GATE_PER_ELEMENT;
    a.g_per_token = desc->g_mode == ARL2_GATE_PER_TOKEN;
    a.sm_scale = desc->sm_scale > 0.f ? desc->sm_scale : 1.0f / sqrtf((float)desc->D);
    a.l2_eps = resolved_eps(desc);
    const hipError_t e = arl2::launch_fwd_bf16(a, reinterpret_cast<hipStream_t>(desc->stream));
    if (e != hipSuccess) return fail(ARL2_ERR_DEVICE, "fwd launch failed: %s", hipGetErrorString(e));
    return ARL2_OK;
}

arl2_status arl2_feature_map(const arl2_desc *desc, const void *x, const void *W,
                             const float *rope_cos, const float *rope_sin, void *y)
{
    arl2_status st = check_desc(desc);
    if (st != ARL2_OK) return st;
    if (!x || !W || !y) return fail(ARL2_ERR_INVALID_ARG, "x, W and y must not be NULL");
    if (!aligned16(x) || !aligned16(W) || !aligned16(y))
        return fail(ARL2_ERR_INVALID_ARG, "x, W and y must be 16-byte aligned");
    if ((rope_cos == nullptr) != (rope_sin == nullptr))
        return fail(ARL2_ERR_INVALID_ARG, "rope_cos and rope_sin must be given together");
    if ((reinterpret_cast<uintptr_t>(rope_cos) & 7u) || (reinterpret_cast<uintptr_t>(rope_sin) & 7u))
        return fail(ARL2_ERR_INVALID_ARG, "rope_cos and rope_sin must be 8-byte aligned");
    if (desc->io_dtype != ARL2_BF16) return fail(ARL2_ERR_UNSUPPORTED, "arl2_feature_map takes bf16 x, W only");
    if (!fits_32bit((double)desc->B * desc->Lq * desc->H * desc->D, 2))
        return fail(ARL2_ERR_UNSUPPORTED, "x must stay below 2 GiB");
    {
        const size_t nx = q_bytes(desc);
        if (overlaps(y, nx, x, nx) || overlaps(y, nx, W, wmap_bytes(desc)) || overlaps(y, nx, rope_cos, table_bytes(desc)) ||
            overlaps(y, nx, rope_sin, table_bytes(desc)))
            return fail(ARL2_ERR_INVALID_ARG, "y must not overlap an input");
    }

    arl2::FmapArgs a;
    a.x = x; a.W = W; a.cs = rope_cos; a.sn = rope_sin; a.y = y;
    a.B = desc->B; a.H = desc->H; a.L = desc->Lq; a.D = desc->D;
    const hipError_t e = arl2::launch_feature_map_bf16(a, reinterpret_cast<hipStream_t>(desc->stream));
    if (e != hipSuccess) return fail(ARL2_ERR_DEVICE, "feature map launch failed: %s", hipGetErrorString(e));
    return ARL2_OK;
}

arl2_status arl2_gate_proj(const arl2_desc *desc, const void *x, const void *Wg, void *g)
{
    arl2_status st = check_desc(desc);
    if (st != ARL2_OK) return st;
    if (!x || !Wg || !g) return fail(ARL2_ERR_INVALID_ARG, "x, Wg and g must not be NULL");
    if (!aligned16(x) || !aligned16(Wg)) return fail(ARL2_ERR_INVALID_ARG, "x and Wg must be 16-byte aligned");
    if (reinterpret_cast<uintptr_t>(g) & 3u) return fail(ARL2_ERR_INVALID_ARG, "g must be 4-byte aligned");
    if (desc->io_dtype != ARL2_BF16) return fail(ARL2_ERR_UNSUPPORTED, "arl2_gate_proj takes bf16 x, Wg only");
    if (!fits_32bit((double)desc->B * desc->Lq * desc->H * desc->D, 2))
        return fail(ARL2_ERR_UNSUPPORTED, "x must stay below 2 GiB");
    const int n_out = desc->g_mode == ARL2_GATE_PER_TOKEN ? 1 : desc->g_mode == ARL2_GATE_PER_ELEMENT ? desc->H * desc->D : desc->H;
    if (!fits_32bit((double)n_out * desc->H * desc->D, 2))
        return fail(ARL2_ERR_UNSUPPORTED, "Wg must stay below 2 GiB");
    {
        const size_t nx = (size_t)desc->B * desc->Lq * desc->H * desc->D * 2;
        const size_t rows = desc->g_mode == ARL2_GATE_PER_TOKEN ? 1 : desc->g_mode == ARL2_GATE_PER_ELEMENT ? (size_t)desc->H * desc->D : (size_t)desc->H;
        if (overlaps(g, g_bytes(desc), x, nx) || overlaps(g, g_bytes(desc), Wg, rows * desc->H * desc->D * 2))
            return fail(ARL2_ERR_INVALID_ARG, "g must not overlap an input");
    }

    arl2::GateArgs a;
    a.x = x; a.Wg = Wg; a.g = g;
    a.B = desc->B; a.H = desc->H; a.L = desc->Lq; a.dm = desc->H * desc->D;
    a.n_out = n_out;
    a.g_is_bf16 = desc->g_dtype == ARL2_BF16;
    const hipError_t e = arl2::launch_gate_proj_bf16(a, reinterpret_cast<hipStream_t>(desc->stream));
    if (e != hipSuccess) return fail(ARL2_ERR_DEVICE, "gate projection launch failed: %s", hipGetErrorString(e));
    return ARL2_OK;
}

static arl2_status commit_common(const arl2_desc *desc, const void *k, const void *v, const float *gate,
                                 const float *beta, bool delta, float *S)
{
    arl2_status st = check_desc(desc);
    if (st != ARL2_OK) return st;
    if (!k || !v || !gate || !S || (delta && !beta))
        return fail(ARL2_ERR_INVALID_ARG, "k, v, gate%s and S must not be NULL", delta ? ", beta" : "");
    if (!aligned16(k) || !aligned16(v) || !aligned16(S))
        return fail(ARL2_ERR_INVALID_ARG, "k, v and S must be 16-byte aligned");
    if ((reinterpret_cast<uintptr_t>(gate) & 3u) || (reinterpret_cast<uintptr_t>(beta) & 3u))
        return fail(ARL2_ERR_INVALID_ARG, "gate and beta must be 4-byte aligned");
    if (desc->Lkv != desc->Lq) return fail(ARL2_ERR_INVALID_ARG, "Lkv must equal Lq in a state commit");
    if (delta && desc->io_dtype != ARL2_BF16)
        return fail(ARL2_ERR_UNSUPPORTED, "arl2_state_commit_delta takes bf16 k, v only");
    if (desc->io_dtype == ARL2_BF16 && !fits_32bit(((double)desc->Lq + 256.0) * desc->H * desc->D, 2))
        return fail(ARL2_ERR_UNSUPPORTED, "one stream's k (or v) must stay below 2 GiB");
    const size_t need = delta ? commit_workspace(desc) : commit_workspace_plain(desc);
    if (desc->workspace == nullptr || desc->workspace_bytes < need)
        return fail(ARL2_ERR_WORKSPACE, "workspace is NULL or smaller than arl2_workspace_bytes()");
    if (!aligned16(desc->workspace)) return fail(ARL2_ERR_INVALID_ARG, "workspace must be 16-byte aligned");
    if (!f32_grid_ok(desc)) return fail(ARL2_ERR_UNSUPPORTED, "fp32 inputs: H and B must stay below 65536");
    {
        const size_t ns = state_bytes(desc), nkv = kv_bytes(desc), ngate = (size_t)desc->B * desc->H * sizeof(float);
        if (overlaps(S, ns, k, nkv) || overlaps(S, ns, v, nkv) || overlaps(S, ns, gate, ngate) || overlaps(S, ns, beta, ngate) ||
            overlaps(S, ns, desc->workspace, need))
            return fail(ARL2_ERR_INVALID_ARG, "S must not overlap k, v, the gates or the workspace");
        if (overlaps(desc->workspace, need, k, nkv) || overlaps(desc->workspace, need, v, nkv) ||
            overlaps(desc->workspace, need, gate, ngate) || overlaps(desc->workspace, need, beta, ngate))
            return fail(ARL2_ERR_INVALID_ARG, "the workspace must not overlap an input");
    }

    arl2::CommitArgs a;
    a.k = k; a.v = v; a.gate = gate; a.beta = delta ? beta : nullptr; a.S = S; a.workspace = desc->workspace;
    a.B = desc->B; a.H = desc->H; a.L = desc->Lq; a.D = desc->D;
    a.nsplit = arl2::commit_nsplit(desc->B, desc->H, desc->Lq);
    a.l2_eps = resolved_eps(desc);
    hipStream_t stream = reinterpret_cast<hipStream_t>(desc->stream);
    const hipError_t e = desc->io_dtype == ARL2_BF16 ? arl2::launch_commit_bf16(a, stream)
                                                     : arl2::launch_commit_f32(a, stream);
    if (e != hipSuccess) return fail(ARL2_ERR_DEVICE, "commit launch failed: %s", hipGetErrorString(e));
    return ARL2_OK;
}

arl2_status arl2_state_commit(const arl2_desc *desc, const void *k, const void *v, const float *gate, float *S)
{
    return commit_common(desc, k, v, gate, nullptr, false, S);
}

arl2_status arl2_state_commit_delta(const arl2_desc *desc, const void *k, const void *v, const float *gate,
                                    const float *beta, float *S)
{
    return commit_common(desc, k, v, gate, beta, true, S);
}

arl2_status arl2_state_commit_fm(const arl2_desc *desc, const void *xk, const void *Wk,
                                 const float *rope_cos, const float *rope_sin,
                                 const void *xv, const void *Wv, const float *gate, float *S)
{
    arl2_status st = check_desc(desc);
    if (st != ARL2_OK) return st;
    if (!xk || !Wk || !xv || !Wv || !gate || !S)
        return fail(ARL2_ERR_INVALID_ARG, "xk, Wk, xv, Wv, gate and S must not be NULL");
    if (!aligned16(xk) || !aligned16(Wk) || !aligned16(xv) || !aligned16(Wv) || !aligned16(S))
        return fail(ARL2_ERR_INVALID_ARG, "xk, Wk, xv, Wv and S must be 16-byte aligned");
    if ((rope_cos == nullptr) != (rope_sin == nullptr))
        return fail(ARL2_ERR_INVALID_ARG, "rope_cos and rope_sin must be given together");
    if ((reinterpret_cast<uintptr_t>(rope_cos) & 7u) || (reinterpret_cast<uintptr_t>(rope_sin) & 7u))
        return fail(ARL2_ERR_INVALID_ARG, "rope_cos and rope_sin must be 8-byte aligned");
    if (reinterpret_cast<uintptr_t>(gate) & 3u) return fail(ARL2_ERR_INVALID_ARG, "gate must be 4-byte aligned");
    if (desc->Lkv != desc->Lq) return fail(ARL2_ERR_INVALID_ARG, "Lkv must equal Lq in a state commit");
    if (desc->io_dtype != ARL2_BF16) return fail(ARL2_ERR_UNSUPPORTED, "arl2_state_commit_fm takes bf16 inputs only");
    if (!fits_32bit(((double)desc->Lq + 256.0) * desc->H * desc->D, 2))
        return fail(ARL2_ERR_UNSUPPORTED, "one stream's xk (or xv) must stay below 2 GiB");
    const size_t need = commit_workspace_plain(desc);
    if (desc->workspace == nullptr || desc->workspace_bytes < need)
        return fail(ARL2_ERR_WORKSPACE, "workspace is NULL or smaller than arl2_workspace_bytes()");
    if (!aligned16(desc->workspace)) return fail(ARL2_ERR_INVALID_ARG, "workspace must be 16-byte aligned");
    {
        const size_t ns = state_bytes(desc), nx = kv_bytes(desc), ngate = (size_t)desc->B * desc->H * sizeof(float);
        const size_t nw = wmap_bytes(desc), nt = table_bytes(desc);
        const void *in[] = {xk, xv, Wk, Wv, rope_cos, rope_sin, gate};
        const size_t nb[] = {nx, nx, nw, nw, nt, nt, ngate};
        for (int i = 0; i < 7; ++i) {
            if (overlaps(S, ns, in[i], nb[i])) return fail(ARL2_ERR_INVALID_ARG, "S must not overlap an input");
            if (overlaps(desc->workspace, need, in[i], nb[i]))
                return fail(ARL2_ERR_INVALID_ARG, "the workspace must not overlap an input");
        }
        if (overlaps(S, ns, desc->workspace, need)) return fail(ARL2_ERR_INVALID_ARG, "S must not overlap the workspace");
    }

    arl2::CommitFmArgs a;
    a.xk = xk; a.xv = xv; a.Wk = Wk; a.Wv = Wv; a.cs = rope_cos; a.sn = rope_sin;
    a.gate = gate; a.S = S; a.workspace = desc->workspace;
    a.B = desc->B; a.H = desc->H; a.L = desc->Lq; a.D = desc->D;
    a.nsplit = arl2::commit_nsplit(desc->B, desc->H, desc->Lq);
    a.l2_eps = resolved_eps(desc);
    const hipError_t e = arl2::launch_commit_fm_bf16(a, reinterpret_cast<hipStream_t>(desc->stream));
    if (e != hipSuccess) return fail(ARL2_ERR_DEVICE, "commit launch failed: %s", hipGetErrorString(e));
    return ARL2_OK;
}

size_t arl2_gdn_workspace_bytes(const arl2_desc *desc)
{
    if (check_desc(desc) != ARL2_OK) return 0;
    return arl2::gdn_workspace_bytes(desc->B, desc->H, desc->Lq, desc->D);
}

arl2_status arl2_state_commit_gdn(const arl2_desc *desc, const void *k, const void *v, const float *alpha,
                                  const float *beta, float *S)
{
    arl2_status st = check_desc(desc);
    if (st != ARL2_OK) return st;
    if (!k || !v || !alpha || !beta || !S)
        return fail(ARL2_ERR_INVALID_ARG, "k, v, alpha, beta and S must not be NULL");
    if (!aligned16(k) || !aligned16(v) || !aligned16(S))
        return fail(ARL2_ERR_INVALID_ARG, "k, v and S must be 16-byte aligned");
    if ((reinterpret_cast<uintptr_t>(alpha) & 3u) || (reinterpret_cast<uintptr_t>(beta) & 3u))
        return fail(ARL2_ERR_INVALID_ARG, "alpha and beta must be 4-byte aligned");
    if (desc->Lkv != desc->Lq) return fail(ARL2_ERR_INVALID_ARG, "Lkv must equal Lq in a state commit");
    if (desc->io_dtype != ARL2_BF16)
        return fail(ARL2_ERR_UNSUPPORTED, "arl2_state_commit_gdn takes bf16 k, v only");
    if (!fits_32bit(((double)desc->Lq + 256.0) * desc->H * desc->D, 2))
        return fail(ARL2_ERR_UNSUPPORTED, "one stream's k (or v) must stay below 2 GiB");
    const size_t need = arl2::gdn_workspace_bytes(desc->B, desc->H, desc->Lq, desc->D);
    if (desc->workspace == nullptr || desc->workspace_bytes < need)
        return fail(ARL2_ERR_WORKSPACE, "workspace is NULL or smaller than arl2_gdn_workspace_bytes()");
    if (!aligned16(desc->workspace)) return fail(ARL2_ERR_INVALID_ARG, "workspace must be 16-byte aligned");
    {
        const size_t ns = state_bytes(desc), nkv = kv_bytes(desc), ngate = (size_t)desc->B * desc->Lq * desc->H * sizeof(float);
        if (overlaps(S, ns, k, nkv) || overlaps(S, ns, v, nkv) || overlaps(S, ns, alpha, ngate) || overlaps(S, ns, beta, ngate) ||
            overlaps(S, ns, desc->workspace, need))
            return fail(ARL2_ERR_INVALID_ARG, "S must not overlap k, v, the gates or the workspace");
        if (overlaps(desc->workspace, need, k, nkv) || overlaps(desc->workspace, need, v, nkv) ||
            overlaps(desc->workspace, need, alpha, ngate) || overlaps(desc->workspace, need, beta, ngate))
            return fail(ARL2_ERR_INVALID_ARG, "the workspace must not overlap an input");
    }

    arl2::GdnArgs a;
    a.k = k; a.v = v; a.alpha = alpha; a.beta = beta; a.S = S; a.workspace = desc->workspace;
    a.B = desc->B; a.H = desc->H; a.L = desc->Lq; a.D = desc->D;
    a.l2_eps = resolved_eps(desc);
    const hipError_t e = arl2::launch_commit_gdn_bf16(a, reinterpret_cast<hipStream_t>(desc->stream));
    if (e != hipSuccess) return fail(ARL2_ERR_DEVICE, "gdn commit launch failed: %s", hipGetErrorString(e));
    return ARL2_OK;
}

// ---- entry point that allocates nothing ---------------------------------------------------------------
// The commit's token-split partial sums go to a fixed device array instead of a caller's workspace.  Every
// GPU the library runs on holds its own copy of the array (at its own address) until the process ends.
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];   // device address of `scratch` per device, looked up once

// The array's name is a host-side stand-in, not a device address: the address on the current device comes
// from the runtime, once per device, and only that pointer is ever handed to a kernel.
arl2_status static_scratch(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(ARL2_ERR_DEVICE, "hipGetDevice failed: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fail(ARL2_ERR_UNSUPPORTED, "device ordinal beyond the static scratch table");
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p == nullptr) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || p == nullptr)
            return fail(ARL2_ERR_DEVICE, "hipGetSymbolAddress(scratch) failed: %s", hipGetErrorString(e));
        g_scratch_ptr[dev].store(p, std::memory_order_release);   // every thread would look up the same address
    }
    *out = p;
    return ARL2_OK;
}

}  // namespace

size_t arl2_static_scratch_bytes(void) { return kStaticScratchBytes; }

arl2_status arl2_state_commit_static(const arl2_desc *desc, const void *k, const void *v, const float *gate, float *S)
{
    arl2_status st = check_desc(desc);
    if (st != ARL2_OK) return st;
    const size_t need = commit_workspace_plain(desc);
    if (need > kStaticScratchBytes)
        return fail(ARL2_ERR_UNSUPPORTED, "problem needs more scratch than the static array holds (arl2_static_scratch_bytes)");
    void *ptr = nullptr;
    st = static_scratch(&ptr);
    if (st != ARL2_OK) return st;
    arl2_desc d = *desc;
    d.workspace = ptr;
    d.workspace_bytes = kStaticScratchBytes;
    return commit_common(&d, k, v, gate, nullptr, false, S);
}

const char *arl2_status_string(arl2_status s)
{
    switch (s) {
    case ARL2_OK: return "ARL2_OK";
    case ARL2_ERR_INVALID_ARG: return "ARL2_ERR_INVALID_ARG";
    case ARL2_ERR_UNSUPPORTED: return "ARL2_ERR_UNSUPPORTED";
    case ARL2_ERR_WORKSPACE: return "ARL2_ERR_WORKSPACE";
    case ARL2_ERR_DEVICE: return "ARL2_ERR_DEVICE";
    }
    return "ARL2_ERR_UNKNOWN";
}

const char *arl2_last_error(void) { return g_err; }

int arl2_version(void) { return 100; }

}  // extern "C"
