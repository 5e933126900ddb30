// Host side of the C ABI declared in include/pskv.h: argument validation, kernel choice,
// launches on the caller's stream.  No device memory is allocated here.
#include "../../include/pskv.h"
#include "pskv_internal.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>

namespace {

thread_local char g_err[512] = "";

pskv_status fail(pskv_status s, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return s;
}

constexpr size_t kSimpleMaxLds = 64 * 1024;

// Fills `a` (without pointers) and `use_mfma` from p, applying every host-side rule.
// np, kp_stride_n: the instruction batch of the multi-instruction form (1, 0 for a single prefix).
pskv_status resolve(const pskv_attn_params *p, int np, long long kp_stride_n, pskv::Args &a, bool &use_mfma)
{
    if (!p)
        return fail(PSKV_ERR_INVALID_ARG, "params is NULL");
    if (np < 1)
        return fail(PSKV_ERR_INVALID_ARG, "Np=%d must be at least 1", np);
    if (p->B >= 1 && p->B % np != 0)
        return fail(PSKV_ERR_INVALID_ARG, "B=%d is not a multiple of Np=%d (every instruction owns B/Np consecutive candidates)",
                    p->B, np);
    if (p->B < 1 || p->S < 1 || p->Hq < 1 || p->Hkv < 1 || p->D < 1 || p->P < 0)
        return fail(PSKV_ERR_INVALID_ARG, "sizes must satisfy B,S,Hq,Hkv,D >= 1 and P >= 0 (got B=%d S=%d P=%d Hq=%d Hkv=%d D=%d)",
                    p->B, p->S, p->P, p->Hq, p->Hkv, p->D);
    if (p->Hq % p->Hkv != 0)
        return fail(PSKV_ERR_INVALID_ARG, "Hq=%d is not a multiple of Hkv=%d", p->Hq, p->Hkv);
    if (p->reserved != 0)
        return fail(PSKV_ERR_INVALID_ARG, "reserved field must be 0");
    if (p->dtype != PSKV_DTYPE_F32 && p->dtype != PSKV_DTYPE_BF16)
        return fail(PSKV_ERR_INVALID_ARG, "unknown dtype %d", p->dtype);
    if (p->impl != PSKV_IMPL_AUTO && p->impl != PSKV_IMPL_SIMPLE && p->impl != PSKV_IMPL_MFMA)
        return fail(PSKV_ERR_INVALID_ARG, "unknown impl %d", p->impl);
    if (!(p->scale == p->scale) || std::isinf(p->scale))
        return fail(PSKV_ERR_INVALID_ARG, "scale is not finite");
    const int vec = p->dtype == PSKV_DTYPE_BF16 ? 8 : 4; // elements per 16 bytes
    if (p->D % vec != 0)
        return fail(PSKV_ERR_UNSUPPORTED, "D=%d must be a multiple of %d so rows stay 16-byte aligned", p->D, vec);
    if (p->D > 256)
        return fail(PSKV_ERR_UNSUPPORTED, "D=%d exceeds the supported maximum of 256", p->D);
    const long long rows = (long long)p->B * p->S * p->Hq;
    if (rows > 0x7fffffffLL)
        return fail(PSKV_ERR_UNSUPPORTED, "B*S*Hq=%lld exceeds 2^31-1", rows);

    a.B = p->B; a.S = p->S; a.P = p->P; a.Hq = p->Hq; a.Hkv = p->Hkv; a.D = p->D;
    a.G = p->Hq / p->Hkv;
    a.Np = np;
    a.C = p->B / np;
    a.plen = nullptr;
    a.div_g = pskv::make_fastdiv((unsigned)a.G);
    a.div_s = pskv::make_fastdiv((unsigned)a.S);
    a.scale = p->scale > 0.f ? p->scale : 1.0f / std::sqrt((float)p->D);

    struct { const char *name; long long given, dflt; long long *dst; } st[] = {
        {"q_stride_h", p->q_stride_h, (long long)p->D, &a.q_sh},
        {"q_stride_s", p->q_stride_s, (long long)p->Hq * p->D, &a.q_ss},
        {"q_stride_b", p->q_stride_b, (long long)p->S * p->Hq * p->D, &a.q_sb},
        {"ks_stride_h", p->ks_stride_h, (long long)p->D, &a.ks_sh},
        {"ks_stride_s", p->ks_stride_s, (long long)p->Hkv * p->D, &a.ks_ss},
        {"ks_stride_b", p->ks_stride_b, (long long)p->S * p->Hkv * p->D, &a.ks_sb},
        {"kp_stride_h", p->kp_stride_h, (long long)p->D, &a.kp_sh},
        {"kp_stride_p", p->kp_stride_p, (long long)p->Hkv * p->D, &a.kp_sp},
        {"o_stride_h", p->o_stride_h, (long long)p->D, &a.o_sh},
        {"o_stride_s", p->o_stride_s, (long long)p->Hq * p->D, &a.o_ss},
        {"o_stride_b", p->o_stride_b, (long long)p->S * p->Hq * p->D, &a.o_sb},
    };
    for (auto &s : st) {
        if (s.given < 0)
            return fail(PSKV_ERR_INVALID_ARG, "%s=%lld is negative", s.name, s.given);
        if (s.given != 0 && s.given % vec != 0)
            return fail(PSKV_ERR_INVALID_ARG, "%s=%lld is not a multiple of %d elements (16 bytes)", s.name, s.given, vec);
        if (s.given != 0 && s.given < p->D)
            return fail(PSKV_ERR_INVALID_ARG, "%s=%lld is smaller than D=%d (rows would overlap)", s.name, s.given, p->D);
        *s.dst = s.given ? s.given : s.dflt;
    }

    {
        const long long one = (long long)p->P * a.kp_sp; // span of one instruction's prefix
        if (kp_stride_n < 0)
            return fail(PSKV_ERR_INVALID_ARG, "kp_stride_n=%lld is negative", kp_stride_n);
        if (kp_stride_n != 0 && kp_stride_n % vec != 0)
            return fail(PSKV_ERR_INVALID_ARG, "kp_stride_n=%lld is not a multiple of %d elements (16 bytes)", kp_stride_n, vec);
        if (kp_stride_n != 0 && np > 1 && kp_stride_n < one)
            return fail(PSKV_ERR_INVALID_ARG, "kp_stride_n=%lld is smaller than one prefix (%lld elements)", kp_stride_n, one);
        a.kp_sn = kp_stride_n ? kp_stride_n : one;
    }

    const bool mfma_ok = pskv::mfma_supported(a, p->dtype);
    if (p->impl == PSKV_IMPL_MFMA && !mfma_ok)
        return fail(PSKV_ERR_UNSUPPORTED, "the MFMA path needs dtype bf16 and D == 128 (got dtype=%d D=%d S=%d)",
                    p->dtype, p->D, p->S);
    use_mfma = mfma_ok && p->impl != PSKV_IMPL_SIMPLE;
    if (!use_mfma && pskv::simple_lds_bytes(a, p->dtype) > kSimpleMaxLds)
        return fail(PSKV_ERR_UNSUPPORTED, "the simple path keeps one score row in LDS: P+S+D=%d is too large",
                    p->P + p->S + p->D);
    return PSKV_OK;
}

bool misaligned(const void *ptr) { return (reinterpret_cast<uintptr_t>(ptr) & 15u) != 0; }

// A tensor as a range of addresses: [lo, hi) covers every byte the strides can reach.  When all of
// its tokens (one position of one candidate: n2 rows of d elements, s2 apart) start on a lattice of
// pitch bytes from lo - the token stride, which the candidate stride is a multiple of - pitch and the
// bytes one token spans (foot) are kept too: that is the shape of a column slice of a fused buffer.
struct Span {
    uintptr_t lo, hi;
    const char *name;
    uintptr_t pitch, foot; // pitch 0: no lattice known
};
Span span4(const void *ptr, long long n0, long long s0, long long n1, long long s1, long long n2, long long s2, long long d,
           int esize, const char *name)
{
    if (!ptr || n0 < 1 || n1 < 1 || n2 < 1)
        return Span{0, 0, name, 0, 0};
    const long long last = (n0 - 1) * s0 + (n1 - 1) * s1 + (n2 - 1) * s2 + d; // elements up to the end of the last row
    const uintptr_t lo = reinterpret_cast<uintptr_t>(ptr);
    Span s{lo, lo + (uintptr_t)last * (uintptr_t)esize, name, 0, 0};
    const long long foot = (n2 - 1) * s2 + d;
    if (s1 > 0 && foot <= s1 && (n0 == 1 || s0 % s1 == 0)) {
        s.pitch = (uintptr_t)s1 * (uintptr_t)esize;
        s.foot = (uintptr_t)foot * (uintptr_t)esize;
    }
    return s;
}
// Whether two tensors may share a byte.  Ranges that do not meet share nothing; two column slices of
// one fused buffer (same token pitch) interleave without sharing a byte when their per-token spans sit
// side by side inside the pitch.  Anything else whose ranges meet is treated as overlapping.
bool overlap(const Span &x, const Span &y)
{
    if (!(x.lo < y.hi && y.lo < x.hi))
        return false;
    if (x.pitch != 0 && x.pitch == y.pitch) {
        const uintptr_t delta = y.lo >= x.lo ? (y.lo - x.lo) % x.pitch : (x.pitch - (x.lo - y.lo) % x.pitch) % x.pitch;
        if (x.foot <= delta && delta + y.foot <= x.pitch)
            return false; // x's tokens fill [0, foot) of every pitch, y's [delta, delta + foot)
    }
    return true;
}

// The address ranges of a problem's tensors (np: prefixes in k_pre / v_pre).
struct Spans {
    Span q, ks, vs, kp, vp, out;
};
Spans tensor_spans(const pskv::Args &a, int esize, const void *q, const void *ks, const void *vs, const void *kp,
                   const void *vp, const void *out)
{
    Spans s;
    s.q = span4(q, a.B, a.q_sb, a.S, a.q_ss, a.Hq, a.q_sh, a.D, esize, "q");
    s.ks = span4(ks, a.B, a.ks_sb, a.S, a.ks_ss, a.Hkv, a.ks_sh, a.D, esize, "k_suf");
    s.vs = span4(vs, a.B, a.ks_sb, a.S, a.ks_ss, a.Hkv, a.ks_sh, a.D, esize, "v_suf");
    s.kp = span4(a.P > 0 ? kp : nullptr, a.Np, a.kp_sn, a.P, a.kp_sp, a.Hkv, a.kp_sh, a.D, esize, "k_pre");
    s.vp = span4(a.P > 0 ? vp : nullptr, a.Np, a.kp_sn, a.P, a.kp_sp, a.Hkv, a.kp_sh, a.D, esize, "v_pre");
    s.out = span4(out, a.B, a.o_sb, a.S, a.o_ss, a.Hq, a.o_sh, a.D, esize, "out");
    return s;
}

// Everything the two forward entry points share: checks, then one launch on the caller's stream.
pskv_status launch(const pskv_attn_params *p, int np, long long kp_stride_n, const void *q, const void *k_suf,
                   const void *v_suf, const void *k_pre, const void *v_pre, const int32_t *pre_len,
                   const int32_t *suf_len, void *out, float *lse, void *hip_stream)
{
    pskv::Args a{};
    bool use_mfma = false;
    pskv_status s = resolve(p, np, kp_stride_n, a, use_mfma);
    if (s != PSKV_OK)
        return s;
    if (!q || !k_suf || !v_suf || !out)
        return fail(PSKV_ERR_INVALID_ARG, "q, k_suf, v_suf and out must not be NULL");
    if (a.P > 0 && (!k_pre || !v_pre))
        return fail(PSKV_ERR_INVALID_ARG, "k_pre and v_pre must not be NULL when P > 0");
    const void *ptrs[] = {q, k_suf, v_suf, k_pre, v_pre, out};
    for (const void *ptr : ptrs)
        if (misaligned(ptr))
            return fail(PSKV_ERR_INVALID_ARG, "data pointer %p is not 16-byte aligned", ptr);
    if ((reinterpret_cast<uintptr_t>(suf_len) & 3u) || (reinterpret_cast<uintptr_t>(lse) & 3u) ||
        (reinterpret_cast<uintptr_t>(pre_len) & 3u))
        return fail(PSKV_ERR_INVALID_ARG, "suf_len, pre_len and lse must be 4-byte aligned");
    {
        const int esize = p->dtype == PSKV_DTYPE_BF16 ? 2 : 4;
        const Spans sp = tensor_spans(a, esize, q, k_suf, v_suf, k_pre, v_pre, out);
        const Span lse_span = span4(lse, 1, 0, 1, 0, 1, 0, (long long)a.B * a.Hq * a.S, 4, "lse");
        for (const Span &in : {sp.q, sp.ks, sp.vs, sp.kp, sp.vp}) {
            if (overlap(sp.out, in))
                return fail(PSKV_ERR_INVALID_ARG, "out overlaps %s: an output must not alias an input", in.name);
            if (overlap(lse_span, in))
                return fail(PSKV_ERR_INVALID_ARG, "lse overlaps %s: an output must not alias an input", in.name);
        }
        if (overlap(sp.out, lse_span))
            return fail(PSKV_ERR_INVALID_ARG, "out overlaps lse");
    }

    a.q = q; a.ks = k_suf; a.vs = v_suf; a.kp = k_pre; a.vp = v_pre;
    a.len = suf_len; a.plen = pre_len; a.out = out; a.lse = lse;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipError_t e = use_mfma ? pskv::launch_mfma(a, stream) : pskv::launch_simple(a, p->dtype, stream);
    if (e != hipSuccess)
        return fail(PSKV_ERR_HIP, "kernel launch failed: %s", hipGetErrorString(e));
    g_err[0] = '\0';
    return PSKV_OK;
}

} // namespace

extern "C" {

int pskv_version(void) { return 100; }

const char *pskv_status_str(int status)
{
    switch (status) {
    case PSKV_OK: return "ok";
    case PSKV_ERR_INVALID_ARG: return "invalid argument";
    case PSKV_ERR_UNSUPPORTED: return "unsupported shape or dtype";
    case PSKV_ERR_WORKSPACE: return "unusable workspace or scratch too small";
    case PSKV_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

const char *pskv_last_error(void) { return g_err; }

size_t pskv_attn_fwd_workspace_bytes(const pskv_attn_params *p)
{
    pskv::Args a{};
    bool use_mfma = false;
    if (resolve(p, 1, 0, a, use_mfma) != PSKV_OK)
        return (size_t)-1;
    return 0; // every path is fully fused
}

size_t pskv_attn_bwd_workspace_bytes(const pskv_attn_params *p)
{
    pskv::Args a{};
    bool use_mfma = false;
    if (resolve(p, 1, 0, a, use_mfma) != PSKV_OK)
        return (size_t)-1;
    return (size_t)p->B * (size_t)p->Hq * (size_t)p->S * sizeof(float);
}

pskv_status pskv_attn_validate(const pskv_attn_params *p)
{
    pskv::Args a{};
    bool use_mfma = false;
    pskv_status s = resolve(p, 1, 0, a, use_mfma);
    if (s == PSKV_OK)
        g_err[0] = '\0';
    return s;
}

pskv_status pskv_attn_fwd(const pskv_attn_params *p, const void *q, const void *k_suf,
                          const void *v_suf, const void *k_pre, const void *v_pre,
                          const int32_t *suf_len, void *out, float *lse, void *workspace,
                          size_t workspace_bytes, void *hip_stream)
{
    (void)workspace;
    (void)workspace_bytes; // no path needs scratch
    return launch(p, 1, 0, q, k_suf, v_suf, k_pre, v_pre, nullptr, suf_len, out, lse, hip_stream);
}

pskv_status pskv_attn_multi_validate(const pskv_multi_params *p)
{
    if (!p)
        return fail(PSKV_ERR_INVALID_ARG, "params is NULL");
    if (p->reserved != 0)
        return fail(PSKV_ERR_INVALID_ARG, "reserved field must be 0");
    pskv::Args a{};
    bool use_mfma = false;
    pskv_status s = resolve(&p->base, p->Np, p->kp_stride_n, a, use_mfma);
    if (s == PSKV_OK)
        g_err[0] = '\0';
    return s;
}

pskv_status pskv_attn_fwd_multi(const pskv_multi_params *p, const void *q, const void *k_suf,
                                const void *v_suf, const void *k_pre, const void *v_pre,
                                const int32_t *pre_len, const int32_t *suf_len, void *out, float *lse,
                                void *workspace, size_t workspace_bytes, void *hip_stream)
{
    (void)workspace;
    (void)workspace_bytes; // no path needs scratch
    if (!p)
        return fail(PSKV_ERR_INVALID_ARG, "params is NULL");
    if (p->reserved != 0)
        return fail(PSKV_ERR_INVALID_ARG, "reserved field must be 0");
    return launch(&p->base, p->Np, p->kp_stride_n, q, k_suf, v_suf, k_pre, v_pre, pre_len, suf_len, out, lse,
                  hip_stream);
}

// Validation and launch shared by the two backward entry points (np == 1, pre_len == NULL: one
// shared prefix).
static pskv_status launch_bwd(const pskv_attn_params *p, int np, int64_t kp_stride_n, const void *q, const void *k_suf,
                              const void *v_suf, const void *k_pre, const void *v_pre, const int32_t *pre_len,
                              const int32_t *suf_len, const void *out, const float *lse, const void *dout, void *dq,
                              void *dk_suf, void *dv_suf, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    pskv::BwdArgs g{};
    pskv::Args &a = g.f;
    bool use_mfma = false;
    pskv_status s = resolve(p, np, kp_stride_n, a, use_mfma);
    if (s != PSKV_OK)
        return s;
    const bool dq_mfma = use_mfma && pskv::bwd_mfma_supported(a, p->dtype);
    if (p->impl == PSKV_IMPL_MFMA && !dq_mfma)
        return fail(PSKV_ERR_UNSUPPORTED, "the MFMA path of the backward pass needs dtype bf16 and D == 128");
    if (!dq_mfma && pskv::bwd_simple_lds_bytes(a, p->dtype) > kSimpleMaxLds)
        return fail(PSKV_ERR_UNSUPPORTED, "the backward pass keeps one score row in LDS: P+S+2D=%d is too large",
                    p->P + p->S + 2 * p->D);
    if (!dq_mfma && pskv::bwd_dkv_lds_bytes(a, p->dtype) > kSimpleMaxLds)
        return fail(PSKV_ERR_UNSUPPORTED, "the dk/dv kernel keeps one value per query row of a group in LDS: G*S=%d is too large",
                    a.G * p->S);
    if (!q || !k_suf || !v_suf || !out || !lse || !dout || !dq || !dk_suf || !dv_suf)
        return fail(PSKV_ERR_INVALID_ARG, "q, k_suf, v_suf, out, lse, dout, dq, dk_suf and dv_suf must not be NULL");
    if (a.P > 0 && (!k_pre || !v_pre))
        return fail(PSKV_ERR_INVALID_ARG, "k_pre and v_pre must not be NULL when P > 0");
    const void *ptrs[] = {q, k_suf, v_suf, k_pre, v_pre, out, dout, dq, dk_suf, dv_suf};
    for (const void *ptr : ptrs)
        if (misaligned(ptr))
            return fail(PSKV_ERR_INVALID_ARG, "data pointer %p is not 16-byte aligned", ptr);
    if ((reinterpret_cast<uintptr_t>(suf_len) & 3u) || (reinterpret_cast<uintptr_t>(lse) & 3u) ||
        (reinterpret_cast<uintptr_t>(pre_len) & 3u))
        return fail(PSKV_ERR_INVALID_ARG, "suf_len, pre_len and lse must be 4-byte aligned");
    const int esize = p->dtype == PSKV_DTYPE_BF16 ? 2 : 4;
    const Spans sp = tensor_spans(a, esize, q, k_suf, v_suf, k_pre, v_pre, out);
    const Span ins[] = {sp.q, sp.ks, sp.vs, sp.kp, sp.vp, sp.out,
                        span4(dout, a.B, a.o_sb, a.S, a.o_ss, a.Hq, a.o_sh, a.D, esize, "dout"),
                        span4(lse, 1, 0, 1, 0, 1, 0, (long long)a.B * a.Hq * a.S, 4, "lse")};
    const Span outs[] = {span4(dq, a.B, a.q_sb, a.S, a.q_ss, a.Hq, a.q_sh, a.D, esize, "dq"),
                         span4(dk_suf, a.B, a.ks_sb, a.S, a.ks_ss, a.Hkv, a.ks_sh, a.D, esize, "dk_suf"),
                         span4(dv_suf, a.B, a.ks_sb, a.S, a.ks_ss, a.Hkv, a.ks_sh, a.D, esize, "dv_suf")};
    for (int x = 0; x < 3; ++x) {
        for (const Span &in : ins)
            if (overlap(outs[x], in))
                return fail(PSKV_ERR_INVALID_ARG, "%s overlaps %s: a gradient output must not alias an input", outs[x].name,
                            in.name);
        for (int y = x + 1; y < 3; ++y)
            if (overlap(outs[x], outs[y]))
                return fail(PSKV_ERR_INVALID_ARG, "%s overlaps %s: gradient outputs must not alias one another",
                            outs[x].name, outs[y].name);
    }
    a.q = q; a.ks = k_suf; a.vs = v_suf; a.kp = k_pre; a.vp = v_pre;
    a.len = suf_len;
    a.plen = pre_len;
    a.out = const_cast<void *>(out); // read-only in every backward kernel
    a.lse = const_cast<float *>(lse);
    g.dout = dout; g.dq = dq; g.dk = dk_suf; g.dv = dv_suf;
    // With enough workspace the matrix-core kernels pass <dout_row, out_row> from the first kernel
    // to the second through it; without, the second reads out again.
    const size_t delta_bytes = (size_t)p->B * (size_t)p->Hq * (size_t)p->S * sizeof(float);
    g.delta = nullptr;
    if (dq_mfma && workspace && workspace_bytes >= delta_bytes) {
        if (reinterpret_cast<uintptr_t>(workspace) & 15u)
            return fail(PSKV_ERR_WORKSPACE, "workspace %p is not 16-byte aligned", workspace);
        const Span ws = span4(workspace, 1, 0, 1, 0, 1, 0, (long long)delta_bytes, 1, "workspace");
        for (const Span &in : ins)
            if (overlap(ws, in))
                return fail(PSKV_ERR_WORKSPACE, "workspace overlaps %s", in.name);
        for (const Span &o : outs)
            if (overlap(ws, o))
                return fail(PSKV_ERR_WORKSPACE, "workspace overlaps %s", o.name);
        g.delta = static_cast<float *>(workspace);
    }
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipError_t e = dq_mfma ? pskv::launch_bwd_dq_mfma(g, stream) : pskv::launch_bwd_dq_simple(g, p->dtype, stream);
    if (e == hipSuccess)
        e = dq_mfma ? pskv::launch_bwd_dkv_mfma(g, stream) : pskv::launch_bwd_dkv_simple(g, p->dtype, stream);
    if (e != hipSuccess)
        return fail(PSKV_ERR_HIP, "kernel launch failed: %s", hipGetErrorString(e));
    g_err[0] = '\0';
    return PSKV_OK;
}

pskv_status pskv_attn_bwd(const pskv_attn_params *p, const void *q, const void *k_suf, const void *v_suf,
                          const void *k_pre, const void *v_pre, const int32_t *suf_len, const void *out,
                          const float *lse, const void *dout, void *dq, void *dk_suf, void *dv_suf,
                          void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return launch_bwd(p, 1, 0, q, k_suf, v_suf, k_pre, v_pre, nullptr, suf_len, out, lse, dout, dq, dk_suf, dv_suf,
                      workspace, workspace_bytes, hip_stream);
}

pskv_status pskv_attn_bwd_multi(const pskv_multi_params *p, const void *q, const void *k_suf, const void *v_suf,
                                const void *k_pre, const void *v_pre, const int32_t *pre_len, const int32_t *suf_len,
                                const void *out, const float *lse, const void *dout, void *dq, void *dk_suf,
                                void *dv_suf, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!p)
        return fail(PSKV_ERR_INVALID_ARG, "params is NULL");
    if (p->reserved != 0)
        return fail(PSKV_ERR_INVALID_ARG, "reserved field must be 0");
    return launch_bwd(&p->base, p->Np, p->kp_stride_n, q, k_suf, v_suf, k_pre, v_pre, pre_len, suf_len, out, lse, dout, dq,
                      dk_suf, dv_suf, workspace, workspace_bytes, hip_stream);
}

pskv_status pskv_attn_bwd_noalloc(const pskv_attn_params *p, const void *q, const void *k_suf, const void *v_suf,
                                  const void *k_pre, const void *v_pre, const int32_t *suf_len, const void *out,
                                  const float *lse, const void *dout, void *dq, void *dk_suf, void *dv_suf,
                                  void *hip_stream)
{
    pskv::Args a{};
    bool use_mfma = false;
    pskv_status s = resolve(p, 1, 0, a, use_mfma);
    if (s != PSKV_OK)
        return s;
    void *scratch_ptr = nullptr;
    size_t scratch_bytes = 0;
    if (use_mfma && pskv::bwd_mfma_supported(a, p->dtype)) { // the kernels that use the scratch
        const size_t need = (size_t)p->B * (size_t)p->Hq * (size_t)p->S * sizeof(float);
        if (need > pskv::kNoAllocScratchBytes)
            return fail(PSKV_ERR_WORKSPACE,
                        "B*Hq*S*4 = %zu bytes of scratch exceed the %zu bytes built into the library: use pskv_attn_bwd "
                        "with a workspace of the caller's",
                        need, (size_t)pskv::kNoAllocScratchBytes);
        const hipError_t e = pskv::noalloc_scratch(&scratch_ptr);
        if (e != hipSuccess)
            return fail(PSKV_ERR_HIP, "address of the built-in scratch: %s", hipGetErrorString(e));
        scratch_bytes = need;
    }
    return launch_bwd(p, 1, 0, q, k_suf, v_suf, k_pre, v_pre, nullptr, suf_len, out, lse, dout, dq, dk_suf, dv_suf,
                      scratch_ptr, scratch_bytes, hip_stream);
}

} // extern "C"
