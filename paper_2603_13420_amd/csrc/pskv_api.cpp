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
    if (out == q || out == k_suf || out == v_suf || out == k_pre || out == v_pre)
        return fail(PSKV_ERR_INVALID_ARG, "out must not alias an input");

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

const char *pskv_status_str(pskv_status s)
{
    switch (s) {
    case PSKV_OK: return "ok";
    case PSKV_ERR_INVALID_ARG: return "invalid argument";
    case PSKV_ERR_UNSUPPORTED: return "unsupported shape or dtype";
    case PSKV_ERR_WORKSPACE: return "workspace too small";
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
    const void *ins[] = {q, k_suf, v_suf, k_pre, v_pre, out, dout, lse};
    void *outs[] = {dq, dk_suf, dv_suf};
    for (int x = 0; x < 3; ++x) {
        for (const void *in : ins)
            if (outs[x] == in)
                return fail(PSKV_ERR_INVALID_ARG, "a gradient output must not alias an input");
        for (int y = x + 1; y < 3; ++y)
            if (outs[x] == outs[y])
                return fail(PSKV_ERR_INVALID_ARG, "gradient outputs must not alias one another");
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
            return fail(PSKV_ERR_INVALID_ARG, "workspace %p is not 16-byte aligned", workspace);
        for (const void *in : ins)
            if (workspace == in)
                return fail(PSKV_ERR_INVALID_ARG, "workspace must not alias an input");
        for (void *o : outs)
            if (workspace == o)
                return fail(PSKV_ERR_INVALID_ARG, "workspace must not alias an output");
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

pskv_status pskv_attn_fwd_timed(const pskv_attn_params *p, const void *q, const void *k_suf,
                                const void *v_suf, const void *k_pre, const void *v_pre,
                                const int32_t *suf_len, void *out, float *lse, void *workspace,
                                size_t workspace_bytes, void *hip_stream, int iters,
                                float *ms_per_call)
{
    if (iters < 1 || !ms_per_call)
        return fail(PSKV_ERR_INVALID_ARG, "iters must be >= 1 and ms_per_call non-NULL");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipEvent_t t0 = nullptr, t1 = nullptr;
    if (hipEventCreate(&t0) != hipSuccess || hipEventCreate(&t1) != hipSuccess) {
        if (t0) (void)hipEventDestroy(t0);
        return fail(PSKV_ERR_HIP, "hipEventCreate failed");
    }
    pskv_status s = PSKV_OK;
    hipError_t e = hipEventRecord(t0, stream);
    for (int it = 0; it < iters && s == PSKV_OK && e == hipSuccess; ++it)
        s = pskv_attn_fwd(p, q, k_suf, v_suf, k_pre, v_pre, suf_len, out, lse, workspace,
                          workspace_bytes, hip_stream);
    if (e == hipSuccess)
        e = hipEventRecord(t1, stream);
    if (e == hipSuccess)
        e = hipEventSynchronize(t1);
    float ms = 0.f;
    if (e == hipSuccess)
        e = hipEventElapsedTime(&ms, t0, t1);
    (void)hipEventDestroy(t0);
    (void)hipEventDestroy(t1);
    if (s != PSKV_OK)
        return s;
    if (e != hipSuccess)
        return fail(PSKV_ERR_HIP, "event timing failed: %s", hipGetErrorString(e));
    *ms_per_call = ms / (float)iters;
    return PSKV_OK;
}

} // extern "C"
