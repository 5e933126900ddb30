/*
 * pskv.h - C ABI of the MI355X (gfx950) batched candidate-suffix attention library.
 *
 * The operation (paper Sec. 3 Eq. 2; Sec. 4.2 "prefix-shared, layer-wise lazy expansion";
 * Sec. 4.3 "suffix-centric alignment"; App. F.5): B candidate suffixes, stored left-aligned
 * and right-padded to S rows, attend (i) with full visibility to ONE shared prefix K/V of
 * P rows that exists once in memory and is never expanded over the candidates, and
 * (ii) causally to their own suffix K/V.  For candidate b, query row i < suf_len[b], query
 * head h (KV head k = h / (Hq/Hkv)):
 *
 *     out[b,i,h,:] = softmax_j( scale * <q[b,i,h,:], Kvis_j> ) * Vvis_j ,
 *     Kvis = k_pre[0..P-1,k,:] followed by k_suf[b,0..i,k,:]   (same for Vvis)
 *
 * which is exactly what a Standard KV cache (Eq. 3: prefix repeated B times) computes.
 * Rows i >= suf_len[b] are written as 0 (lse: -inf); padded Q/K/V rows may hold anything,
 * NaN included, and never influence a valid row.
 *
 * All pointers except the params struct and the returned strings are DEVICE pointers owned
 * by the caller.  The library allocates, frees and retains no device memory and keeps no
 * state between calls apart from a one-time set-up per device (compute-unit count, LDS limits
 * of its kernels, address of its built-in scratch), done at the first call on that device and
 * safe against host threads that make that first call at the same time.  The stream must belong
 * to the device that is current when the call is made.  Work is enqueued on the given stream and
 * the call returns without synchronising (no entry point synchronises, creates events or waits);
 * suf_len is read on the device.  No part of an input may share a byte with an output, nor two
 * outputs with each other: address ranges are compared, not just first bytes; column slices of one
 * fused buffer (same token stride, per-token spans side by side) are recognised as disjoint, any
 * other pair of tensors whose ranges meet is refused.
 * No exception crosses this boundary: every failure is a status code, with a thread-local
 * detail string available from pskv_last_error().  Validation happens on the host before
 * anything is launched: a call that returns INVALID_ARG, UNSUPPORTED or WORKSPACE has launched
 * nothing.  PSKV_ERR_HIP reports what the HIP runtime said about the library's own launch (not
 * an error left behind by earlier, unrelated calls); the backward calls launch two kernels, so
 * there the first may already be enqueued when the second is refused.
 */
#ifndef PSKV_H
#define PSKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PSKV_OK = 0,
    PSKV_ERR_INVALID_ARG = 1, /* null pointer, non-positive size, Hq % Hkv != 0, misaligned pointer/stride */
    PSKV_ERR_UNSUPPORTED = 2, /* shape or dtype outside what the kernels cover */
    PSKV_ERR_WORKSPACE = 3,   /* a workspace that cannot be used (misaligned, overlapping a tensor), or a
                                 problem that needs more scratch than pskv_attn_bwd_noalloc has built in */
    PSKV_ERR_HIP = 4          /* the HIP runtime refused a launch or query */
} pskv_status;

typedef enum {
    PSKV_DTYPE_F32 = 0, /* q/k/v/out are float; fp64 arithmetic on the vector ALU, results rounded to fp32 once */
    PSKV_DTYPE_BF16 = 1 /* q/k/v/out are bfloat16; bf16 MFMA with fp32 accumulation and fp32 softmax */
} pskv_dtype;

/* Kernel selection. AUTO picks the MFMA path whenever it covers the problem; the other two values
 * exist so that tests and benchmarks can run one problem through both implementations. */
typedef enum {
    PSKV_IMPL_AUTO = 0,
    PSKV_IMPL_SIMPLE = 1, /* one wavefront per query row, fp32 vector arithmetic; any D <= 256, any dtype */
    PSKV_IMPL_MFMA = 2    /* stacked-M bf16 MFMA path; bf16, D == 128 */
} pskv_impl;

/*
 * Problem description.  Notation follows the paper: P = N_p (prefix length), S = padded
 * suffix-side length (L_dec = N_s + N_t after padding), B = number of candidates
 * (N_cand, the "expand factor" of App. F.2), Hkv KV heads shared by groups of Hq/Hkv
 * consecutive query heads (GQA, App. C.1).
 *
 * Strides are in ELEMENTS; 0 means "contiguous" for the layouts
 *     q, out: [B,S,Hq,D]     k_suf, v_suf: [B,S,Hkv,D]     k_pre, v_pre: [P,Hkv,D]
 * and the innermost D dimension always has stride 1.  Non-zero strides must be multiples
 * of 8 elements (bf16) / 4 elements (f32) so that every row stays 16-byte aligned.
 */
typedef struct {
    int32_t B, S, P, Hq, Hkv, D; /* B,S,Hq,Hkv,D >= 1; P >= 0; Hq % Hkv == 0 */
    int32_t dtype;               /* pskv_dtype */
    int32_t impl;                /* pskv_impl */
    float scale;                 /* softmax scale; <= 0 selects 1/sqrt(D) (Eq. 2) */
    int32_t reserved;            /* must be 0 */
    int64_t q_stride_b, q_stride_s, q_stride_h;
    int64_t ks_stride_b, ks_stride_s, ks_stride_h; /* shared by k_suf and v_suf */
    int64_t kp_stride_p, kp_stride_h;              /* shared by k_pre and v_pre */
    int64_t o_stride_b, o_stride_s, o_stride_h;
} pskv_attn_params;

/* Library version as major*10000 + minor*100 + patch. Never fails. */
int pskv_version(void);

/* Static English name of a status code; "unknown status" for any other number. Never NULL.  (Takes an
 * int so that a number outside the enumeration is a defined argument in C++ callers as well.) */
const char *pskv_status_str(int status);

/* Detail text of the last error raised on the calling thread ("" if none). The pointer is
 * valid until the next library call on the same thread. */
const char *pskv_last_error(void);

/*
 * Device workspace, in bytes, that pskv_attn_fwd needs for this problem (0 when the chosen
 * kernels are fully fused, which is the case for every path in this version).  Returns
 * (size_t)-1 if the params are invalid.  Host-only, touches no device.
 */
size_t pskv_attn_fwd_workspace_bytes(const pskv_attn_params *p);

/*
 * Host-only check of a params struct (sizes, divisibility, dtype, strides, kernel coverage)
 * with the same rules pskv_attn_fwd applies.  Touches no device.
 */
pskv_status pskv_attn_validate(const pskv_attn_params *p);

/*
 * Batched candidate-suffix attention, forward (the whole hot path of one attention layer:
 * stacking of the B*S suffix queries into one dense row dimension, prefix scores and values
 * on the matrix cores, per-candidate causal suffix attention, online-softmax combine,
 * normalisation and store - Eq. 2 over the keys that App. F.5's concatenation would hold).
 *
 *   q       [B,S,Hq,D]   device, read-only
 *   k_suf   [B,S,Hkv,D]  device, read-only      v_suf likewise
 *   k_pre   [P,Hkv,D]    device, read-only, ONE copy for all candidates (may be NULL iff P == 0)
 *   v_pre   likewise
 *   suf_len [B] int32    device, values in [0,S]; NULL means every candidate has S rows.
 *                        Values outside [0,S] are clamped on the device.
 *   out     [B,S,Hq,D]   device, written in full (padded rows = 0)
 *   lse     [B,Hq,S] f32 device or NULL: natural-log sum of exp of the scaled visible scores
 *                        (-inf on padded rows)
 *   workspace / workspace_bytes: device scratch of at least pskv_attn_fwd_workspace_bytes();
 *                        may be NULL when that is 0
 *   hip_stream           a hipStream_t passed as void*; NULL is the default stream
 *
 * All data pointers must be 16-byte aligned.  Returns PSKV_OK once the kernels are enqueued.
 */
pskv_status pskv_attn_fwd(const pskv_attn_params *p,
                          const void *q, const void *k_suf, const void *v_suf,
                          const void *k_pre, const void *v_pre,
                          const int32_t *suf_len,
                          void *out, float *lse,
                          void *workspace, size_t workspace_bytes,
                          void *hip_stream);

/*
 * Batched multi-instruction form (paper Sec. 4.3, suffix-centric alignment; App. F.1, position
 * consistency under padding).  Np instructions are evaluated in one call: every instruction has
 * its own prefix K/V, LEFT-padded to the common length base.P (its real rows are the last
 * pre_len[n] ones; the padding rows are excluded from attention and may hold anything), and
 * owns C = base.B / Np consecutive candidates: candidate b belongs to instruction b / C.
 * All suffixes start at column 0 of the same dense [B,S,...] tensors, exactly as in the
 * single-instruction call.  A candidate attends to the real prefix rows of its own instruction
 * and causally to its own suffix rows; one prefix cache per instruction is read once and
 * reused by that instruction's candidates, never expanded over them.
 *
 * base describes everything but the prefix batch: base.B = Np*C candidates, base.P = padded
 * prefix length, base.kp_stride_p / kp_stride_h = strides inside one instruction's prefix.
 */
typedef struct {
    pskv_attn_params base;
    int32_t Np;          /* number of instructions, >= 1; base.B % Np == 0 */
    int32_t reserved;    /* must be 0 */
    int64_t kp_stride_n; /* elements between instructions in k_pre / v_pre; 0 = contiguous [Np,P,Hkv,D] */
} pskv_multi_params;

/* Host-only check of a multi-instruction params struct, same rules as pskv_attn_fwd_multi. */
pskv_status pskv_attn_multi_validate(const pskv_multi_params *p);

/*
 * Forward pass of the multi-instruction form.  Arguments as for pskv_attn_fwd, except:
 *
 *   k_pre, v_pre [Np,P,Hkv,D]  device, read-only, one left-padded prefix per instruction
 *   pre_len      [Np] int32    device, real prefix rows of each instruction, values in [0,P]
 *                              (clamped on the device); NULL means every prefix has P real rows
 *
 * With Np == 1 and pre_len == NULL this is pskv_attn_fwd.  Same ownership, stream and error
 * rules; no workspace is needed (workspace may be NULL).
 */
pskv_status pskv_attn_fwd_multi(const pskv_multi_params *p,
                                const void *q, const void *k_suf, const void *v_suf,
                                const void *k_pre, const void *v_pre,
                                const int32_t *pre_len, const int32_t *suf_len,
                                void *out, float *lse,
                                void *workspace, size_t workspace_bytes,
                                void *hip_stream);

/*
 * Backward pass of pskv_attn_fwd with respect to the suffix side.  The paper's cache keeps the
 * suffix/target segment in the computation graph so that gradient-based suffix synthesis can
 * differentiate through cached execution (Sec. 1, Sec. 4.2); the prefix K/V is a constant and
 * gets no gradient.  Given dout = dL/dout, this computes, for L any function of out,
 *
 *     dq = dL/dq,   dk_suf = dL/dk_suf,   dv_suf = dL/dv_suf
 *
 * by the derivative of Eq. 2 (with p_j the softmax weights of a query row over its visible
 * rows: ds_j = p_j (<dout_row, V_j> - <dout_row, out_row>), dq_row = scale sum_j ds_j K_j,
 * dK_j = scale sum_rows ds_j q_row, dV_j = sum_rows p_j dout_row; suffix rows only, summed over
 * the query heads that share the KV head).
 *
 *   q, k_suf, v_suf, k_pre, v_pre, suf_len   as for pskv_attn_fwd (same params struct)
 *   out   [B,S,Hq,D]  device, read-only: the forward result
 *   lse   [B,Hq,S]    device, read-only, REQUIRED: the forward log-sum-exp
 *   dout  [B,S,Hq,D]  device, read-only, laid out like out (o_stride_*)
 *   dq    [B,S,Hq,D]  device, written in full, laid out like q (q_stride_*); padded rows = 0
 *   dk_suf, dv_suf [B,S,Hkv,D] device, written in full, laid out like k_suf; padded rows = 0
 *
 *   workspace           optional device scratch of the caller's, 16-byte aligned, not aliasing any
 *                       other argument.  With at least pskv_attn_bwd_workspace_bytes(p) bytes the
 *                       matrix-core kernels pass <dout_row, out_row> of every row from the first
 *                       kernel to the second through it, so that `out` is read once; with NULL or
 *                       fewer bytes the call works all the same and reads `out` twice.  Its
 *                       contents after the call are unspecified.
 *
 * Padded rows of dout are ignored.  Same ownership, stream and error rules as the forward call;
 * outputs must not alias inputs or one another.  p->impl: SIMPLE selects the vector-ALU kernels
 * (fp64 arithmetic for f32 tensors, fp32 for bf16); AUTO uses the matrix-core kernels when the
 * tensors are bf16 with D == 128; MFMA insists on that and is refused otherwise.
 */
size_t pskv_attn_bwd_workspace_bytes(const pskv_attn_params *p); /* B*Hq*S*4; (size_t)-1 for invalid params */

pskv_status pskv_attn_bwd(const pskv_attn_params *p,
                          const void *q, const void *k_suf, const void *v_suf,
                          const void *k_pre, const void *v_pre,
                          const int32_t *suf_len,
                          const void *out, const float *lse, const void *dout,
                          void *dq, void *dk_suf, void *dv_suf,
                          void *workspace, size_t workspace_bytes,
                          void *hip_stream);

/*
 * Backward pass of pskv_attn_fwd_multi (the batched multi-instruction form of Sec. 4.3): the
 * instructions are independent, so candidate b's gradients are those of pskv_attn_bwd for the
 * problem made of its instruction's candidates and the real rows of that instruction's prefix
 * (the last pre_len[n] of the P left-padded ones, App. F.1).  Prefixes get no gradient.
 *
 *   k_pre, v_pre, pre_len   as for pskv_attn_fwd_multi (same params struct)
 *   everything else         as for pskv_attn_bwd (workspace: pskv_attn_bwd_workspace_bytes(&p->base))
 *
 * With Np == 1 and pre_len == NULL this is pskv_attn_bwd.
 */
pskv_status pskv_attn_bwd_multi(const pskv_multi_params *p,
                                const void *q, const void *k_suf, const void *v_suf,
                                const void *k_pre, const void *v_pre,
                                const int32_t *pre_len, const int32_t *suf_len,
                                const void *out, const float *lse, const void *dout,
                                void *dq, void *dk_suf, void *dv_suf,
                                void *workspace, size_t workspace_bytes,
                                void *hip_stream);

/*
 * pskv_attn_bwd for callers that cannot allocate device memory and have no workspace to bring: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and
 * results as pskv_attn_bwd without the workspace pair: the B*Hq*S floats that the first kernel hands
 * to the second live in a fixed array of PSKV_NOALLOC_SCRATCH_BYTES that is part of the library's
 * code object (every GPU the library runs on holds one copy until the process ends).  The call
 * allocates and frees nothing, on the device or through any library.  A problem with
 * B*Hq*S*4 > PSKV_NOALLOC_SCRATCH_BYTES is refused with PSKV_ERR_WORKSPACE (nothing launched); shapes
 * whose kernels use no scratch (fp32 tensors, D != 128) are served whatever their size.
 * All calls on one GPU share that array: two such calls that may run at the same time on one GPU
 * (different streams, or different host threads) race on it and must be ordered by the caller.
 * Nothing in it has to start from zero: the first kernel writes every entry the second reads.
 * The first call on a device looks up the array's address (one-time set-up): make it outside any
 * graph capture.
 */
#define PSKV_NOALLOC_SCRATCH_BYTES (8u << 20)
pskv_status pskv_attn_bwd_noalloc(const pskv_attn_params *p,
                                  const void *q, const void *k_suf, const void *v_suf,
                                  const void *k_pre, const void *v_pre,
                                  const int32_t *suf_len,
                                  const void *out, const float *lse, const void *dout,
                                  void *dq, void *dk_suf, void *dv_suf,
                                  void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* PSKV_H */
