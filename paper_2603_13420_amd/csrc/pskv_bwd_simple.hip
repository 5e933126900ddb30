// Simple path of the backward pass of batched candidate-suffix attention: gradients of
// sum(dout * out) with respect to q, k_suf and v_suf.  The prefix K/V is a constant of the
// candidate evaluation (Sec. 4.2: the prefix cache is built once, only the suffix/target side
// stays in the computation graph), so it receives no gradient.
//
// Two kernels, both written straight from the derivative of Eq. 2 for one query row with
// probabilities p_j = exp(s_j - lse) over its visible rows:
//     dp_j = <dout_row, V_j>,  ds_j = p_j (dp_j - <dout_row, out_row>),
//     dq_row = scale * sum_j ds_j K_j,  dK_j = scale * sum_rows ds_j q_row,  dV_j = sum_rows p_j dout_row.
//   dq kernel:  one wavefront per query row (b,i,h): a sweep with one visible key per lane for
//               ds_j, then one output column per lane for the sum over keys.
//   dkv kernel: one wavefront per suffix key row (b,j,kv head): it visits the query rows i >= j
//               of the G query heads that share the KV head; each lane owns output columns.
// The forward pass's lse and out are taken as given (out only through <dout_row, out_row>).
// Arithmetic: fp64 when the tensors are f32, fp32 when they are bf16; any head dimension up
// to 256 and any GQA group size.
#include "pskv_internal.h"

namespace pskv {

namespace {

__device__ inline float load_as_float(const float *p) { return *p; }
__device__ inline float load_as_float(const unsigned short *p) { return __uint_as_float(((unsigned)*p) << 16); }
__device__ inline void store_from(float *p, double v) { *p = (float)v; }
__device__ inline void store_from(unsigned short *p, float v)
{
    unsigned u = __float_as_uint(v); // round to nearest even; NaN stays NaN
    if ((u & 0x7fffffffu) > 0x7f800000u) {
        *p = 0x7fc0;
        return;
    }
    u += 0x7fffu + ((u >> 16) & 1u);
    *p = (unsigned short)(u >> 16);
}
template <typename C> __device__ inline C wave_sum(C v)
{
    for (int off = 32; off > 0; off >>= 1)
        v += __shfl_xor(v, off, 64);
    return v;
}
__device__ inline float exp_c(float x) { return __expf(x); }
__device__ inline double exp_c(double x) { return exp(x); }

template <typename T, typename C>
__global__ __launch_bounds__(64) void bwd_dq_kernel(BwdArgs g)
{
    const Args &a = g.f;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    C *qs = reinterpret_cast<C *>(smem_raw); // [D]
    C *dos = qs + a.D;                       // [D]
    C *sc = dos + a.D;                       // [P + S]

    const int lane = threadIdx.x;
    const long long row = blockIdx.x; // (b*S + i)*Hq + h
    const int h = (int)(row % a.Hq);
    const long long bi = row / a.Hq;
    const int i = (int)(bi % a.S);
    const int b = (int)(bi / a.S);
    const int k = h / a.G;

    int len = a.len ? a.len[b] : a.S;
    len = len < 0 ? 0 : (len > a.S ? a.S : len);
    T *dq = reinterpret_cast<T *>(g.dq) + b * a.q_sb + i * a.q_ss + h * a.q_sh;
    if (i >= len) { // padded query row: no gradient
        for (int d = lane; d < a.D; d += 64)
            store_from(dq + d, (C)0);
        return;
    }
    const T *q = reinterpret_cast<const T *>(a.q) + b * a.q_sb + i * a.q_ss + h * a.q_sh;
    const T *o = reinterpret_cast<const T *>(a.out) + b * a.o_sb + i * a.o_ss + h * a.o_sh;
    const T *dor = reinterpret_cast<const T *>(g.dout) + b * a.o_sb + i * a.o_ss + h * a.o_sh;
    C drow = 0;
    for (int d = lane; d < a.D; d += 64) {
        qs[d] = (C)load_as_float(q + d);
        const C dv = (C)load_as_float(dor + d);
        dos[d] = dv;
        drow += dv * (C)load_as_float(o + d);
    }
    drow = wave_sum(drow); // <dout_row, out_row>
    const C lse = (C)a.lse[((long long)b * a.Hq + h) * a.S + i];
    __syncthreads();

    const T *kp = reinterpret_cast<const T *>(a.kp) + k * a.kp_sh;
    const T *vp = reinterpret_cast<const T *>(a.vp) + k * a.kp_sh;
    const T *ks = reinterpret_cast<const T *>(a.ks) + b * a.ks_sb + k * a.ks_sh;
    const T *vs = reinterpret_cast<const T *>(a.vs) + b * a.ks_sb + k * a.ks_sh;
    const int nvis = a.P + i + 1; // whole prefix, then suffix rows 0..i

    for (int j = lane; j < nvis; j += 64) {
        const T *kr = j < a.P ? kp + j * a.kp_sp : ks + (j - a.P) * a.ks_ss;
        const T *vr = j < a.P ? vp + j * a.kp_sp : vs + (j - a.P) * a.ks_ss;
        C s = 0, dp = 0;
        for (int d = 0; d < a.D; ++d) {
            s += qs[d] * (C)load_as_float(kr + d);
            dp += dos[d] * (C)load_as_float(vr + d);
        }
        const C p = exp_c(s * (C)a.scale - lse);
        sc[j] = p * (dp - drow);
    }
    __syncthreads();
    for (int d = lane; d < a.D; d += 64) {
        C acc = 0;
        for (int j = 0; j < a.P; ++j)
            acc += sc[j] * (C)load_as_float(kp + j * a.kp_sp + d);
        for (int t = 0; t <= i; ++t)
            acc += sc[a.P + t] * (C)load_as_float(ks + t * a.ks_ss + d);
        store_from(dq + d, acc * (C)a.scale);
    }
}

template <typename T, typename C>
__global__ __launch_bounds__(64) void bwd_dkv_kernel(BwdArgs g)
{
    const Args &a = g.f;
    const int lane = threadIdx.x;
    const long long row = blockIdx.x; // (b*S + j)*Hkv + k
    const int k = (int)(row % a.Hkv);
    const long long bj = row / a.Hkv;
    const int j = (int)(bj % a.S);
    const int b = (int)(bj / a.S);

    int len = a.len ? a.len[b] : a.S;
    len = len < 0 ? 0 : (len > a.S ? a.S : len);
    T *dk = reinterpret_cast<T *>(g.dk) + b * a.ks_sb + j * a.ks_ss + k * a.ks_sh;
    T *dv = reinterpret_cast<T *>(g.dv) + b * a.ks_sb + j * a.ks_ss + k * a.ks_sh;
    constexpr int U = 4; // output columns per lane: D <= 256
    C kj[U], vj[U], dka[U], dva[U];
    const T *kr = reinterpret_cast<const T *>(a.ks) + b * a.ks_sb + j * a.ks_ss + k * a.ks_sh;
    const T *vr = reinterpret_cast<const T *>(a.vs) + b * a.ks_sb + j * a.ks_ss + k * a.ks_sh;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int d = lane + 64 * u;
        const bool in = d < a.D && j < len;
        kj[u] = in ? (C)load_as_float(kr + d) : (C)0;
        vj[u] = in ? (C)load_as_float(vr + d) : (C)0;
        dka[u] = 0;
        dva[u] = 0;
    }
    if (j < len) {
        for (int gq = 0; gq < a.G; ++gq) {
            const int h = k * a.G + gq;
            for (int i = j; i < len; ++i) { // the query rows that see suffix key j
                const T *q = reinterpret_cast<const T *>(a.q) + b * a.q_sb + i * a.q_ss + h * a.q_sh;
                const T *o = reinterpret_cast<const T *>(a.out) + b * a.o_sb + i * a.o_ss + h * a.o_sh;
                const T *dor = reinterpret_cast<const T *>(g.dout) + b * a.o_sb + i * a.o_ss + h * a.o_sh;
                C qv[U], dov[U];
                C s = 0, dp = 0, drow = 0;
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int d = lane + 64 * u;
                    const bool in = d < a.D;
                    qv[u] = in ? (C)load_as_float(q + d) : (C)0;
                    dov[u] = in ? (C)load_as_float(dor + d) : (C)0;
                    const C ov = in ? (C)load_as_float(o + d) : (C)0;
                    s += qv[u] * kj[u];
                    dp += dov[u] * vj[u];
                    drow += dov[u] * ov;
                }
                s = wave_sum(s);
                dp = wave_sum(dp);
                drow = wave_sum(drow);
                const C p = exp_c(s * (C)a.scale - (C)a.lse[((long long)b * a.Hq + h) * a.S + i]);
                const C ds = p * (dp - drow) * (C)a.scale;
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    dka[u] += ds * qv[u];
                    dva[u] += p * dov[u];
                }
            }
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int d = lane + 64 * u;
        if (d < a.D) {
            store_from(dk + d, dka[u]);
            store_from(dv + d, dva[u]);
        }
    }
}

} // namespace

size_t bwd_simple_lds_bytes(const Args &a, int dtype)
{
    const size_t c = dtype == 0 ? sizeof(double) : sizeof(float);
    return c * (2 * (size_t)a.D + (size_t)a.P + (size_t)a.S);
}

hipError_t launch_bwd_dq_simple(const BwdArgs &g, int dtype, hipStream_t stream)
{
    const Args &a = g.f;
    const long long rows = (long long)a.B * a.S * a.Hq;
    const size_t lds = bwd_simple_lds_bytes(a, dtype);
    if (dtype == 0)
        hipLaunchKernelGGL((bwd_dq_kernel<float, double>), dim3((unsigned)rows), dim3(64), lds, stream, g);
    else
        hipLaunchKernelGGL((bwd_dq_kernel<unsigned short, float>), dim3((unsigned)rows), dim3(64), lds, stream, g);
    return hipGetLastError();
}

hipError_t launch_bwd_dkv_simple(const BwdArgs &g, int dtype, hipStream_t stream)
{
    const Args &a = g.f;
    const long long rows = (long long)a.B * a.S * a.Hkv;
    if (dtype == 0)
        hipLaunchKernelGGL((bwd_dkv_kernel<float, double>), dim3((unsigned)rows), dim3(64), 0, stream, g);
    else
        hipLaunchKernelGGL((bwd_dkv_kernel<unsigned short, float>), dim3((unsigned)rows), dim3(64), 0, stream, g);
    return hipGetLastError();
}

} // namespace pskv
