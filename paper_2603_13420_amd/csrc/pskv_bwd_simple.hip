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
//   dkv kernel: one wavefront per suffix key row (b,j,kv head): the query rows i >= j of the G
//               query heads that share the KV head, one per lane for ds and p, then one output
//               column per lane for the sums over those rows.
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

    // the candidate's instruction and its prefix: the last P of the a.P left-padded rows (Sec. 4.3, App. F.1)
    const int n = b / a.C;
    int P = a.P;
    if (a.plen) {
        P = a.plen[n];
        P = P < 0 ? 0 : (P > a.P ? a.P : P);
    }
    const long long pre_off = (long long)n * a.kp_sn + (long long)(a.P - P) * a.kp_sp + (long long)k * a.kp_sh;
    const T *kp = reinterpret_cast<const T *>(a.kp) + pre_off;
    const T *vp = reinterpret_cast<const T *>(a.vp) + pre_off;
    const T *ks = reinterpret_cast<const T *>(a.ks) + b * a.ks_sb + k * a.ks_sh;
    const T *vs = reinterpret_cast<const T *>(a.vs) + b * a.ks_sb + k * a.ks_sh;
    const int nvis = P + i + 1; // whole prefix, then suffix rows 0..i

    for (int j = lane; j < nvis; j += 64) {
        const T *kr = j < P ? kp + j * a.kp_sp : ks + (j - P) * a.ks_ss;
        const T *vr = j < P ? vp + j * a.kp_sp : vs + (j - P) * a.ks_ss;
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
        for (int j = 0; j < P; ++j)
            acc += sc[j] * (C)load_as_float(kp + j * a.kp_sp + d);
        for (int t = 0; t <= i; ++t)
            acc += sc[P + t] * (C)load_as_float(ks + t * a.ks_ss + d);
        store_from(dq + d, acc * (C)a.scale);
    }
}

// 16 bytes of a row as numbers: 8 bf16 or 4 f32 elements.
__device__ inline int load_vec(const unsigned short *p, float (&v)[8])
{
    const uint4 w = *reinterpret_cast<const uint4 *>(p);
    const unsigned u[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        v[2 * e] = __uint_as_float(u[e] << 16);
        v[2 * e + 1] = __uint_as_float(u[e] & 0xffff0000u);
    }
    return 8;
}
__device__ inline int load_vec(const float *p, float (&v)[8])
{
    const float4 w = *reinterpret_cast<const float4 *>(p);
    v[0] = w.x; v[1] = w.y; v[2] = w.z; v[3] = w.w;
    v[4] = v[5] = v[6] = v[7] = 0.f;
    return 4;
}

// dk_suf, dv_suf of one suffix key row (b, j, KV head).  The query rows that see the key are
// the pairs (query head of the group, i >= j); first one lane per pair computes that row's
// ds and p (three dot products over the head dimension with 16-byte loads, the key's K and V
// rows broadcast from LDS), then one lane per output column sums over the pairs.
template <typename T, typename C>
__global__ __launch_bounds__(64) void bwd_dkv_kernel(BwdArgs g)
{
    const Args &a = g.f;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    C *kj = reinterpret_cast<C *>(smem_raw); // [D]
    C *vj = kj + a.D;                        // [D]
    C *dss = vj + a.D;                       // [G*S]  scale * ds of each pair
    C *ps = dss + a.G * a.S;                 // [G*S]  p of each pair

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
    if (j >= len) { // padded suffix row: no gradient
        for (int d = lane; d < a.D; d += 64) {
            store_from(dk + d, (C)0);
            store_from(dv + d, (C)0);
        }
        return;
    }
    const T *kr = reinterpret_cast<const T *>(a.ks) + b * a.ks_sb + j * a.ks_ss + k * a.ks_sh;
    const T *vr = reinterpret_cast<const T *>(a.vs) + b * a.ks_sb + j * a.ks_ss + k * a.ks_sh;
    for (int d = lane; d < a.D; d += 64) {
        kj[d] = (C)load_as_float(kr + d);
        vj[d] = (C)load_as_float(vr + d);
    }
    __syncthreads();
    const int nrow = len - j;         // query rows i = j .. len-1 see suffix key j
    const int npairs = a.G * nrow;    // for each of the G query heads of the group
    for (int pr = lane; pr < npairs; pr += 64) {
        const int gq = pr / nrow, i = j + pr - gq * nrow, h = k * a.G + gq;
        const T *q = reinterpret_cast<const T *>(a.q) + b * a.q_sb + i * a.q_ss + h * a.q_sh;
        const T *o = reinterpret_cast<const T *>(a.out) + b * a.o_sb + i * a.o_ss + h * a.o_sh;
        const T *dor = reinterpret_cast<const T *>(g.dout) + b * a.o_sb + i * a.o_ss + h * a.o_sh;
        C s = 0, dp = 0, drow = 0;
        for (int d = 0; d < a.D;) {
            float qv[8], dov[8], ov[8];
            const int n = load_vec(q + d, qv);
            load_vec(dor + d, dov);
            load_vec(o + d, ov);
            for (int e = 0; e < n; ++e) {
                s += (C)qv[e] * kj[d + e];
                dp += (C)dov[e] * vj[d + e];
                drow += (C)dov[e] * (C)ov[e];
            }
            d += n;
        }
        const C p = exp_c(s * (C)a.scale - (C)a.lse[((long long)b * a.Hq + h) * a.S + i]);
        dss[pr] = p * (dp - drow) * (C)a.scale;
        ps[pr] = p;
    }
    __syncthreads();
    for (int d = lane; d < a.D; d += 64) {
        C dka = 0, dva = 0;
        for (int pr = 0; pr < npairs; ++pr) {
            const int gq = pr / nrow, i = j + pr - gq * nrow, h = k * a.G + gq;
            dka += dss[pr] * (C)load_as_float(reinterpret_cast<const T *>(a.q) + b * a.q_sb + i * a.q_ss + h * a.q_sh + d);
            dva += ps[pr] * (C)load_as_float(reinterpret_cast<const T *>(g.dout) + b * a.o_sb + i * a.o_ss + h * a.o_sh + d);
        }
        store_from(dk + d, dka);
        store_from(dv + d, dva);
    }
}

} // namespace

size_t bwd_simple_lds_bytes(const Args &a, int dtype)
{
    const size_t c = dtype == 0 ? sizeof(double) : sizeof(float);
    return c * (2 * (size_t)a.D + (size_t)a.P + (size_t)a.S);
}

size_t bwd_dkv_lds_bytes(const Args &a, int dtype)
{
    const size_t c = dtype == 0 ? sizeof(double) : sizeof(float);
    return c * (2 * (size_t)a.D + 2 * (size_t)a.G * a.S);
}

hipError_t launch_bwd_dq_simple(const BwdArgs &g, int dtype, hipStream_t stream)
{
    const Args &a = g.f;
    const long long rows = (long long)a.B * a.S * a.Hq;
    const size_t lds = bwd_simple_lds_bytes(a, dtype);
    if (dtype == 0)
        return launch_kernel((bwd_dq_kernel<float, double>), dim3((unsigned)rows), dim3(64), lds, stream, g);
    else
        return launch_kernel((bwd_dq_kernel<unsigned short, float>), dim3((unsigned)rows), dim3(64), lds, stream, g);
}

hipError_t launch_bwd_dkv_simple(const BwdArgs &g, int dtype, hipStream_t stream)
{
    const Args &a = g.f;
    const long long rows = (long long)a.B * a.S * a.Hkv;
    const size_t lds = bwd_dkv_lds_bytes(a, dtype);
    if (dtype == 0)
        return launch_kernel((bwd_dkv_kernel<float, double>), dim3((unsigned)rows), dim3(64), lds, stream, g);
    else
        return launch_kernel((bwd_dkv_kernel<unsigned short, float>), dim3((unsigned)rows), dim3(64), lds, stream, g);
}

} // namespace pskv
