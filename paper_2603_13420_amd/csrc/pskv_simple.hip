// Simple path of batched candidate-suffix attention: one wavefront per query row (b,i,h).
//
// It follows Eq. 2 of the paper literally over the visible keys - the real rows of the prefix
// K/V of the candidate's instruction (read in place, never expanded over candidates) and rows
// 0..i of the candidate's own suffix K/V - in three sweeps: scores (lane per key), max/exp/sum, and the
// weighted V sum (lane per output column, so V rows are read coalesced).
//
// Arithmetic type: fp64 when the tensors are f32 (this is the verification-grade path, whose
// results are the correctly rounded fp32 values up to a final rounding), fp32 when they are
// bf16.  It covers any head dimension up to 256 and any GQA group size, and is the path for
// the f32 dtype; bf16 problems normally take the MFMA path instead.
#include "pskv_internal.h"
#include <hip/hip_bf16.h>

namespace pskv {

namespace {

__device__ inline float load_as_float(const float *p) { return *p; }
__device__ inline float load_as_float(const unsigned short *p)
{
    return __uint_as_float(((unsigned)*p) << 16);
}
__device__ inline void store_from(float *p, double v) { *p = (float)v; }
__device__ inline void store_from(unsigned short *p, float v)
{
    // round to nearest even; NaN stays NaN
    unsigned u = __float_as_uint(v);
    if ((u & 0x7fffffffu) > 0x7f800000u) {
        *p = 0x7fc0;
        return;
    }
    u += 0x7fffu + ((u >> 16) & 1u);
    *p = (unsigned short)(u >> 16);
}

template <typename C> __device__ inline C wave_max(C v)
{
    for (int off = 32; off > 0; off >>= 1) {
        C o = __shfl_xor(v, off, 64);
        v = o > v ? o : v;
    }
    return v;
}
template <typename C> __device__ inline C wave_sum(C v)
{
    for (int off = 32; off > 0; off >>= 1)
        v += __shfl_xor(v, off, 64);
    return v;
}
__device__ inline float exp_c(float x) { return __expf(x); }
__device__ inline double exp_c(double x) { return exp(x); }
__device__ inline float log_c(float x) { return logf(x); }
__device__ inline double log_c(double x) { return log(x); }

// T: storage element (float or bf16 bits), C: arithmetic type.
template <typename T, typename C>
__global__ __launch_bounds__(64) void simple_kernel(Args a)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    C *qs = reinterpret_cast<C *>(smem_raw); // [D]
    C *sc = qs + a.D;                        // [P + S]

    const int lane = threadIdx.x;
    const long long row = blockIdx.x; // (b*S + i)*Hq + h
    const int h = (int)(row % a.Hq);
    const long long bi = row / a.Hq;
    const int i = (int)(bi % a.S);
    const int b = (int)(bi / a.S);
    const int k = h / a.G;

    int len = a.len ? a.len[b] : a.S;
    len = len < 0 ? 0 : (len > a.S ? a.S : len);

    T *o = reinterpret_cast<T *>(a.out) + b * a.o_sb + i * a.o_ss + h * a.o_sh;
    if (i >= len) { // padded query row: defined as zero
        for (int d = lane; d < a.D; d += 64)
            store_from(o + d, (C)0);
        if (a.lse && lane == 0)
            a.lse[((long long)b * a.Hq + h) * a.S + i] = -INFINITY;
        return;
    }

    const T *q = reinterpret_cast<const T *>(a.q) + b * a.q_sb + i * a.q_ss + h * a.q_sh;
    for (int d = lane; d < a.D; d += 64)
        qs[d] = (C)load_as_float(q + d);
    __syncthreads();

    // the real prefix rows of the candidate's instruction: the last P of its a.P left-padded rows
    const int n = b / a.C;
    int P = a.plen ? a.plen[n] : a.P;
    P = P < 0 ? 0 : (P > a.P ? a.P : P);
    const long long poff = n * a.kp_sn + (long long)(a.P - P) * a.kp_sp + k * a.kp_sh;
    const T *kp = reinterpret_cast<const T *>(a.kp) + poff;
    const T *vp = reinterpret_cast<const T *>(a.vp) + poff;
    const T *ks = reinterpret_cast<const T *>(a.ks) + b * a.ks_sb + k * a.ks_sh;
    const T *vs = reinterpret_cast<const T *>(a.vs) + b * a.ks_sb + k * a.ks_sh;
    const int nvis = P + i + 1; // the instruction's real prefix rows, then suffix rows 0..i

    // sweep 1: scaled scores, one key per lane
    C mx = -INFINITY;
    for (int j = lane; j < nvis; j += 64) {
        const T *kr = j < P ? kp + j * a.kp_sp : ks + (j - P) * a.ks_ss;
        C acc = 0;
        for (int d = 0; d < a.D; ++d)
            acc += qs[d] * (C)load_as_float(kr + d);
        acc *= (C)a.scale;
        sc[j] = acc;
        mx = acc > mx ? acc : mx;
    }
    mx = wave_max(mx);

    // sweep 2: exponentials and their sum
    C den = 0;
    for (int j = lane; j < nvis; j += 64) {
        C e = exp_c(sc[j] - mx);
        sc[j] = e;
        den += e;
    }
    den = wave_sum(den);
    __syncthreads();

    // sweep 3: weighted sum of the visible V rows, one output column per lane
    for (int d = lane; d < a.D; d += 64) {
        C acc = 0;
        for (int j = 0; j < P; ++j)
            acc += sc[j] * (C)load_as_float(vp + j * a.kp_sp + d);
        for (int t = 0; t <= i; ++t)
            acc += sc[P + t] * (C)load_as_float(vs + t * a.ks_ss + d);
        store_from(o + d, acc / den);
    }
    if (a.lse && lane == 0)
        a.lse[((long long)b * a.Hq + h) * a.S + i] = (float)(mx + log_c(den));
}

} // namespace

size_t simple_lds_bytes(const Args &a, int dtype)
{
    const size_t c = dtype == 0 ? sizeof(double) : sizeof(float);
    return c * ((size_t)a.D + (size_t)a.P + (size_t)a.S);
}

hipError_t launch_simple(const Args &a, int dtype, hipStream_t stream)
{
    const long long rows = (long long)a.B * a.S * a.Hq;
    const dim3 grid((unsigned)rows), block(64);
    const size_t lds = simple_lds_bytes(a, dtype);
    if (dtype == 0)
        return launch_kernel((simple_kernel<float, double>), grid, block, lds, stream, a);
    else
        return launch_kernel((simple_kernel<unsigned short, float>), grid, block, lds, stream, a);
}

} // namespace pskv
