// Measurement helper of bench.py, built into a library of its own (libpskv_probe.so): it is not part
// of the attention library or of its ABI.  One kernel that does nothing but issue
// v_mfma_f32_32x32x16_bf16 on four independent accumulators per wavefront, two wavefronts per SIMD on
// every compute unit: the rate it reaches is what the matrix cores of THIS machine sustain under
// their own power and clock limits, the figure the attention kernels' achieved rate is set against
// next to the published peak.
#include <hip/hip_runtime.h>

typedef __bf16 probe_bf16x8 __attribute__((ext_vector_type(8)));
typedef float probe_floatx16 __attribute__((ext_vector_type(16)));

namespace {
constexpr int kMfmaPerIter = 16;

__global__ __attribute__((amdgpu_flat_work_group_size(512, 512), amdgpu_waves_per_eu(2, 2)))
void mfma_only_kernel(int iters, float *sink)
{
    probe_bf16x8 a, b;
    for (int i = 0; i < 8; ++i) {
        a[i] = (__bf16)(threadIdx.x * 0.001f + i);
        b[i] = (__bf16)(i * 0.5f);
    }
    probe_floatx16 c0 = {}, c1 = {}, c2 = {}, c3 = {};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < kMfmaPerIter / 4; ++u) {
            c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
            c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
            c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
            c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
        }
    }
    float s = 0.f;
    for (int i = 0; i < 16; ++i)
        s += c0[i] + c1[i] + c2[i] + c3[i];
    if (s == 12345.678f) // never true: keeps the accumulators alive
        sink[0] = s;
}
} // namespace

extern "C" {
// Enqueues one launch of the MFMA-only kernel on `hip_stream` (one workgroup of 8 wavefronts per compute
// unit, `iters` rounds of 16 matrix instructions per wavefront) and returns the HIP status.  sink: 4 bytes
// of device memory, never written.  *flops receives the matrix-core work of the launch (2 flop per
// multiply-add).
int pskv_probe_mfma_launch(int iters, float *sink, void *hip_stream, double *flops)
{
    int dev = 0, cus = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess)
        e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess)
        return (int)e;
    if (iters < 1 || !sink || !flops)
        return (int)hipErrorInvalidValue;
    *flops = (double)cus * 8.0 * iters * kMfmaPerIter * (2.0 * 32 * 32 * 16);
    void *args[] = {&iters, &sink};
    return (int)hipLaunchKernel(reinterpret_cast<const void *>(mfma_only_kernel), dim3(cus), dim3(512), args, 0,
                                static_cast<hipStream_t>(hip_stream));
}
}
