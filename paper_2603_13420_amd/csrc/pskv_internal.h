// Internal declarations shared by the host entry points and the kernel translation units.
// Nothing in here is part of the public ABI (that is include/pskv.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <mutex>
#include <tuple>
#include <utility>

namespace pskv {

// A fully resolved problem: every stride filled in (elements), scale resolved, pointers typed
// by the launcher. Passed to kernels by value.
// Exact unsigned division by a runtime constant d for numerators below 2^31:
// n / d == (n * mul) >> shift, with shift = 31 + ceil(log2 d) and mul = ceil(2^shift / d).
struct FastDiv {
    unsigned mul, shift;
};
inline FastDiv make_fastdiv(unsigned d)
{
    unsigned s = 0;
    while ((1ull << s) < d)
        ++s;
    FastDiv f;
    f.shift = 31 + s;
    f.mul = (unsigned)(((1ull << f.shift) + d - 1) / d);
    return f;
}

struct Args {
    int B, S, P, Hq, Hkv, D, G;
    // Batched multi-instruction form (Sec. 4.3): Np instructions with C = B / Np consecutive
    // candidates each; the prefix tensors are [Np, P, Hkv, D], every prefix LEFT-padded to P rows
    // with plen[n] real rows at the end.  Np == 1, plen == nullptr is the single shared prefix.
    int Np, C;
    const int *plen; // may be null: every prefix has P real rows
    long long kp_sn; // elements from one instruction's prefix to the next
    FastDiv div_g, div_s; // division by G and by S
    float scale;
    const void *q, *ks, *vs, *kp, *vp;
    const int *len; // may be null: every candidate has S rows
    void *out;
    float *lse; // may be null
    long long q_sb, q_ss, q_sh;
    long long ks_sb, ks_ss, ks_sh;
    long long kp_sp, kp_sh;
    long long o_sb, o_ss, o_sh;
};

// Whether one candidate's part of q, of out and of the suffix K/V each spans less than 2^31
// bytes (16-bit elements), so that kernels may address rows within a candidate by 32-bit offsets.
inline bool block_offsets_fit(const Args &a)
{
    const long long lim = 0x7fffffffLL / 2;
    return a.S * a.q_ss + a.Hq * a.q_sh < lim && a.S * a.o_ss + a.Hq * a.o_sh < lim && a.S * a.ks_ss + a.Hkv * a.ks_sh < lim;
}

// Backward pass: the forward problem (f.out and f.lse are the forward results, read-only here),
// the incoming gradient dout (laid out like out) and the three outputs (dq like q; dk, dv like
// k_suf, v_suf).
struct BwdArgs {
    Args f;
    const void *dout;
    void *dq, *dk, *dv;
    // Optional [B,Hq,S] floats (laid out like lse) in the caller's workspace: the matrix-core dq
    // kernels leave <dout_row, out_row> of every row they process there and the dk/dv kernel, which
    // runs after them on the same stream, takes it from there instead of reading out again.
    float *delta;
};
size_t bwd_simple_lds_bytes(const Args &a, int dtype);
size_t bwd_dkv_lds_bytes(const Args &a, int dtype);
hipError_t launch_bwd_dq_simple(const BwdArgs &g, int dtype, hipStream_t stream);
hipError_t launch_bwd_dkv_simple(const BwdArgs &g, int dtype, hipStream_t stream);
// Matrix-core kernels for dq and for dk/dv: bf16, D == 128 (prefixes of up to 256 rows stay resident
// in LDS for dq, longer ones are streamed).
bool bwd_mfma_supported(const Args &a, int dtype);
// Scratch for callers that cannot allocate: a fixed array in device memory that is part of the
// library's code object.  noalloc_scratch() hands out its address on the current device (looked
// up once per device: every device holds its own copy at its own address).
constexpr size_t kNoAllocScratchBytes = 8u << 20;
hipError_t noalloc_scratch(void **ptr);
hipError_t launch_bwd_dq_mfma(const BwdArgs &g, hipStream_t stream);
hipError_t launch_bwd_dkv_mfma(const BwdArgs &g, hipStream_t stream);

// Simple path: one wavefront per query row. dtype 0 = f32 storage (fp64 arithmetic),
// 1 = bf16 storage (fp32 arithmetic). Returns the HIP launch status.
hipError_t launch_simple(const Args &a, int dtype, hipStream_t stream);
// Largest dynamic LDS the simple path needs for this problem, in bytes.
size_t simple_lds_bytes(const Args &a, int dtype);

// MFMA path: bf16, D == 128.  Prefixes of up to 256 rows take the kernel that keeps the whole
// prefix K/V of one head resident in LDS; longer ones are streamed through LDS in tiles.
bool mfma_supported(const Args &a, int dtype);
hipError_t launch_mfma(const Args &a, hipStream_t stream);
bool resident_supported(const Args &a);
hipError_t launch_resident(const Args &a, hipStream_t stream);
hipError_t launch_stream(const Args &a, hipStream_t stream);

// One-time set-up per device and source file: `slots` is that file's table of compute-unit
// counts by device number (zero = not set up yet), `setup()` raises the LDS limits of the file's
// kernels on the current device.  Returns the current device's compute-unit count, 0 with e set
// on failure (the next call tries again).  Host threads that meet in the first call on a device
// are serialised by the table's mutex: one of them does the set-up, the others find it done.
constexpr int kMaxDevices = 64;
struct DeviceSlots {
    std::mutex mu;
    int cu[kMaxDevices] = {};
};
template <typename F>
inline int device_setup_once(DeviceSlots &slots, hipError_t &e, F setup)
{
    int dev = 0;
    e = hipGetDevice(&dev);
    if (e != hipSuccess)
        return 0;
    if (dev < 0 || dev >= kMaxDevices) {
        e = hipErrorInvalidDevice;
        return 0;
    }
    std::lock_guard<std::mutex> guard(slots.mu);
    if (slots.cu[dev] == 0) {
        int n = 0;
        e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
        if (e == hipSuccess)
            e = setup();
        if (e != hipSuccess)
            return 0;
        slots.cu[dev] = n > 0 ? n : 256;
    }
    return slots.cu[dev];
}

// Launches `kernel` and returns the status of THIS launch (hipLaunchKernel reports it directly), so
// that an error left behind by earlier, unrelated HIP activity of the caller is neither picked up
// nor cleared, as reading the thread's last-error slot after the launch would.
template <typename... KArgs, size_t... I>
inline hipError_t launch_kernel_impl(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds, hipStream_t stream,
                                     std::tuple<KArgs...> &vals, std::index_sequence<I...>)
{
    void *ptrs[] = {static_cast<void *>(&std::get<I>(vals))...};
    return hipLaunchKernel(reinterpret_cast<const void *>(kernel), grid, block, ptrs, lds, stream);
}
template <typename... KArgs, typename... Args>
inline hipError_t launch_kernel(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds, hipStream_t stream, Args... args)
{
    static_assert(sizeof...(KArgs) == sizeof...(Args), "argument count does not match the kernel's");
    std::tuple<KArgs...> vals{static_cast<KArgs>(args)...};
    return launch_kernel_impl(kernel, grid, block, lds, stream, vals, std::index_sequence_for<KArgs...>{});
}

} // namespace pskv
