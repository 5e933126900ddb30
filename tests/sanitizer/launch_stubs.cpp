// Stand-ins for the kernel launchers, linked with the host side of the C ABI (pskv_api.cpp) in the
// sanitizer build: that build exercises argument validation only and never reaches a launch, so
// every launcher just reports that there is no device.
#include "../../paper_2603_13420_amd/csrc/pskv_internal.h"

namespace pskv {
size_t bwd_simple_lds_bytes(const Args &a, int) { return (size_t)(a.P + a.S + 2 * a.D) * 8; }
size_t bwd_dkv_lds_bytes(const Args &a, int) { return (size_t)a.G * a.S * 8; }
size_t simple_lds_bytes(const Args &a, int) { return (size_t)(a.P + a.S + a.D) * 8; }
hipError_t launch_bwd_dq_simple(const BwdArgs &, int, hipStream_t) { return hipErrorNoDevice; }
hipError_t launch_bwd_dkv_simple(const BwdArgs &, int, hipStream_t) { return hipErrorNoDevice; }
bool bwd_mfma_supported(const Args &a, int dtype) { return mfma_supported(a, dtype); }
hipError_t noalloc_scratch(void **) { return hipErrorNoDevice; }
hipError_t launch_bwd_dq_mfma(const BwdArgs &, hipStream_t) { return hipErrorNoDevice; }
hipError_t launch_bwd_dkv_mfma(const BwdArgs &, hipStream_t) { return hipErrorNoDevice; }
hipError_t launch_simple(const Args &, int, hipStream_t) { return hipErrorNoDevice; }
bool mfma_supported(const Args &a, int dtype) { return dtype == 1 && a.D == 128; }
hipError_t launch_mfma(const Args &, hipStream_t) { return hipErrorNoDevice; }
bool resident_supported(const Args &a) { return a.P <= 256; }
hipError_t launch_resident(const Args &, hipStream_t) { return hipErrorNoDevice; }
hipError_t launch_stream(const Args &, hipStream_t) { return hipErrorNoDevice; }
} // namespace pskv
