// Stand-ins for the kernel launch functions in host-only sanitizer builds of the library (the CPU
// tests build kvfs.cpp, desc.cpp, sched.cpp and capi.cpp with g++ -fsanitize=... and run the host
// tests against that build): a host-only context never launches anything, so none of these is called.
#include "kernels.hpp"
namespace symkv {
hipError_t static_scratch_address(int, uint8_t**) { return hipErrorNotSupported; }
hipError_t launch_attn(const DecodeArgs&, const PrefillArgs&, int, int, hipStream_t, hipEvent_t, hipEvent_t) { return hipErrorNotSupported; }
hipError_t launch_merge(const MergeArgs&, int, int, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_prologue(PrologueArgs, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_gather(const GatherArgs&, void*, void*, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_move(const MoveArgs&, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_swap(const SwapArgs&, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_calib_read(const void*, int64_t, void*, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_calib_copy(void*, const void*, int64_t, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_calib_mfma(float*, int, int, hipStream_t) { return hipErrorNotSupported; }
}
