// Optional instrumentation of the layer kernel, compiled in only with -DDSVT_PHASE_CLOCKS (the library that
// `python -m paper_2301_06051_amd.phase_clocks` builds beside the product library; the product build has none of
// it): thread 0 of every workgroup notes the shader clock at the kernel's phase boundaries, and
// dsvt_debug_phase_clocks copies the notes of the last launch to the host.  Not part of the C-ABI in dsvt.h.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#ifdef DSVT_PHASE_CLOCKS
constexpr int kPhaseSlots = 12, kPhaseBlocks = 2048;
__device__ unsigned long long dsvt_phase_clk[kPhaseBlocks][kPhaseSlots];
#define DSVT_PHASE(i)                                                                                    \
  do {                                                                                                   \
    if (threadIdx.x == 0 && blockIdx.x < (unsigned)kPhaseBlocks) dsvt_phase_clk[blockIdx.x][i] = clock64(); \
  } while (0)
// out: [kPhaseBlocks][kPhaseSlots] shader-clock values (host memory); synchronises the device first.
extern "C" int dsvt_debug_phase_clocks(unsigned long long* out, int32_t* blocks, int32_t* slots) {
  if (!out || !blocks || !slots) return -1;
  *blocks = kPhaseBlocks;
  *slots = kPhaseSlots;
  if (hipDeviceSynchronize() != hipSuccess) return -3;
  return hipMemcpyFromSymbol(out, HIP_SYMBOL(dsvt_phase_clk), sizeof(unsigned long long) * kPhaseBlocks * kPhaseSlots) == hipSuccess ? 0 : -3;
}
#else
#define DSVT_PHASE(i) do {} while (0)
#endif
