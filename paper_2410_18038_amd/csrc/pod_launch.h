// Host-callable launchers implemented in pod_kernels.hip.
#pragma once
#include <hip/hip_runtime_api.h>

#include "pod_common.h"

namespace pod {

enum LaunchKind : int { kLaunchPrefill = 0, kLaunchDecode = 1, kLaunchFused = 2, kLaunchCombine = 3, kLaunchFusedCta = 4,
                        kLaunchPrefillHeavy = 5, kLaunchDecodeLite = 6 };

// Enqueue one kernel of the given kind for (dtype, head_dim, layout) on `stream`.
hipError_t launch(int which, const KernelArgs &a, int dtype, int head_dim, bool paged, hipStream_t stream);
// Zero the counters at the head of a workspace.
hipError_t clear_header(WsHeader *hdr, hipStream_t stream);

// The library's own workspace for callers that may not allocate: a fixed array in device memory,
// one copy per GPU, held from the moment the library is loaded on that GPU until the process ends.
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
// Address of the current device's copy (looked up once per device, then remembered).
hipError_t static_scratch(void **ptr);

}  // namespace pod
