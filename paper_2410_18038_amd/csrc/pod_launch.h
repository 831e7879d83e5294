// Host-callable launchers implemented in pod_kernels.hip.
#pragma once
#include <hip/hip_runtime_api.h>

#include "pod_common.h"

namespace pod {

enum LaunchKind : int { kLaunchPrefill = 0, kLaunchDecode = 1, kLaunchFused = 2, kLaunchCombine = 3 };

// Enqueue one kernel of the given kind for (dtype, head_dim, layout) on `stream`.
hipError_t launch(int which, const KernelArgs &a, int dtype, int head_dim, bool paged, hipStream_t stream);
// Zero the counters at the head of a workspace.
hipError_t clear_header(WsHeader *hdr, hipStream_t stream);

}  // namespace pod
