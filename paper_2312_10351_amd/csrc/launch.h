// Interface between the kernel translation unit and the graph capturer.
#pragma once
#include <hip/hip_runtime.h>
#include "kernel_args.h"

namespace opara {
hipError_t launch_plan(const KernelPlan &p, hipStream_t s);
const void *kernel_symbol(int kernel_id);
}  // namespace opara
