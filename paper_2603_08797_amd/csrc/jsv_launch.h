// Entry points of the kernel translation unit, called by the host planner.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "jsv_device.h"

namespace jsv {

size_t prune_lds_bytes(uint32_t c_max);
size_t mix_lds_bytes(uint32_t c_max);
size_t enumerate_lds_bytes(uint32_t t_max, uint32_t k_max);

// cost table + prune (mixture mode: options + prune), then plan (with the tile scan): two
// launches on `stream`
hipError_t launch_prune_plan_scan(const Plan& pl, hipStream_t stream);
// which instantiation of the enumeration kernel a search runs
int enumerate_mode(bool objective, bool mixtures);
hipError_t enumerate_blocks_per_cu(uint32_t t_max, uint32_t k_max, int mode, bool bounds, int* blocks);
// pl.grid blocks, as many as enumerate_blocks_per_cu says are resident at once (more would only start later)
hipError_t launch_enumerate(const Plan& pl, hipStream_t stream);
hipError_t launch_finalize(const Plan& pl, hipStream_t stream);
// all pointers are device pointers; pl.inst / pl.entries address ONE instance
hipError_t launch_eval(const Plan& pl, const uint64_t* index, uint32_t n, uint32_t* latency,
                       uint32_t* replicas, int32_t* cost, double* accuracy, uint8_t* mask,
                       uint32_t* bad, hipStream_t stream);

}  // namespace jsv
