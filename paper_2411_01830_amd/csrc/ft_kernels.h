// Launchers of the HIP kernels (defined in ft_kernels.hip), private to the library.
#pragma once
#include <hip/hip_runtime_api.h>

#include "ft_tables.h"

namespace ft {

// Persistent copy kernel of one link class (0 host->pool, 1 pool->host, 2 pool->pool).
// *T.ticket must be zero when it starts. ev_start / ev_stop (both or neither)
// are timing events that will read the start and the end of this dispatch.
hipError_t launch_copy(const ClassTable &T, int link_class, uint32_t workgroups, hipStream_t stream,
                       hipEvent_t ev_start, hipEvent_t ev_stop);
// Decode every chunk rank with the device function the copy kernel uses (test hook).
hipError_t launch_decode(const ClassTable &T, uint32_t *func_out, uint32_t *chunk_out, uint64_t cap,
                         hipStream_t stream);
// Plain grid-stride copy, no tickets and no tables.
hipError_t launch_plain_copy(void *dst, const void *src, uint64_t bytes, uint32_t workgroups, hipStream_t stream);

}  // namespace ft
