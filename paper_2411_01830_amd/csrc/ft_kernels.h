// Launchers of the HIP kernels (defined in ft_kernels.hip), private to the library.
#pragma once
#include <hip/hip_runtime_api.h>

#include "ft_tables.h"

namespace ft {

constexpr int kLightPoolToPool = 3;

// Persistent copy kernel of one link class (0 host->pool, 1 pool->host, 2 pool->pool), or
// kLightPoolToPool: the pool->pool class in the build of the kernel that moves blocks of 16 KiB
// instead of 64 KiB and leaves room for two workgroups per compute unit (jobs of short pitched
// rows, which memory latency bounds, not HBM).
// Workgroup b starts on ticket b, the counter *T.ticket hands out the following ones: it
// must be zero when the kernel starts unless workgroups >= the launch's tickets (then its
// value does not matter). ev_start / ev_stop (both, neither, or ev_stop alone) are events that will
// read the start and the end of this dispatch. `tables`: the job's tables when
// T.inline_tables is set, else null.
hipError_t launch_copy(const ClassTable &T, int link_class, uint32_t workgroups, hipStream_t stream,
                       hipEvent_t ev_start, hipEvent_t ev_stop, const InlineBlob *tables = nullptr);
// Decode every chunk rank with the device function the copy kernel uses (test hook).
hipError_t launch_decode(const ClassTable &T, uint32_t *func_out, uint32_t *chunk_out, uint64_t cap,
                         hipStream_t stream, const InlineBlob *tables = nullptr);
// Plain grid-stride copy, no tickets and no tables.
hipError_t launch_plain_copy(void *dst, const void *src, uint64_t bytes, uint32_t workgroups, hipStream_t stream);
hipError_t launch_plain_read(const void *src, uint64_t bytes, uint32_t workgroups, hipStream_t stream);
hipError_t launch_plain_fill(void *dst, uint64_t bytes, uint32_t word, uint32_t workgroups, hipStream_t stream);

}  // namespace ft
