// Host planning of one submit: validation, split by link class, per-function byte
// streams, and the phase/slot tables that encode the proportional chunk order of
// Sec. 6.1 (see ft_tables.h for the encoding).
#pragma once
#include <stdint.h>
#include <vector>

#include "../../include/faastube.h"
#include "ft_pool.h"
#include "ft_tables.h"

namespace ft {

struct HostWindow {
  uint64_t base;
  uint64_t bytes;
  bool pageable;  // ordinary host memory (FT_PAGEABLE), not device-visible pinned memory
};

struct ClassPlan {
  std::vector<Phase> phases;
  std::vector<Slot> slots;
  std::vector<Func> funcs;
  std::vector<Xfer> xfers;
  std::vector<uint32_t> chunk_desc;  // empty when the job has more chunks than kMaxChunkTable
  uint32_t desc_per = 1;             // entries per chunk in chunk_desc: 1, or tiles per chunk
  uint64_t nchunks = 0;
  uint64_t payload = 0;
};

struct SubmitPlan {
  ClassPlan cls[FT_NCLASS];
  std::vector<uint64_t> allocs;  // start offsets of the pool allocations referred to (unique)
  bool has_pageable = false;     // some source or destination is pageable host memory: needs the staging ring
};

// Phases and slots for the given functions (nchunks > 0, weight >= 1 each, ascending
// caller function id). Divides the weights by their gcd in place. FT_EINVAL if the
// slot tables would exceed kMaxSlots entries.
constexpr uint64_t kMaxSlots = 1ull << 22;
// Most entries the descriptor table per chunk or tile may have (4 bytes each); jobs with more
// chunks than this search the function's whole descriptor range instead.
constexpr uint64_t kMaxChunkTable = 1ull << 20;
int build_phases(std::vector<Func> &funcs, std::vector<Phase> &phases, std::vector<Slot> &slots,
                 uint64_t *nchunks_out);

// Full planning of a submit. Returns FT_OK or the first error in the documented order.
int plan_submit(SlabPool &pool, const std::vector<HostWindow> &windows, const ft_desc *descs,
                uint32_t ndesc, const uint32_t *weights, uint32_t nfunc, uint64_t chunk_bytes,
                uint32_t flags, SubmitPlan *out);

// Per function and chunk of the order, the descriptor holding the chunk's first stream
// byte - or, for a job with many descriptors per chunk, per tile the descriptor holding
// the tile's first byte (desc_per = tiles per chunk) - and per function a closing entry,
// its last descriptor. Left empty above kMaxChunkTable entries. Needs funcs, xfers and
// nchunks. plan_submit does not call it: the tile shape is chosen afterwards.
void build_chunk_table(ClassPlan &cp, uint64_t chunk_bytes, uint64_t tile_bytes, uint32_t tiles_per_chunk);

// Runs of empty tiles (past the end of each function's last chunk) for the given tile
// shape, in ticket order, and the number of tickets left once they are taken out.
void build_skips(const ClassPlan &cp, uint64_t chunk_bytes, uint64_t tile_bytes, uint32_t tiles_per_chunk,
                 std::vector<Skip> *skips, uint64_t *ntickets);

// Bytes per ticket and tickets per chunk for a chunk size and a wanted tile size.
void tile_shape(uint64_t chunk_bytes, uint64_t want_tile, uint64_t *tile_bytes, uint32_t *tiles_per_chunk);

}  // namespace ft
