// Device-resident tables of one link class of one job, and the rank decoder.
//
// The chunk order of Sec. 6.1 (proportional interleave; stride reading: sort every
// chunk (f, j) by finish tag (j+1)/w_f, then by f) is not stored chunk by chunk.
// Chunk tags of different functions do not interact, so the order decomposes into
// rounds: round R holds the chunks whose tag lies in (R, R+1], i.e. chunks
// [R*w_f, (R+1)*w_f) of every function that still has them. While the set of
// functions that fill their whole share of a round stays the same, every round has
// the same slot pattern. The host therefore emits a few phases, each a run of rounds
// sharing one slot table, plus at most one single-round phase per function for the
// round in which it runs dry part-way. Decoding a chunk rank is a binary search over
// at most 2F+1 phases (the copy kernel, whose ranks only grow, keeps a cursor instead),
// one division and one table read.
//
// A second table lists, per function and chunk, the descriptor that holds the chunk's
// first stream byte, so that finding a tile's descriptor is a search over the few
// descriptors of one chunk instead of all descriptors of the function.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define FT_HD __host__ __device__ inline
#else
#define FT_HD inline
#endif

namespace ft {

struct Phase {
  uint64_t rank_base;   // rank (ticket / tiles_per_chunk) of the phase's first chunk
  uint64_t round_base;  // round number R of its first round
  uint32_t slot_off;    // first entry in the slot table
  uint32_t nslots;      // chunks per round in this phase (> 0)
};

struct Slot {
  uint32_t fl;         // index into the class's function table
  uint32_t i;          // chunk index inside the round: k = R * w + i
  uint32_t weight;     // copy of funcs[fl].weight: k is known after this one read
  uint32_t chunk_off;  // copy of funcs[fl].chunk_off
};

struct Func {
  uint64_t stream_bytes;  // S_f
  uint64_t nchunks;       // chunks in this order: ceil(S_f / C) - chunk_base
  uint32_t func;          // caller's function id
  uint32_t weight;        // w_f divided by the gcd of the class's weights
  uint32_t desc_off;      // first descriptor of this function in the class's table
  uint32_t ndesc;
  uint32_t chunk_off;     // first of the function's nchunks + 1 entries in the chunk table
  uint32_t _pad;
  uint64_t chunk_base;    // stream chunk that the function's chunk 0 of this order is: 0 unless
                          // the order was rebuilt when jobs joined (then: chunks triggered before)
};

// One transfer with both sides resolved to device-visible virtual addresses.
struct Xfer {
  uint64_t src;
  uint64_t dst;
  uint64_t row_bytes;
  uint64_t rows;       // 1 => contiguous (pitches unused)
  uint64_t src_pitch;
  uint64_t dst_pitch;
  uint64_t stream_off;  // payload bytes of the function's earlier descriptors
  uint64_t staged;      // kStagedSrc: src is pageable host memory that the device cannot read, the
                        // bytes reach it through the staging ring (see ClassTable::stage_base);
                        // kStagedDst: dst is pageable host memory, the device writes the ring
};
constexpr uint64_t kStagedSrc = 1, kStagedDst = 2;

// Tickets number only tiles that hold bytes. Tile v of the uniform grid (chunk rank
// v / tiles_per_chunk, tile v % tiles_per_chunk) is empty when it lies past the end of a
// function's last chunk; `at` is the first ticket at or after such a run of empty tiles
// and `gap` their number: v = t + the gaps of all entries with at <= t.
struct Skip {
  uint64_t at;
  uint64_t gap;
};

struct LogEntry {
  uint64_t t_begin;
  uint64_t t_end;
  uint32_t wg;  // workgroup that moved the ticket
  // what the copy kernel's own decode made of the ticket, written by the kernel: index into the
  // class's function table, chunk of that function's stream, stream bytes [b0, b1) of the tile
  uint32_t fl;
  uint64_t k;
  uint64_t b0, b1;
};

struct WgLogEntry {
  uint64_t t_entry;  // device clock when the workgroup started
  uint64_t t_exit;   // and when it found no ticket left
  uint32_t unit;     // the compute unit it ran on: die << 8 | shader engine << 5 | shader array << 4 | unit
  uint32_t _pad;
};

// Everything one class's kernel needs; passed by value as the kernel argument.
struct ClassTable {
  const Phase *phases;
  const Slot *slots;
  const Func *funcs;
  const Xfer *xfers;
  // per function nchunks * desc_per + 1 entries: the descriptor (index into xfers) holding
  // the first stream byte of each chunk (desc_per = 1) or of each tile (desc_per =
  // tiles_per_chunk; for jobs of many small descriptors, which then need no search), then
  // the function's last descriptor. Function fl's first entry is
  // (chunk_off - fl) * desc_per + fl. Null when the job has too many chunks for the table
  // to be worth its memory.
  const uint32_t *chunk_desc;
  const Skip *skips;           // ascending `at`
  unsigned long long *ticket;  // device counter, zero at launch
  LogEntry *log;               // one per ticket, or null
  WgLogEntry *wg_log;          // one per workgroup; set whenever log is
  uint64_t nchunks;            // N
  uint64_t ntickets;           // end of this launch's tickets (at most N * tiles_per_chunk minus
                               // the empty tiles)
  uint64_t ticket_base;        // first ticket of this launch: ticket = ticket_base + counter
  uint64_t skip_acc0;          // where the cursors stand at ticket_base: empty tiles before it,
  uint32_t skip0;              // index of the next run of empty tiles,
  uint32_t phase0;             // and the phase that holds its chunk
  // copies of phases[phase0], of the next phase's rank_base and of skips[skip0].at (all ones
  // where there is none): a workgroup's first decode starts without reading those tables
  Phase first_phase;
  uint64_t first_next_base;
  uint64_t first_skip_at;
  // Staging ring (pinned host memory, slots of chunk_bytes): chunk rank r of this launch has
  // slot stage_slot0 + (r - stage_rank0). The stream bytes of the chunk's staged descriptors
  // lie there, each at its offset inside the chunk: put there by the host before the launch
  // (pageable sources) or by the device for the host to take away after it (pageable
  // destinations).
  uint64_t stage_base;
  uint64_t stage_rank0;
  uint64_t stage_slot0;
  uint64_t chunk_bytes;        // C
  uint64_t tile_bytes;         // bytes per ticket, multiple of 16
  uint32_t tiles_per_chunk;
  uint32_t nphases;
  uint32_t nfuncs;
  uint32_t nskips;
  uint32_t desc_per;
  // 1: the table pointers above are byte offsets into the InlineBlob that the kernel
  // received as its second argument (a small job carries its tables in the launch itself)
  uint32_t inline_tables;
  // 1: ticket[0] is the counter and ticket[1] counts the workgroups that have finished; the
  // last one to finish sets both back to zero, so the pair serves the next launch that
  // gets it without anybody clearing it in between
  uint32_t self_reset;
  // 1: one function with one descriptor (xfers[0]) and no chunks triggered before: tile v
  // is stream bytes [v / tiles_per_chunk * chunk_bytes + v % tiles_per_chunk * tile_bytes, ...)
  // of that descriptor and ticket t is tile t, so the decode reads no schedule table.
  // 2: moreover the descriptor is contiguous, its two sides are multiples of 16
  // and nothing is logged: the workgroups deal the tiles out among themselves round robin.
  // 3: as 2, with ordinary instead of nontemporal loads and stores (a tensor small enough to
  // stay in the last-level cache between its producer and its consumer)
  uint32_t single;
};

// Tables of a small job, passed by value as a kernel argument next to the ClassTable.
constexpr uint32_t kInlineBytes = 3072;
struct InlineBlob {
  uint64_t w[kInlineBytes / 8];
};
static_assert(sizeof(ClassTable) % 8 == 0, "the InlineBlob argument follows the ClassTable without padding");

// Fills first_phase / first_next_base / first_skip_at from phase0 and skip0 (host side).
inline void set_cursor_start(ClassTable &T, const Phase *phases, uint32_t nphases, const Skip *skips,
                             uint32_t nskips) {
  T.first_phase = phases[T.phase0];
  T.first_next_base = T.phase0 + 1 < nphases ? phases[T.phase0 + 1].rank_base : ~0ull;
  T.first_skip_at = T.skip0 < nskips ? skips[T.skip0].at : ~0ull;
}

// Ticket -> tile of the uniform grid (host side; the copy kernel keeps a cursor).
inline uint64_t ticket_to_tile(const Skip *skips, uint32_t nskips, uint64_t t) {
  uint64_t v = t;
  for (uint32_t j = 0; j < nskips && skips[j].at <= t; ++j) v += skips[j].gap;
  return v;
}

struct ChunkId {
  uint32_t fl;  // index into funcs
  uint64_t k;   // chunk index within this order; the stream chunk is funcs[fl].chunk_base + k
};

// rank -> (function, chunk). rank < nchunks. The pointer types are template
// parameters so that the device can read the tables through constant-address-space
// pointers (scalar loads); only scalar members are read through them.
template <class PhaseP, class SlotP>
FT_HD ChunkId decode_rank(PhaseP phases, uint32_t nphases, SlotP slots, uint64_t rank) {
  uint32_t lo = 0, hi = nphases;  // last phase with rank_base <= rank
  while (hi - lo > 1) {
    uint32_t mid = (lo + hi) >> 1;
    if (phases[mid].rank_base <= rank) lo = mid; else hi = mid;
  }
  const uint64_t rel = rank - phases[lo].rank_base;
  const uint32_t nslots = phases[lo].nslots;
  const uint64_t round = rel / nslots;
  const uint32_t s = phases[lo].slot_off + (uint32_t)(rel - round * nslots);
  ChunkId id;
  id.fl = slots[s].fl;
  id.k = (phases[lo].round_base + round) * (uint64_t)slots[s].weight + slots[s].i;
  return id;
}

// Descriptor among [first, last] (one function's, stream_off ascending, xfers[first]
// at or before pos) that holds stream byte `pos`.
template <class XferP>
FT_HD uint32_t find_xfer(XferP xfers, uint32_t first, uint32_t last, uint64_t pos) {
  uint32_t lo = first, hi = last + 1;
  while (hi - lo > 1) {
    uint32_t mid = (lo + hi) >> 1;
    if (xfers[mid].stream_off <= pos) lo = mid; else hi = mid;
  }
  return lo;
}

}  // namespace ft
