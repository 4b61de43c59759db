// HIP kernels of the transfer engine for gfx950 (CDNA4, 64-wide wavefronts).
//
// ft_copy_kernel is the whole device side of Sec. 5.1 / 6.1 for one link class:
// persistent workgroups draw tickets from one device counter; a ticket names a tile
// of a chunk, chunks are numbered in the proportional order of Sec. 6.1, so the
// counter hands the link's bandwidth out to functions by weight at tile granularity.
// Bytes move as 16-byte vectors, one per lane, consecutive lanes on consecutive
// vectors, so every wavefront load/store covers 1 KiB of contiguous memory.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include "ft_kernels.h"

namespace ft {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// The job's tables are written before the launch and never during it. Reading them
// through constant-address-space pointers lets uniform reads go through the scalar
// unit and its cache, which the streaming vector traffic does not evict.
#define FT_CONST __attribute__((address_space(4)))
typedef const FT_CONST Phase *CPhaseP;
typedef const FT_CONST Slot *CSlotP;
typedef const FT_CONST Func *CFuncP;
typedef const FT_CONST Xfer *CXferP;
typedef const FT_CONST Skip *CSkipP;

struct ConstTables {
  CPhaseP phases;
  CSlotP slots;
  CFuncP funcs;
  CXferP xfers;
  CSkipP skips;
  const FT_CONST uint32_t *chunk_desc;  // null if the job has none
};

// The tables as constant-address-space pointers. A small job's tables came with the launch:
// they lie in the kernel-argument segment, behind the ClassTable, and T holds offsets.
__device__ __forceinline__ ConstTables const_tables(const ClassTable &T) {
  uintptr_t base = 0;
  if (T.inline_tables)
    base = reinterpret_cast<uintptr_t>(__builtin_amdgcn_kernarg_segment_ptr()) + sizeof(ClassTable);
  ConstTables c;
  c.phases = reinterpret_cast<CPhaseP>(base + reinterpret_cast<uintptr_t>(T.phases));
  c.slots = reinterpret_cast<CSlotP>(base + reinterpret_cast<uintptr_t>(T.slots));
  c.funcs = reinterpret_cast<CFuncP>(base + reinterpret_cast<uintptr_t>(T.funcs));
  c.xfers = reinterpret_cast<CXferP>(base + reinterpret_cast<uintptr_t>(T.xfers));
  c.skips = reinterpret_cast<CSkipP>(base + reinterpret_cast<uintptr_t>(T.skips));
  c.chunk_desc = T.chunk_desc != nullptr  // as an offset it is never 0: the phases come first
                     ? reinterpret_cast<const FT_CONST uint32_t *>(base + reinterpret_cast<uintptr_t>(T.chunk_desc))
                     : nullptr;
  return c;
}

__device__ __forceinline__ Xfer read_xfer(CXferP xfers, uint32_t x) {
  Xfer X;
  X.src = xfers[x].src;
  X.dst = xfers[x].dst;
  X.row_bytes = xfers[x].row_bytes;
  X.rows = xfers[x].rows;
  X.src_pitch = xfers[x].src_pitch;
  X.dst_pitch = xfers[x].dst_pitch;
  X.stream_off = xfers[x].stream_off;
  X.staged = xfers[x].staged;
  return X;
}

constexpr uint32_t kThreads = 256;  // 4 wavefronts per workgroup, one workgroup per CU for pool->pool
// U, a template parameter of the copy routines: 16-byte loads a lane has in flight before
// its first store, so a workgroup moves blocks of 256 lanes x U x 16 B. pool->pool uses
// U = 16 (64 KiB blocks, the whole tile in registers). The host-link classes use U = 4:
// their tiles are 8-16 KiB, and the smaller register footprint lets a host-link
// workgroup share a CU with a pool->pool workgroup instead of taking the CU for itself.
// CLS 3 (kLightPoolToPool) is pool->pool with U = 4: two such workgroups fit a CU.
template <int CLS>
struct UnrollOf {
  static constexpr uint32_t value = CLS == 2 ? 16u : 4u;
};

// Every payload address (pool memory or pinned host memory) is a global-segment
// address. Saying so keeps the copies off the flat path, whose loads also count on
// the scalar/LDS wait counter and would serialise with the table reads.
#define FT_GLOBAL __attribute__((address_space(1)))
typedef u32x4 FT_GLOBAL *GVecP;
typedef uint8_t FT_GLOBAL *GByteP;

// How a routine reaches memory, its first template parameter NT: 0 ordinary loads and stores (data that
// is wanted in the caches); kStream nontemporal loads and stores (payload streaming through HBM once);
// kToHost nontemporal loads and stores that are written through to the fabric at once (the `sc1` bit)
// for destinations in host memory. A nontemporal or ordinary store to host memory stays in the L2 until
// that evicts it or the kernel ends: the tiny workload's pool->host kernel had every store issued after
// 260 us and then ended 80 us later, when the L2 had written its lines back over the link (50 GB/s);
// written through, the link carries them while the kernel runs (55 GB/s, what host->pool reaches on the
// same buffers). `sc0 sc1` measured 53.4 GB/s, `sc0 sc1 nt` 53.5. Towards HBM every other combination
// of the bits is slower than `nt` alone.
constexpr int kStream = 1, kToHost = 2;

template <int NT>
__device__ __forceinline__ u32x4 ld16(uint64_t addr) {
  if (NT) return __builtin_nontemporal_load(reinterpret_cast<const u32x4 FT_GLOBAL *>(addr));
  return *reinterpret_cast<const u32x4 FT_GLOBAL *>(addr);
}
// 16 bytes from any address (the hardware splits an access that straddles aligned granules).
typedef uint32_t u32x4_any __attribute__((ext_vector_type(4), aligned(1)));
template <int NT>
__device__ __forceinline__ u32x4 ld16_any(uint64_t addr) {
  if (NT) return __builtin_nontemporal_load(reinterpret_cast<const u32x4_any FT_GLOBAL *>(addr));
  return *reinterpret_cast<const u32x4_any FT_GLOBAL *>(addr);
}
template <int NT>
__device__ __forceinline__ void st16(uint64_t addr, u32x4 v) {
  if (NT == kToHost) asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(addr), "v"(v) : "memory");
  else if (NT) __builtin_nontemporal_store(v, reinterpret_cast<GVecP>(addr));
  else *reinterpret_cast<GVecP>(addr) = v;
}
__device__ __forceinline__ uint8_t ld8(uint64_t addr) { return *reinterpret_cast<const uint8_t FT_GLOBAL *>(addr); }
__device__ __forceinline__ void st8(uint64_t addr, uint8_t v) { *reinterpret_cast<GByteP>(addr) = v; }

// 16 bytes starting `shift` (0..15, per lane) bytes into the 32-byte pair (A, B): select
// the five dwords by shift / 4 in two halving steps, then byte-align neighbours.
__device__ __forceinline__ u32x4 funnel(u32x4 A, u32x4 B, uint32_t shift) {
  const bool s1 = (shift & 4) != 0, s2 = (shift & 8) != 0;
  const uint32_t r = shift & 3;
  const uint32_t y0 = s1 ? A.y : A.x, y1 = s1 ? A.z : A.y, y2 = s1 ? A.w : A.z, y3 = s1 ? B.x : A.w;
  const uint32_t y4 = s1 ? B.y : B.x, y5 = s1 ? B.z : B.y, y6 = s1 ? B.w : B.z;
  const uint32_t z0 = s2 ? y2 : y0, z1 = s2 ? y3 : y1, z2 = s2 ? y4 : y2, z3 = s2 ? y5 : y3, z4 = s2 ? y6 : y4;
  u32x4 v;
  v.x = __builtin_amdgcn_alignbyte(z1, z0, r);
  v.y = __builtin_amdgcn_alignbyte(z2, z1, r);
  v.z = __builtin_amdgcn_alignbyte(z3, z2, r);
  v.w = __builtin_amdgcn_alignbyte(z4, z3, r);
  return v;
}

// Write the bytes [lo, hi) of v to the aligned granule at ga.
template <int NT>
__device__ __forceinline__ void store_granule(uint64_t ga, u32x4 v, uint32_t lo, uint32_t hi) {
  if (lo == 0 && hi == 16) {
    st16<NT>(ga, v);
  } else {
    for (uint32_t b = lo; b < hi; ++b) {
      const uint32_t w = (b >> 2) == 0 ? v.x : (b >> 2) == 1 ? v.y : (b >> 2) == 2 ? v.z : v.w;
      st8(ga + b, (uint8_t)(w >> ((b & 3) * 8)));
    }
  }
}

// Short rows of a pitched descriptor. A group of L lanes owns a row and every lane one
// destination granule (aligned 16 bytes) of it, so L >= granules per row. Each pass a
// group takes R rows: all 2*R aligned source loads are issued before the first store.
// Loads are never predicated - the address of a granule that holds no byte of the row
// is clamped into the row's own source range, and what it returns is never stored - so
// the code stays a straight line. Stores write only bytes of the destination range:
// whole granules with one vector store, the first and last of a row byte-wise.
template <int NT, uint32_t L, uint32_t R>
__device__ __forceinline__ void copy_rows_grouped(const Xfer &X, uint64_t r0, uint64_t c0, uint64_t rl, uint64_t cl,
                                                  uint32_t tid) {
  constexpr uint32_t kGroups = kThreads / L;
  const uint32_t g = tid / L, l = tid % L;
  const uint64_t rb = X.row_bytes;
  for (uint64_t base = r0; base <= rl; base += (uint64_t)kGroups * R) {
    u32x4 A[R], B[R];
    uint64_t ga[R];
    uint32_t lo[R], hi[R], sh[R];
#pragma unroll
    for (uint32_t k = 0; k < R; ++k) {
      uint64_t r = base + g + (uint64_t)k * kGroups;
      const bool valid = r <= rl;
      r = valid ? r : rl;
      const uint64_t ca = r == r0 ? c0 : 0, cb = r == rl ? cl : rb;
      const uint64_t d0 = X.dst + r * X.dst_pitch + ca, d1 = d0 + (cb - ca);
      const uint64_t s0 = X.src + r * X.src_pitch + ca, s1 = s0 + (cb - ca);
      const uint64_t first = s0 & ~15ull, last = (s1 - 1) & ~15ull;
      ga[k] = (d0 & ~15ull) + ((uint64_t)l << 4);
      const bool active = valid && ga[k] < d1;
      lo[k] = ga[k] < d0 ? (uint32_t)(d0 - ga[k]) : 0u;
      hi[k] = !active ? 0u : ga[k] + 16 > d1 ? (uint32_t)(d1 - ga[k]) : 16u;
      const uint64_t sa = ga[k] + (s0 - d0);
      sh[k] = (uint32_t)(sa & 15);
      uint64_t a0 = sa & ~15ull, a1 = a0 + 16;
      a0 = a0 < first ? first : a0 > last ? last : a0;
      a1 = a1 < first ? first : a1 > last ? last : a1;
      A[k] = ld16<NT>(a0);
      B[k] = ld16<NT>(a1);
    }
#pragma unroll
    for (uint32_t k = 0; k < R; ++k) {
      if (lo[k] < hi[k]) store_granule<NT>(ga[k], funnel(A[k], B[k], sh[k]), lo[k], hi[k]);
    }
  }
}

// R rows of kThreads aligned vectors each (R * 4 KiB), every lane issuing its R loads
// before its first store. No lane is predicated, so the code is one straight line and
// the loads are waited for once, not one by one.
template <int NT, uint32_t R>
__device__ __forceinline__ void copy_rows_of_vectors(uint64_t d, uint64_t s, uint32_t tid) {
  u32x4 v[R];
#pragma unroll
  for (uint32_t j = 0; j < R; ++j) v[j] = ld16<NT>(s + ((uint64_t)(tid + j * kThreads) << 4));
#pragma unroll
  for (uint32_t j = 0; j < R; ++j) st16<NT>(d + ((uint64_t)(tid + j * kThreads) << 4), v[j]);
}

// The same, and lane 0 draws the workgroup's next ticket on the way: the atomic is issued three quarters
// through the stores. Issued before the loads (its answer is not needed before the stores are out) it
// sat in front of them in the memory pipeline - no store could leave before the counter had answered,
// 2.2 us, however early the tile's data was there - and the workgroup held a ticket it had not started
// for a whole tile, which is what the end of a launch waits for. Issued here the answer still arrives
// while the stores drain (feature: 181.5 -> 178 us, the pool->pool launches of large_mixed 83.5 -> 82.5).
template <int NT, uint32_t R>
__device__ __forceinline__ unsigned long long copy_rows_of_vectors_draw(uint64_t d, uint64_t s, uint32_t tid,
                                                                        unsigned long long *ticket) {
  u32x4 v[R];
#pragma unroll
  for (uint32_t j = 0; j < R; ++j) v[j] = ld16<NT>(s + ((uint64_t)(tid + j * kThreads) << 4));
  unsigned long long claimed = 0;
#pragma unroll
  for (uint32_t j = 0; j < R; ++j) {
    if (j == R * 3 / 4 && tid == 0) claimed = atomicAdd(ticket, 1ull);
    st16<NT>(d + ((uint64_t)(tid + j * kThreads) << 4), v[j]);
  }
  return claimed;
}

// 1 <= nvec <= R * kThreads aligned vectors in one pass. Loads are never predicated: a
// lane whose vector lies past the end loads the last vector instead (and does not store
// it), so all R loads of a lane are in flight before its first store whatever nvec is.
template <int NT, uint32_t R>
__device__ __forceinline__ void copy_rows_clamped(uint64_t d, uint64_t s, uint32_t nvec, uint32_t tid) {
  u32x4 v[R];
  const uint32_t lastv = nvec - 1;
#pragma unroll
  for (uint32_t j = 0; j < R; ++j) {
    uint32_t i = tid + j * kThreads;
    i = i < lastv ? i : lastv;
    v[j] = ld16<NT>(s + ((uint64_t)i << 4));
  }
#pragma unroll
  for (uint32_t j = 0; j < R; ++j) {
    const uint32_t i = tid + j * kThreads;
    if (i < nvec) st16<NT>(d + ((uint64_t)i << 4), v[j]);
  }
}

// nvec aligned 16-byte vectors with the whole workgroup: full blocks of U rows, then one
// clamped pass over what is left.
template <int NT, uint32_t U>
__device__ __forceinline__ void copy_vectors(uint64_t d, uint64_t s, uint64_t nvec, uint32_t tid) {
  constexpr uint32_t kBlockVec = kThreads * U;
  while (nvec >= kBlockVec) {
    copy_rows_of_vectors<NT, U>(d, s, tid);
    d += (uint64_t)kBlockVec << 4;
    s += (uint64_t)kBlockVec << 4;
    nvec -= kBlockVec;
  }
  const uint32_t rest = (uint32_t)nvec;
  if (U > 4 && rest > 4 * kThreads) copy_rows_clamped<NT, U>(d, s, rest, tid);
  else if (rest > kThreads) copy_rows_clamped<NT, 4>(d, s, rest, tid);
  else if (rest > 0) copy_rows_clamped<NT, 1>(d, s, rest, tid);
}

// Lane i receives lane i+1's value of v; lane 63, which has no such neighbour, receives
// `last` (wave_shl:1 moves data one lane towards lane 0 and leaves the old value in a
// lane without a source). Must run with all 64 lanes enabled.
__device__ __forceinline__ uint32_t from_next_lane(uint32_t v, uint32_t last) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)last, (int)v, 0x130 /* wave_shl:1 */, 0xf, 0xf, false);
}

// 16 bytes starting 4*Q + r bytes into the 32-byte pair (A, next granule), where the
// next granule is the next lane's A, or for lane 63 lane 0's value of `nextrow`.
// Q and r are the same for a whole run, so every selection is fixed at compile time:
// Q+1 lane exchanges and four byte-aligns per vector.
template <uint32_t Q>
__device__ __forceinline__ u32x4 shifted_vector(u32x4 A, u32x4 nextrow, uint32_t r) {
  uint32_t c[8] = {A.x, A.y, A.z, A.w, 0u, 0u, 0u, 0u};
  c[4] = from_next_lane(A.x, __builtin_amdgcn_readfirstlane(nextrow.x));
  if (Q >= 1) c[5] = from_next_lane(A.y, __builtin_amdgcn_readfirstlane(nextrow.y));
  if (Q >= 2) c[6] = from_next_lane(A.z, __builtin_amdgcn_readfirstlane(nextrow.z));
  if (Q >= 3) c[7] = from_next_lane(A.w, __builtin_amdgcn_readfirstlane(nextrow.w));
  u32x4 v;
  v.x = __builtin_amdgcn_alignbyte(c[Q + 1], c[Q + 0], r);
  v.y = __builtin_amdgcn_alignbyte(c[Q + 2], c[Q + 1], r);
  v.z = __builtin_amdgcn_alignbyte(c[Q + 3], c[Q + 2], r);
  v.w = __builtin_amdgcn_alignbyte(c[Q + 4], c[Q + 3], r);
  return v;
}

// One pass over up to R * kThreads whole destination granules of a run whose destination
// is aligned and whose source is not. d, a: first destination granule of the pass and the
// aligned source granule under it; left: granules the run still has from here on (> 0).
// Destination granule i is made of source granules i and i+1, so the last source granule
// the run touches has index `left`.
// A wavefront owns R * 64 consecutive granules (row j = granules j*64 .. j*64+63): every
// lane loads the source granule under each of its destination granules and takes the
// following one from the next lane, lane 63 from lane 0 of the next row (the row after
// the last one is one more granule, loaded at the same address by all lanes). HBM traffic
// equals the aligned case, there is no barrier and nothing is parked in LDS. Loads are
// never predicated: an index past the run's last source granule is clamped to it and
// what it returns is never stored.
template <int NT, uint32_t R, uint32_t Q>
__device__ __forceinline__ void shifted_pass(uint64_t d, uint64_t a, uint32_t left, uint32_t r, uint32_t tid) {
  const uint32_t wave = tid >> 6, lane = tid & 63;
  const uint32_t wbase = wave * (R * 64);
  u32x4 A[R], N;
#pragma unroll
  for (uint32_t j = 0; j < R; ++j) {
    uint32_t gi = wbase + j * 64 + lane;
    gi = gi < left ? gi : left;
    A[j] = ld16<NT>(a + ((uint64_t)gi << 4));
  }
  {
    uint32_t gi = wbase + R * 64;
    gi = gi < left ? gi : left;
    N = ld16<NT>(a + ((uint64_t)gi << 4));
  }
#pragma unroll
  for (uint32_t j = 0; j < R; ++j) {
    // control flow is uniform across the workgroup up to here, so all 64 lanes take part
    // in the exchange; the per-lane choice comes after it
    const u32x4 v = shifted_vector<Q>(A[j], j + 1 < R ? A[j + 1] : N, r);
    const uint32_t gi = wbase + j * 64 + lane;
    if (gi < left) st16<NT>(d + ((uint64_t)gi << 4), v);
  }
}

// nfull whole destination granules from aligned d; s is the (unaligned) source of d.
template <int NT, uint32_t U, uint32_t Q>
__device__ __forceinline__ void copy_shifted_q(uint64_t d, uint64_t s, uint64_t nfull, uint32_t tid) {
  const uint32_t r = (uint32_t)s & 3;
  const uint64_t a_base = s & ~15ull;
  for (uint64_t blk = 0; blk < nfull;) {
    const uint64_t left64 = nfull - blk;
    const uint32_t left = left64 > 0x7fffffffull ? 0x7fffffffu : (uint32_t)left64;
    if (left > kThreads) {
      shifted_pass<NT, U, Q>(d + (blk << 4), a_base + (blk << 4), left, r, tid);
      blk += kThreads * U;
    } else {
      shifted_pass<NT, 1, Q>(d + (blk << 4), a_base + (blk << 4), left, r, tid);
      blk += kThreads;
    }
  }
}

// Source and destination differ in alignment: the bytes before the first and after the
// last whole destination granule go one by one, the granules between as aligned vectors
// built from shifted source granules.
template <int NT, uint32_t U>
__device__ __forceinline__ void copy_shifted(uint64_t d0, uint64_t s0, uint64_t n, uint32_t tid) {
  uint64_t head = (16 - (d0 & 15)) & 15;
  if (head > n) head = n;
  const uint64_t nfull = (n - head) >> 4;
  const uint64_t tail = (n - head) & 15;
  const uint64_t toff = head + (nfull << 4);
  // lanes 0..15 carry the head bytes, lanes 16..31 the tail bytes; they are loaded
  // before and stored after the body so that their latency is not paid on its own
  const bool edge = tid < head || (tid >= 16 && tid - 16 < tail);
  const uint64_t eoff = tid < 16 ? tid : toff + (tid - 16);
  uint8_t ev = 0;
  if (edge) ev = ld8(s0 + eoff);
  if (nfull != 0) {
    const uint64_t d = d0 + head, s = s0 + head;  // d is aligned, s is not
    switch (((uint32_t)s & 15) >> 2) {
      case 0: copy_shifted_q<NT, U, 0>(d, s, nfull, tid); break;
      case 1: copy_shifted_q<NT, U, 1>(d, s, nfull, tid); break;
      case 2: copy_shifted_q<NT, U, 2>(d, s, nfull, tid); break;
      default: copy_shifted_q<NT, U, 3>(d, s, nfull, tid); break;
    }
  }
  if (edge) st8(d0 + eoff, ev);
}

// One contiguous piece with the whole workgroup.
template <int NT, uint32_t U>
__device__ __forceinline__ void copy_piece(uint64_t d0, uint64_t s0, uint64_t n, uint32_t tid) {
  if (((d0 ^ s0) & 15) == 0) {
    if (n < 64) {
      if (tid < n) st8(d0 + tid, ld8(s0 + tid));
      return;
    }
    // same alignment on both sides: byte head up to the boundary, vector body, byte tail;
    // head and tail bytes are loaded before and stored after the body
    const uint64_t head = (16 - (d0 & 15)) & 15;
    const uint64_t nvec = (n - head) >> 4;
    const uint64_t tail = (n - head) & 15;
    const uint64_t toff = head + (nvec << 4);
    const bool edge = tid < head || (tid >= 16 && tid - 16 < tail);
    const uint64_t eoff = tid < 16 ? tid : toff + (tid - 16);
    uint8_t ev = 0;
    if (edge) ev = ld8(s0 + eoff);
    copy_vectors<NT, U>(d0 + head, s0 + head, nvec, tid);
    if (edge) st8(d0 + eoff, ev);
  } else {
    copy_shifted<NT, U>(d0, s0, n, tid);
  }
}

// Dword d of a 16-byte vector whose bytes at positions >= split come from b, the rest from a.
__device__ __forceinline__ uint32_t merge_dword(uint32_t a, uint32_t b, uint32_t split, uint32_t d) {
  const uint32_t first = 4 * d;
  const uint32_t m = split <= first ? 0xffffffffu : split >= first + 4 ? 0u : 0xffffffffu << (8 * (split - first));
  return (b & m) | (a & ~m);
}

// The gather of the host-link classes, with aligned loads only (the source may be host memory,
// where an access that straddles granules is two requests on the link). Rows gathered into a
// contiguous destination (dst_pitch == row_bytes >= 16): payload
// bytes [p, p+take), take < 2^30, land in one run of destination bytes, so every lane
// owns whole destination granules and only the first and last granule of the run are
// partial. A granule holds bytes of at most two source rows: for each of the two pieces
// a lane loads the two aligned source granules around it, funnels them into place and
// merges the pieces, R granules per lane and pass, all 4*R loads before the first store.
// Loads are never predicated: an address outside the aligned granules that hold bytes of
// its piece is clamped into them and what it returns is never stored; a granule without
// a second piece repeats the first piece's addresses.
template <int NT, uint32_t R>
__device__ __forceinline__ void copy_rows_packed_pairs(const Xfer &X, uint64_t p, uint64_t take, uint32_t tid) {
  const uint32_t rb = (uint32_t)X.row_bytes;
  const uint64_t d0 = X.dst + p, d1 = d0 + take;
  const uint64_t g0 = d0 & ~15ull;
  const uint32_t ngran = (uint32_t)((((d1 + 15) & ~15ull) - g0) >> 4);
  const uint32_t head = (uint32_t)(d0 - g0);  // bytes of the first granule before the run
  const uint64_t r_base = p / rb;
  const uint32_t c_base = (uint32_t)(p - r_base * rb);
  const uint64_t src_base = X.src + r_base * X.src_pitch;  // row r_base, column 0
  const uint32_t magic = (uint32_t)((1ull << 32) / rb) + 1;  // e / rb = mulhi(e, magic) or one less
  for (uint32_t blk = 0; blk < ngran; blk += R * kThreads) {
    u32x4 A0[R], A1[R], B0[R], B1[R];
    uint32_t meta[R];  // lo | hi << 5 | split << 10 | shift A << 15 | shift B << 20
#pragma unroll
    for (uint32_t k = 0; k < R; ++k) {
      uint32_t gi = blk + tid + k * kThreads;
      const bool active = gi < ngran;
      gi = active ? gi : ngran - 1;
      // bytes [lo, hi) of this granule belong to the run
      const uint32_t lo = gi == 0 ? head : 0u;
      const uint64_t gend = g0 + ((uint64_t)gi << 4) + 16;
      const uint32_t top = gend > d1 ? 16u - (uint32_t)(gend - d1) : 16u;
      const uint32_t hi = active ? top : lo;
      const uint32_t n = top - lo;
      // row (relative to r_base) and column of the granule's first run byte
      const uint32_t e = c_base + (gi << 4) + lo - head;
      uint32_t dr = __umulhi(e, magic);
      dr -= (dr * rb > e) ? 1u : 0u;
      const uint32_t c = e - dr * rb;
      const uint32_t nA = n < rb - c ? n : rb - c;
      const uint32_t nB = n - nA;
      const uint32_t split = lo + nA;
      const uint64_t sA = src_base + (uint64_t)dr * X.src_pitch + c;
      const uint64_t sB = nB ? src_base + (uint64_t)(dr + 1) * X.src_pitch : sA;
      const uint32_t lenB = nB ? nB : nA;
      const uint32_t posB = nB ? split : lo;
      // window of 16 bytes that puts piece A (B) at its place in the granule
      const uint64_t wA = sA - lo, wB = sB - posB;
      meta[k] = lo | hi << 5 | split << 10 | ((uint32_t)wA & 15) << 15 | ((uint32_t)wB & 15) << 20;
      const uint64_t fA = sA & ~15ull, lA = (sA + nA - 1) & ~15ull;
      const uint64_t fB = sB & ~15ull, lB = (sB + lenB - 1) & ~15ull;
      uint64_t a0 = wA & ~15ull, a1 = a0 + 16, b0 = wB & ~15ull, b1 = b0 + 16;
      a0 = a0 < fA ? fA : a0 > lA ? lA : a0;
      a1 = a1 < fA ? fA : a1 > lA ? lA : a1;
      b0 = b0 < fB ? fB : b0 > lB ? lB : b0;
      b1 = b1 < fB ? fB : b1 > lB ? lB : b1;
      A0[k] = ld16<NT>(a0);
      A1[k] = ld16<NT>(a1);
      B0[k] = ld16<NT>(b0);
      B1[k] = ld16<NT>(b1);
    }
#pragma unroll
    for (uint32_t k = 0; k < R; ++k) {
      const uint32_t lo = meta[k] & 31, hi = (meta[k] >> 5) & 31, split = (meta[k] >> 10) & 31;
      const u32x4 va = funnel(A0[k], A1[k], (meta[k] >> 15) & 15);
      const u32x4 vb = funnel(B0[k], B1[k], (meta[k] >> 20) & 15);
      u32x4 v;
      v.x = merge_dword(va.x, vb.x, split, 0);
      v.y = merge_dword(va.y, vb.y, split, 1);
      v.z = merge_dword(va.z, vb.z, split, 2);
      v.w = merge_dword(va.w, vb.w, split, 3);
      if (lo < hi) {
        const uint32_t gi = blk + tid + k * kThreads;
        store_granule<NT>(g0 + ((uint64_t)gi << 4), v, lo, hi);
      }
    }
  }
}

// 16 bytes to any address.
template <int NT>
__device__ __forceinline__ void st16_any(uint64_t addr, u32x4 v) {
  if (NT) __builtin_nontemporal_store(v, reinterpret_cast<u32x4_any FT_GLOBAL *>(addr));
  else *reinterpret_cast<u32x4_any FT_GLOBAL *>(addr) = v;
}

// Part of one row (fewer than 4096 bytes), a lane's share of it: a window of 16 bytes at any address,
// the last one moved back so that it ends with the part (it overlaps the one before with the same
// bytes), or one byte if the part is shorter than a window. Loaded in one call, stored in another, so
// that the caller can put other work between the two.
struct RowPart {
  uint64_t d = 0, s = 0;  // first byte of the part on either side; d == 0: no such part
  uint32_t len = 0;
  u32x4 v;
  uint8_t b;
};

template <int NT>
__device__ __forceinline__ void row_part_load(RowPart &P, uint32_t tid) {
  if (P.d == 0) return;
  if (P.len < 16) {
    if (tid < P.len) P.b = ld8(P.s + tid);
  } else if ((tid << 4) < P.len) {
    const uint32_t col = (tid << 4) + 16 <= P.len ? tid << 4 : P.len - 16;
    P.v = ld16_any<NT>(P.s + col);
  }
}

template <int NT>
__device__ __forceinline__ void row_part_store(const RowPart &P, uint32_t tid) {
  if (P.d == 0) return;
  if (P.len < 16) {
    if (tid < P.len) st8(P.d + tid, P.b);
  } else if ((tid << 4) < P.len) {
    const uint32_t col = (tid << 4) + 16 <= P.len ? tid << 4 : P.len - 16;
    st16_any<NT>(P.d + col, P.v);
  }
}

// Whole rows r0 .. rl of a pitched descriptor, R windows per lane and pass (see copy_rows_windows).
template <int NT, uint32_t R>
__device__ __forceinline__ void move_windows(const Xfer &X, uint64_t r0, uint64_t rl, uint32_t tid) {
  const uint32_t rb = (uint32_t)X.row_bytes;
  const uint32_t S = (rb + 15) >> 4;
  const uint32_t magic = (uint32_t)((1ull << 32) / S) + 1;  // q / S = mulhi(q, magic) or one less
  const uint32_t Q = (uint32_t)(rl - r0 + 1) * S;
  const uint64_t sb = X.src + r0 * X.src_pitch, db = X.dst + r0 * X.dst_pitch;
  for (uint32_t blk = 0; blk < Q; blk += R * kThreads) {
    u32x4 v[R];
    uint64_t to[R];
#pragma unroll
    for (uint32_t k = 0; k < R; ++k) {
      uint32_t q = blk + tid + k * kThreads;
      const bool active = q < Q;
      q = active ? q : Q - 1;
      uint32_t i = S == 1 ? q : __umulhi(q, magic);  // (2^32 / 1 + 1 does not fit the magic)
      i -= (i * S > q) ? 1u : 0u;
      const uint32_t j = q - i * S;
      const uint32_t col = j + 1 < S ? j << 4 : rb - 16;
      v[k] = ld16_any<NT>(sb + (uint64_t)i * X.src_pitch + col);
      to[k] = active ? db + (uint64_t)i * X.dst_pitch + col : 0;
    }
#pragma unroll
    for (uint32_t k = 0; k < R; ++k)
      if (to[k] != 0) st16_any<NT>(to[k], v[k]);
  }
}

// Rows of 16 .. 4096 bytes between any two pitches (a gather into a packed buffer, a scatter out of
// one, or pitched on both sides), window by window: a row of rb bytes is ceil(rb / 16) windows of 16 bytes, the last one moved back to end
// with the row, and a lane moves a window with one load and one store at whatever addresses they
// have (the memory pipeline splits an access that straddles aligned granules). Nothing is merged or
// masked and a lane's arithmetic is one division by a constant: for rows of 64-256 bytes a tenth of
// the vector instructions of a gather that owns aligned destination granules, and one load per
// window instead of two. R windows per lane and pass, all loads before the first store. The rows
// that the piece holds only a part of (its first and its last, where a tile boundary cuts a row) are
// loaded before the whole rows and stored after them, so that they cost no memory round trip of
// their own. Windows aligned to the destination's granules (51 against 46.5 us on the crops of the
// traffic workload) or to the source's (46.6) measured no better than windows counted from the
// row's first byte.
template <int NT, uint32_t R>
__device__ __forceinline__ void copy_rows_windows(const Xfer &X, uint64_t p, uint64_t take, uint32_t tid) {
  const uint32_t rb = (uint32_t)X.row_bytes;
  const uint64_t pend = p + take;
  uint64_t r0 = p / rb;
  const uint32_t c0 = (uint32_t)(p - r0 * rb);
  uint64_t rl = (pend - 1) / rb;
  const uint32_t cl = (uint32_t)(pend - rl * rb);  // one past the last column in the last row
  RowPart first, last;
  if (r0 == rl) {
    first.d = X.dst + r0 * X.dst_pitch + c0;
    first.s = X.src + r0 * X.src_pitch + c0;
    first.len = cl - c0;
    row_part_load<NT>(first, tid);
    row_part_store<NT>(first, tid);
    return;
  }
  if (c0 != 0) {
    first.d = X.dst + r0 * X.dst_pitch + c0;
    first.s = X.src + r0 * X.src_pitch + c0;
    first.len = rb - c0;
    r0 += 1;
  }
  if (cl != rb) {
    last.d = X.dst + rl * X.dst_pitch;
    last.s = X.src + rl * X.src_pitch;
    last.len = cl;
    rl -= 1;
  }
  row_part_load<NT>(first, tid);
  row_part_load<NT>(last, tid);
  if (r0 <= rl) {
    // whole rows r0 .. rl; a lane without a window repeats the last one's load (no load is predicated),
    // so a short piece takes a pass with fewer loads per lane
    const uint64_t windows = (rl - r0 + 1) * ((rb + 15) >> 4);
    if (windows <= 2 * kThreads) move_windows<NT, 2>(X, r0, rl, tid);
    else if (windows <= 4 * kThreads) move_windows<NT, 4>(X, r0, rl, tid);
    else move_windows<NT, R>(X, r0, rl, tid);
  }
  row_part_store<NT>(first, tid);
  row_part_store<NT>(last, tid);
}

// Payload bytes [p, p+take) of a pitched descriptor.
template <int NT, uint32_t U, bool P2P>
__device__ __forceinline__ void copy_rows(const Xfer &X, uint64_t p, uint64_t take, uint32_t tid) {
  const uint64_t rb = X.row_bytes;
  const uint64_t pend = p + take;
  const uint64_t r0 = p / rb;
  const uint64_t c0 = p - r0 * rb;
  const uint64_t rl = (pend - 1) / rb;
  const uint64_t cl = pend - rl * rb;  // one past the last column in the last row
  if (P2P && rb >= 16 && rb <= 4096 && take < (1ull << 30)) {
    // pool->pool. Ordinary rather than nontemporal accesses: neighbouring windows share memory lines,
    // and such rows come out of frames that several consumers crop (47.2 -> 45.5 us on the crops
    // of the traffic workload)
    copy_rows_windows<false, 8>(X, p, take, tid);
    return;
  }
  if (X.dst_pitch == rb && rb >= 16 && rb <= 4096 && take < (1ull << 30)) {
    copy_rows_packed_pairs<NT, 2>(X, p, take, tid);
    return;
  }
  // a row of rb bytes at any alignment spans at most (rb + 30) / 16 granules
  constexpr uint32_t RS = 4, RL = 2;  // rows per group and pass
  if (rb <= 16 * 16 - 30) {
    copy_rows_grouped<NT, 16, RS>(X, r0, c0, rl, cl, tid);
  } else if (rb <= 32 * 16 - 30) {
    copy_rows_grouped<NT, 32, RS>(X, r0, c0, rl, cl, tid);
  } else if (rb <= 128 * 16 - 30) {
    copy_rows_grouped<NT, 128, RL>(X, r0, c0, rl, cl, tid);
  } else {
    for (uint64_t r = r0; r <= rl; ++r) {
      const uint64_t ca = r == r0 ? c0 : 0, cb = r == rl ? cl : rb;
      copy_piece<NT, U>(X.dst + r * X.dst_pitch + ca, X.src + r * X.src_pitch + ca, cb - ca, tid);
    }
  }
}


// What a ticket names, decoded: bytes [b0, b1) of one function's stream (empty if
// b0 >= b1) and the descriptor holding b0.
struct Work {
  uint64_t b0, b1;
  uint32_t fl;     // the function (index into the class's table) and
  uint64_t k;      // the chunk of its stream that the tile belongs to: only the log wants them
  uint32_t x;      // index of the descriptor that holds stream byte b0
  uint64_t stage;  // address of stream byte 0 of this function if its chunk's ring slot went on for ever
  Xfer first;      // that descriptor (already pointing into the ring if it is staged)
};

// A staged descriptor's bytes of the current chunk lie in the chunk's ring slot, packed
// in stream order: stream byte b at `stage + b`.
__device__ __forceinline__ void into_ring(Xfer &X, uint64_t stage) {
  if (X.staged & kStagedSrc) {
    X.src = stage + X.stream_off;
    X.src_pitch = X.row_bytes;
  }
  if (X.staged & kStagedDst) {
    X.dst = stage + X.stream_off;
    X.dst_pitch = X.row_bytes;
  }
}

// A value that is the same in every lane of the wavefront, moved to scalar registers: what
// is computed from it stays on the scalar unit and table reads indexed by it are scalar
// loads.
__device__ __forceinline__ uint32_t uniform32(uint32_t v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ uint64_t uniform64(uint64_t v) {
  uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
  uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return (uint64_t)hi << 32 | lo;
}

// Where a workgroup is in the phase table. The ranks it decodes only grow (its tickets
// come from one counter that only grows), so the phase is found by stepping forward,
// and for nearly every ticket without a single table read.
struct PhaseCursor {
  uint32_t idx;
  uint32_t slot_off, nslots;
  uint64_t rank_base, round_base;
  uint64_t next_base;  // rank_base of the following phase; all ones after the last
};

__device__ __forceinline__ void cursor_set(PhaseCursor &pc, CPhaseP phases, uint32_t nphases, uint32_t idx) {
  pc.idx = idx;
  pc.rank_base = phases[idx].rank_base;
  pc.round_base = phases[idx].round_base;
  pc.slot_off = phases[idx].slot_off;
  pc.nslots = phases[idx].nslots;
  pc.next_base = idx + 1 < nphases ? phases[idx + 1].rank_base : ~0ull;
}

// Where a workgroup is in the list of empty-tile runs (its tickets only grow).
struct SkipCursor {
  uint32_t idx;
  uint64_t acc;      // empty tiles before the current ticket
  uint64_t next_at;  // ticket at which the next run applies; all ones after the last
};

// Dependent table reads on the way from a ticket to its bytes: the slot; then the
// function and the chunk's first and last descriptor index side by side; then the
// descriptor itself (plus a short search when a chunk spans several descriptors).
//
// Only the first wavefront decodes, so to the compiler everything that lives across
// iterations here (the cursors) differs between lanes and would sit in vector registers,
// its table reads vector loads - which wait behind every store of the tile. The cursors
// are therefore brought to scalar registers on entry and written back on exit.
__device__ __forceinline__ Work decode_ticket(const ClassTable &T, const ConstTables &CT, PhaseCursor &pc_v,
                                              SkipCursor &sc_v, uint64_t t) {
  Work w;
  w.b0 = w.b1 = 0;
  w.fl = 0;
  w.k = 0;
  w.x = 0;
  w.stage = 0;
  w.first = Xfer{};  // an empty ticket is handed on like any other: nothing of it is left unset
  if (t >= T.ntickets) return w;
  if (T.single) {
    // the only run of empty tiles lies behind the last ticket
    uint64_t rank, ti;
    if (t < (1ull << 32)) {
      rank = (uint32_t)t / T.tiles_per_chunk;
      ti = (uint32_t)t - (uint32_t)rank * T.tiles_per_chunk;
    } else {
      rank = t / T.tiles_per_chunk;
      ti = t - rank * T.tiles_per_chunk;
    }
    w.first = read_xfer(CT.xfers, 0);
    const uint64_t stream_bytes = w.first.row_bytes * w.first.rows;
    const uint64_t c0 = rank * T.chunk_bytes;
    uint64_t lo = ti * T.tile_bytes, hi = lo + T.tile_bytes;
    if (hi > T.chunk_bytes) hi = T.chunk_bytes;
    uint64_t b0 = c0 + lo, b1 = c0 + hi;
    if (b1 > stream_bytes) b1 = stream_bytes;
    if (b0 >= b1) return w;
    w.b0 = b0;
    w.b1 = b1;
    w.k = rank;
    return w;
  }
  SkipCursor sc;
  sc.idx = uniform32(sc_v.idx);
  sc.acc = uniform64(sc_v.acc);
  sc.next_at = uniform64(sc_v.next_at);
  while (t >= sc.next_at) {
    sc.acc += CT.skips[sc.idx].gap;
    sc.idx += 1;
    sc.next_at = sc.idx < T.nskips ? CT.skips[sc.idx].at : ~0ull;
  }
  sc_v = sc;
  const uint64_t v = t + sc.acc;  // tile of the uniform grid
  uint64_t rank, ti;
  if (v < (1ull << 32)) {
    rank = (uint32_t)v / T.tiles_per_chunk;
    ti = (uint32_t)v - (uint32_t)rank * T.tiles_per_chunk;
  } else {
    rank = v / T.tiles_per_chunk;
    ti = v - rank * T.tiles_per_chunk;
  }
  PhaseCursor pc;
  pc.idx = uniform32(pc_v.idx);
  pc.slot_off = uniform32(pc_v.slot_off);
  pc.nslots = uniform32(pc_v.nslots);
  pc.rank_base = uniform64(pc_v.rank_base);
  pc.round_base = uniform64(pc_v.round_base);
  pc.next_base = uniform64(pc_v.next_base);
  while (rank >= pc.next_base) cursor_set(pc, CT.phases, T.nphases, pc.idx + 1);
  pc_v = pc;
  const uint64_t rel = rank - pc.rank_base;
  uint64_t round;
  uint32_t s;
  if (rel < (1ull << 32)) {
    round = (uint32_t)rel / pc.nslots;
    s = pc.slot_off + ((uint32_t)rel - (uint32_t)round * pc.nslots);
  } else {
    round = rel / pc.nslots;
    s = pc.slot_off + (uint32_t)(rel - round * pc.nslots);
  }
  const uint32_t fl = CT.slots[s].fl;
  const uint64_t k = (pc.round_base + round) * (uint64_t)CT.slots[s].weight + CT.slots[s].i;
  const uint64_t stream_bytes = CT.funcs[fl].stream_bytes;
  uint32_t x0, x1;
  if (CT.chunk_desc != nullptr) {
    const FT_CONST uint32_t *cd = CT.chunk_desc;
    const uint64_t per = T.desc_per;
    const uint64_t e = ((uint64_t)CT.slots[s].chunk_off - fl + k) * per + fl + (per > 1 ? ti : 0);
    x0 = cd[e];
    x1 = per > 1 ? x0 : cd[e + 1];  // an entry per tile names the tile's descriptor itself
  } else {
    x0 = CT.funcs[fl].desc_off;
    x1 = x0 + CT.funcs[fl].ndesc - 1;
  }
  const uint64_t c0 = (CT.funcs[fl].chunk_base + k) * T.chunk_bytes;
  uint64_t lo = ti * T.tile_bytes, hi = lo + T.tile_bytes;
  if (hi > T.chunk_bytes) hi = T.chunk_bytes;
  uint64_t b0 = c0 + lo, b1 = c0 + hi;
  if (b1 > stream_bytes) b1 = stream_bytes;
  if (b0 >= b1) return w;
  w.b0 = b0;
  w.b1 = b1;
  w.fl = fl;
  w.k = CT.funcs[fl].chunk_base + k;
  w.x = x0 == x1 ? x0 : find_xfer(CT.xfers, x0, x1, b0);
  w.first = read_xfer(CT.xfers, w.x);
  w.stage = T.stage_base + (T.stage_slot0 + (rank - T.stage_rank0)) * T.chunk_bytes - c0;
  into_ring(w.first, w.stage);
  return w;
}

// FT_LOG: what the decode made of ticket t goes into the ticket's log entry as it is, so that the
// order the copy kernel really follows can be held against the proportional order of Sec. 6.1.
__device__ __forceinline__ void log_decoded(const ClassTable &T, uint64_t t, const Work &w) {
  if (T.log == nullptr || t >= T.ntickets) return;
  T.log[t].fl = w.fl;
  T.log[t].k = w.k;
  T.log[t].b0 = w.b0;
  T.log[t].b1 = w.b1;
}

// A decoded ticket on its way from the first wavefront to the others, in LDS.
struct WorkSlot {
  // what the common case needs, in the first 32 bytes: one full aligned block
  uint64_t t;     // the ticket; >= ntickets: none left
  uint64_t fd;    // destination and
  uint64_t fs;    // source of the block, or 0 / 0 if the ticket is not of that kind
  uint64_t _pad;
  // everything else
  uint64_t b0, b1;
  uint64_t x;
  uint64_t stage;
  Xfer first;
};

// block_bytes: the size of a full block of this class's copy routines
__device__ __forceinline__ void put_work(WorkSlot &slot, uint64_t t, const Work &w, uint64_t block_bytes) {
  const uint64_t p0 = w.b0 - w.first.stream_off;
  const uint64_t len = w.b1 - w.b0;
  const uint64_t fd = w.first.dst + p0, fs = w.first.src + p0;
  const bool fast = w.first.rows == 1 && len == block_bytes && ((fd | fs) & 15) == 0 && p0 + len <= w.first.row_bytes;
  slot.t = t;
  slot.fd = fast ? fd : 0;
  slot.fs = fast ? fs : 0;
  slot.b0 = w.b0;
  slot.b1 = w.b1;
  slot.x = w.x;
  slot.stage = w.stage;
  slot.first = w.first;
}

__device__ __forceinline__ void get_work(const WorkSlot &slot, Work &w) {
  w.b0 = uniform64(slot.b0);
  w.b1 = uniform64(slot.b1);
  w.x = (uint32_t)uniform64(slot.x);
  w.stage = uniform64(slot.stage);
  w.first.src = uniform64(slot.first.src);
  w.first.dst = uniform64(slot.first.dst);
  w.first.row_bytes = uniform64(slot.first.row_bytes);
  w.first.rows = uniform64(slot.first.rows);
  w.first.src_pitch = uniform64(slot.first.src_pitch);
  w.first.dst_pitch = uniform64(slot.first.dst_pitch);
  w.first.stream_off = uniform64(slot.first.stream_off);
  w.first.staged = 0;  // already applied
}

// The tiles of one contiguous transfer whose two sides are 16-byte aligned, dealt out round robin among
// the workgroups.
template <int NT, uint32_t U>
__device__ __forceinline__ void deal_out_tiles(const ClassTable &T, uint64_t src, uint64_t dst, uint64_t nbytes, uint32_t tid) {
  for (uint64_t v = blockIdx.x; v < T.ntickets; v += gridDim.x) {
    uint64_t rank, ti;
    if (v < (1ull << 32)) {
      rank = (uint32_t)v / T.tiles_per_chunk;
      ti = (uint32_t)v - (uint32_t)rank * T.tiles_per_chunk;
    } else {
      rank = v / T.tiles_per_chunk;
      ti = v - rank * T.tiles_per_chunk;
    }
    uint64_t lo = ti * T.tile_bytes, hi = lo + T.tile_bytes;
    if (hi > T.chunk_bytes) hi = T.chunk_bytes;
    const uint64_t b0 = rank * T.chunk_bytes + lo;
    uint64_t b1 = rank * T.chunk_bytes + hi;
    if (b1 > nbytes) b1 = nbytes;
    if (b0 < b1) {
      if (b1 - b0 == (uint64_t)kThreads * U * 16) copy_rows_of_vectors<NT, U>(dst + b0, src + b0, tid);
      else if (((b1 - b0) & 15) == 0) copy_vectors<NT, U>(dst + b0, src + b0, (b1 - b0) >> 4, tid);
      else copy_piece<NT, U>(dst + b0, src + b0, b1 - b0, tid);  // the tensor's last tile, a length that is no multiple of 16
    }
    __syncthreads();  // keeps a workgroup's loads and stores in separate bursts, as in the ticket loop
  }
}

// Which compute unit this wavefront runs on, from the hardware's identification registers: the
// accelerator die (HW_REG_XCC_ID, 4 bits) above shader engine, shader array and unit (bits 15:8 of
// HW_REG_HW_ID). Equal values mean the same compute unit; used by the log only.
__device__ __forceinline__ uint32_t compute_unit_id() {
  const uint32_t hw = __builtin_amdgcn_s_getreg((8 - 1) << 11 | 8 << 6 | 4);    // HW_ID[15:8]: se_id, sh_id, cu_id
  const uint32_t die = __builtin_amdgcn_s_getreg((4 - 1) << 11 | 0 << 6 | 20);  // XCC_ID[3:0]
  return die << 8 | hw;
}

// A barrier for LDS traffic alone: what this wavefront wrote to LDS is there and every wavefront
// has arrived; outstanding vector memory operations (the tile's stores) are not waited for.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// A barrier behind which every vector memory operation of the workgroup issued before it has
// completed (its stores are acknowledged). The wavefronts of a workgroup touch disjoint payload
// bytes, so nothing more is asked of it than that.
__device__ __forceinline__ void drain_barrier() {
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Persistent workgroups. Workgroup b starts on ticket b and every later ticket comes from
// the counter (which therefore hands out the tickets from the grid size on; the host never
// launches more workgroups than there are tickets). When all workgroups of a launch ask
// the counter at once it answers them one after the other, about 14 ns each: the last of
// 256 would wait 4 us for its first tile, against 2 us for the decode alone. A workgroup
// that the GPU starts late (its CU was busy with other work) holds its first tile back
// until then, but the launch could not have ended before that workgroup has run anyway.
// A workgroup holds one ticket beyond the one it is moving: the atomic for ticket i+1 is
// issued among tile i's stores (behind the last of them for a tile that moves in several
// pieces or through the byte-shifting routines) and read after them.
// A workgroup moves its tile in two phases - every load of the tile, then every store.
// While the stores drain, the first wavefront alone decodes ticket i+1 (scalar table
// reads) and leaves the result in LDS; the barrier at the end of the iteration waits
// for the stores and publishes it. Keeping a CU's reads and writes in separate bursts,
// one workgroup per CU, is what the memory controllers serve fastest.
//
// CLS (the link class, or kLightPoolToPool) selects the block size of the copy routines and gives each
// class's kernel a name of its own, so that profiles keep host-link launches and
// pool->pool launches apart.
template <bool NT, int CLS>
__global__ __launch_bounds__(kThreads, (CLS == 2 ? 1 : 2)) void ft_copy_kernel(ClassTable T, InlineBlob) {
  constexpr uint32_t U = UnrollOf<CLS>::value;
  constexpr int MODE = !NT ? 0 : CLS == 1 ? kToHost : kStream;
  __shared__ WorkSlot s_work[2];
  const uint32_t tid = threadIdx.x;
  const ConstTables CT = const_tables(T);
  if (T.single >= 2) {
    // One contiguous transfer, both sides multiples of 16, nothing to record:
    // passing a single tensor. With one function there is nothing to interleave - ticket t is
    // tile t of the one stream - so the tiles are dealt out round robin, workgroup b taking
    // tiles b, b + workgroups, ...: no counter, no decode by one wavefront for the others, no
    // hand-over through LDS, and the first tile's loads are issued a microsecond after entry.
    if (T.single == 3) deal_out_tiles<false, U>(T, CT.xfers[0].src, CT.xfers[0].dst, CT.xfers[0].row_bytes, tid);
    else deal_out_tiles<MODE, U>(T, CT.xfers[0].src, CT.xfers[0].dst, CT.xfers[0].row_bytes, tid);
    return;
  }
  const bool lead = tid < 64;  // the first wavefront: draws and decodes tickets
  if (T.log && tid == 0) {
    T.wg_log[blockIdx.x].t_entry = wall_clock64();
    T.wg_log[blockIdx.x].unit = compute_unit_id();
  }
  PhaseCursor pc;
  SkipCursor sc;
  if (lead) {
    pc.idx = T.phase0;
    pc.rank_base = T.first_phase.rank_base;
    pc.round_base = T.first_phase.round_base;
    pc.slot_off = T.first_phase.slot_off;
    pc.nslots = T.first_phase.nslots;
    pc.next_base = T.first_next_base;
    sc.idx = T.skip0;
    sc.acc = T.skip_acc0;
    sc.next_at = T.first_skip_at;
    // workgroup b starts on ticket b; the counter hands out the tickets from gridDim.x on
    const uint64_t t_first = T.ticket_base + blockIdx.x;
    const Work w = decode_ticket(T, CT, pc, sc, t_first);
    if (tid == 0) {
      put_work(s_work[0], t_first, w, (uint64_t)kThreads * U * 16);
      log_decoded(T, t_first, w);
    }
  }
  __syncthreads();
  uint32_t slot = 0;
  uint64_t t_cur = uniform64(s_work[0].t), fd = uniform64(s_work[0].fd), fs = uniform64(s_work[0].fs);
  while (t_cur < T.ntickets) {
    uint64_t t_begin = 0;
    if (T.log) t_begin = wall_clock64();
    unsigned long long claimed = 0;
    if (fd != 0) {
      // the common case, one full aligned block (64 KiB for pool->pool): 32 bytes read
      // from LDS, then straight-line code to the last store, the ticket draw on the way
      claimed = copy_rows_of_vectors_draw<MODE, U>(fd, fs, tid, T.ticket);
    } else {
      // Host-link classes draw before the tile's pieces: a tile lasts as long as the link takes, the
      // counter's answer is there long before, and the workgroups run ahead of the link anyway.
      if (CLS < 2 && tid == 0) claimed = atomicAdd(T.ticket, 1ull);
      Work cur;
      get_work(s_work[slot], cur);
      uint64_t pos = cur.b0;
      uint32_t x = cur.x;
      Xfer X = cur.first;
      while (pos < cur.b1) {
        const uint64_t p = pos - X.stream_off;
        uint64_t take = X.row_bytes * X.rows - p;
        if (take > cur.b1 - pos) take = cur.b1 - pos;
        // the next piece's descriptor is on its way (scalar load) while this piece moves
        const bool more = pos + take < cur.b1;
        Xfer Xn = X;
        if (more) Xn = read_xfer(CT.xfers, ++x);
        if (X.rows == 1) copy_piece<MODE, U>(X.dst + p, X.src + p, take, tid);
        else copy_rows<MODE, U, (CLS >= 2)>(X, p, take, tid);
        pos += take;
        if (more) {
          X = Xn;
          into_ring(X, cur.stage);
        }
      }
      // pool->pool: the draw follows the last piece's stores. In front of the tile's loads it would hold
      // every store back until the counter has answered, and the ticket would be held for the whole of a
      // tile that takes long (several pieces, rows): large_mixed 83.4 -> 80.8 us per launch, crops 38.6 -> 34.7
      if (CLS >= 2 && tid == 0) claimed = atomicAdd(T.ticket, 1ull);
    }
    if (lead) {
      // lane 0 holds the counter's answer; all 64 lanes of this wavefront are enabled
      const uint64_t t_drawn = T.ticket_base + gridDim.x + uniform64(claimed);
      const Work next = decode_ticket(T, CT, pc, sc, t_drawn);
      if (tid == 0) {
        put_work(s_work[slot ^ 1], t_drawn, next, (uint64_t)kThreads * U * 16);
        log_decoded(T, t_drawn, next);
      }
    }

    if (T.log) {
      // the tile counts as done when every store of the workgroup has been acknowledged
      __builtin_amdgcn_s_waitcnt(0);
      __syncthreads();
      if (tid == 0) {
        T.log[t_cur].t_begin = t_begin;
        T.log[t_cur].t_end = wall_clock64();
        T.log[t_cur].wg = blockIdx.x;
      }
    }
    // Two barriers end the tile. The first concerns LDS only (the decoded ticket is there; nobody
    // waits for stores): behind it every wavefront fetches the next tile's ticket and addresses
    // while its own stores still drain. The second waits for the stores of the whole workgroup,
    // and the first load of the next tile follows it directly (0.1 us per tile less between the
    // last acknowledged store and the first load than with the reads behind a single barrier).
    lds_barrier();
    const uint64_t t_next = uniform64(s_work[slot ^ 1].t);
    const uint64_t fd_next = uniform64(s_work[slot ^ 1].fd), fs_next = uniform64(s_work[slot ^ 1].fs);
    drain_barrier();
    slot ^= 1;
    t_cur = t_next;
    fd = fd_next;
    fs = fs_next;
  }
  if (T.log && tid == 0) T.wg_log[blockIdx.x].t_exit = wall_clock64();
  if (T.self_reset && tid == 0) {
    // this workgroup's draws have all been answered (the last answer ended its loop)
    if (atomicAdd(T.ticket + 1, 1ull) == gridDim.x - 1) {
      __hip_atomic_store(T.ticket, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(T.ticket + 1, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

__global__ void ft_decode_kernel(ClassTable T, InlineBlob, uint32_t *func_out, uint32_t *chunk_out, uint64_t cap) {
  uint64_t rank = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (rank >= T.nchunks || rank >= cap) return;
  const ConstTables CT = const_tables(T);
  const ChunkId id = decode_rank(CT.phases, T.nphases, CT.slots, rank);
  func_out[rank] = CT.funcs[id.fl].func;
  chunk_out[rank] = (uint32_t)(CT.funcs[id.fl].chunk_base + id.k);
}

__global__ __launch_bounds__(kThreads) void ft_plain_copy_kernel(u32x4 *dst, const u32x4 *src, uint64_t nvec) {
  constexpr uint32_t kUnroll = 4;
  const uint64_t stride = (uint64_t)gridDim.x * kThreads;
  uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
  for (; i + (kUnroll - 1) * stride < nvec; i += kUnroll * stride) {
    u32x4 v[kUnroll];
#pragma unroll
    for (uint32_t j = 0; j < kUnroll; ++j) v[j] = __builtin_nontemporal_load(src + i + j * stride);
#pragma unroll
    for (uint32_t j = 0; j < kUnroll; ++j) __builtin_nontemporal_store(v[j], dst + i + j * stride);
  }
  for (; i < nvec; i += stride) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// Reads `nvec` vectors and keeps nothing (the store below practically never happens: it only
// keeps the loads alive), and writes `nvec` vectors of a fixed value: what the memory system
// gives to reads alone and to writes alone, the two numbers that bound any copy.
__global__ __launch_bounds__(kThreads) void ft_plain_read_kernel(const u32x4 *src, uint64_t nvec, u32x4 *sink) {
  constexpr uint32_t kUnroll = 8;
  const uint64_t stride = (uint64_t)gridDim.x * kThreads;
  u32x4 acc = {0, 0, 0, 0};
  uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
  for (; i + (kUnroll - 1) * stride < nvec; i += kUnroll * stride) {
    u32x4 v[kUnroll];
#pragma unroll
    for (uint32_t j = 0; j < kUnroll; ++j) v[j] = __builtin_nontemporal_load(src + i + j * stride);
#pragma unroll
    for (uint32_t j = 0; j < kUnroll; ++j) acc ^= v[j];
  }
  for (; i < nvec; i += stride) acc ^= __builtin_nontemporal_load(src + i);
  if (sink != nullptr && (acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u && acc.x == 0x7f4a7c15u) sink[0] = acc;
}

__global__ __launch_bounds__(kThreads) void ft_plain_fill_kernel(u32x4 *dst, uint64_t nvec, uint32_t word) {
  const uint64_t stride = (uint64_t)gridDim.x * kThreads;
  const u32x4 v = {word, word, word, word};
  for (uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x; i < nvec; i += stride)
    __builtin_nontemporal_store(v, dst + i);
}

// What a launch passes as tables when the job's own are in device memory.
static const InlineBlob kNoTables{};

hipError_t launch_copy(const ClassTable &T, int link_class, uint32_t workgroups, hipStream_t stream,
                       hipEvent_t ev_start, hipEvent_t ev_stop, const InlineBlob *tables) {
  if (workgroups == 0 || (T.inline_tables != 0) != (tables != nullptr)) return hipErrorInvalidValue;
  const dim3 grid(workgroups), block(kThreads);
  const InlineBlob &B = tables ? *tables : kNoTables;
  // with events, they are bound to this dispatch: they read the kernel's own start and end
  switch (link_class) {
    case 0: hipExtLaunchKernelGGL((ft_copy_kernel<true, 0>), grid, block, 0, stream, ev_start, ev_stop, 0, T, B); break;
    case 1: hipExtLaunchKernelGGL((ft_copy_kernel<true, 1>), grid, block, 0, stream, ev_start, ev_stop, 0, T, B); break;
    case 2: hipExtLaunchKernelGGL((ft_copy_kernel<true, 2>), grid, block, 0, stream, ev_start, ev_stop, 0, T, B); break;
    case kLightPoolToPool:
      hipExtLaunchKernelGGL((ft_copy_kernel<true, kLightPoolToPool>), grid, block, 0, stream, ev_start, ev_stop, 0, T, B);
      break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_decode(const ClassTable &T, uint32_t *func_out, uint32_t *chunk_out, uint64_t cap,
                         hipStream_t stream, const InlineBlob *tables) {
  if ((T.inline_tables != 0) != (tables != nullptr)) return hipErrorInvalidValue;
  uint64_t n = T.nchunks < cap ? T.nchunks : cap;
  if (n == 0) return hipSuccess;
  uint32_t blocks = (uint32_t)((n + 255) / 256);
  hipLaunchKernelGGL(ft_decode_kernel, dim3(blocks), dim3(256), 0, stream, T, tables ? *tables : kNoTables, func_out,
                     chunk_out, cap);
  return hipGetLastError();
}

hipError_t launch_plain_copy(void *dst, const void *src, uint64_t bytes, uint32_t workgroups, hipStream_t stream) {
  if (bytes == 0) return hipSuccess;
  if (workgroups == 0) workgroups = 2048;
  hipLaunchKernelGGL(ft_plain_copy_kernel, dim3(workgroups), dim3(kThreads), 0, stream,
                     static_cast<u32x4 *>(dst), static_cast<const u32x4 *>(src), bytes >> 4);
  return hipGetLastError();
}

hipError_t launch_plain_read(const void *src, uint64_t bytes, uint32_t workgroups, hipStream_t stream) {
  if (bytes == 0) return hipSuccess;
  if (workgroups == 0) workgroups = 256;
  hipLaunchKernelGGL(ft_plain_read_kernel, dim3(workgroups), dim3(kThreads), 0, stream,
                     static_cast<const u32x4 *>(src), bytes >> 4, static_cast<u32x4 *>(nullptr));
  return hipGetLastError();
}

hipError_t launch_plain_fill(void *dst, uint64_t bytes, uint32_t word, uint32_t workgroups, hipStream_t stream) {
  if (bytes == 0) return hipSuccess;
  if (workgroups == 0) workgroups = 256;
  hipLaunchKernelGGL(ft_plain_fill_kernel, dim3(workgroups), dim3(kThreads), 0, stream, static_cast<u32x4 *>(dst),
                     bytes >> 4, word);
  return hipGetLastError();
}

}  // namespace ft
