// HIP kernels of the transfer engine for gfx950 (CDNA4, 64-wide wavefronts).
//
// ft_copy_kernel is the whole device side of Sec. 5.1 / 6.1 for one link class:
// persistent workgroups draw tickets from one device counter; a ticket names a tile
// of a chunk, chunks are numbered in the proportional order of Sec. 6.1, so the
// counter hands the link's bandwidth out to functions by weight at tile granularity.
// Bytes move as 16-byte vectors, one per lane, consecutive lanes on consecutive
// vectors, so every wavefront load/store covers 1 KiB of contiguous memory.
#include <hip/hip_runtime.h>

#include "ft_kernels.h"

namespace ft {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr uint32_t kThreads = 256;  // 4 wavefronts per workgroup
constexpr uint32_t kUnroll = 4;     // independent 16-byte loads per lane before the first store

template <bool NT>
__device__ __forceinline__ u32x4 ld16(uint64_t addr) {
  if (NT) return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(addr));
  return *reinterpret_cast<const u32x4 *>(addr);
}
template <bool NT>
__device__ __forceinline__ void st16(uint64_t addr, u32x4 v) {
  if (NT) __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(addr));
  else *reinterpret_cast<u32x4 *>(addr) = v;
}

// 16 bytes starting `shift` (1..15) bytes into the 32-byte pair (A, B).
__device__ __forceinline__ u32x4 funnel(u32x4 A, u32x4 B, uint32_t shift) {
  const uint32_t q = shift >> 2, r8 = (shift & 3) * 8;
  uint32_t x0 = q == 0 ? A.x : q == 1 ? A.y : q == 2 ? A.z : A.w;
  uint32_t x1 = q == 0 ? A.y : q == 1 ? A.z : q == 2 ? A.w : B.x;
  uint32_t x2 = q == 0 ? A.z : q == 1 ? A.w : q == 2 ? B.x : B.y;
  uint32_t x3 = q == 0 ? A.w : q == 1 ? B.x : q == 2 ? B.y : B.z;
  uint32_t x4 = q == 0 ? B.x : q == 1 ? B.y : q == 2 ? B.z : B.w;
  u32x4 v;
  v.x = (uint32_t)(((uint64_t)x1 << 32 | x0) >> r8);
  v.y = (uint32_t)(((uint64_t)x2 << 32 | x1) >> r8);
  v.z = (uint32_t)(((uint64_t)x3 << 32 | x2) >> r8);
  v.w = (uint32_t)(((uint64_t)x4 << 32 | x3) >> r8);
  return v;
}

// Copy n bytes from s0 to d0, any alignment, with lanes lane, lane+L, ... of a group of
// L lanes. Works in destination granules (aligned 16 bytes): full granules are written
// with one vector store, the first and last with byte stores of only the bytes that
// belong to the range. Source reads are aligned 16-byte loads of granules that hold at
// least one byte of the source range, so nothing outside the pages of the range is
// touched; when source and destination differ in alignment two loads are merged.
template <bool NT>
__device__ __forceinline__ void copy_span(uint64_t d0, uint64_t s0, uint64_t n, uint32_t lane, uint32_t L) {
  const uint64_t d1 = d0 + n, s1 = s0 + n;
  const uint64_t g0 = d0 & ~15ull;
  const uint64_t ngran = (((d1 + 15) & ~15ull) - g0) >> 4;
  const uint64_t delta = s0 - d0;
  const uint32_t shift = (uint32_t)(delta & 15);
  for (uint64_t g = lane; g < ngran; g += L) {
    const uint64_t ga = g0 + (g << 4);
    const uint64_t sa = ga + delta;
    u32x4 v;
    if (shift == 0) {
      v = ld16<NT>(sa);
    } else {
      const uint64_t a0 = sa & ~15ull, a1 = a0 + 16;
      u32x4 A = {0, 0, 0, 0}, B = {0, 0, 0, 0};
      if (a0 + 16 > s0 && a0 < s1) A = ld16<false>(a0);
      if (a1 + 16 > s0 && a1 < s1) B = ld16<false>(a1);
      v = funnel(A, B, shift);
    }
    const uint32_t lo = ga < d0 ? (uint32_t)(d0 - ga) : 0u;
    const uint32_t hi = ga + 16 > d1 ? (uint32_t)(d1 - ga) : 16u;
    if (lo == 0 && hi == 16) {
      st16<NT>(ga, v);
    } else {
      for (uint32_t b = lo; b < hi; ++b) {
        const uint32_t w = (b >> 2) == 0 ? v.x : (b >> 2) == 1 ? v.y : (b >> 2) == 2 ? v.z : v.w;
        *reinterpret_cast<uint8_t *>(ga + b) = (uint8_t)(w >> ((b & 3) * 8));
      }
    }
  }
}

// nvec aligned 16-byte vectors, all threads of the workgroup, kUnroll loads in flight per lane.
template <bool NT>
__device__ __forceinline__ void copy_vectors(uint64_t d, uint64_t s, uint64_t nvec, uint32_t tid) {
  uint64_t i = tid;
  for (; i + (kUnroll - 1) * kThreads < nvec; i += kUnroll * kThreads) {
    u32x4 v[kUnroll];
#pragma unroll
    for (uint32_t j = 0; j < kUnroll; ++j) v[j] = ld16<NT>(s + ((i + j * kThreads) << 4));
#pragma unroll
    for (uint32_t j = 0; j < kUnroll; ++j) st16<NT>(d + ((i + j * kThreads) << 4), v[j]);
  }
  for (; i < nvec; i += kThreads) st16<NT>(d + (i << 4), ld16<NT>(s + (i << 4)));
}

// One contiguous piece with the whole workgroup.
template <bool NT>
__device__ __forceinline__ void copy_piece(uint64_t d0, uint64_t s0, uint64_t n, uint32_t tid) {
  if (((d0 ^ s0) & 15) == 0 && n >= 256) {
    // same alignment on both sides: byte head up to the boundary, vector body, byte tail
    const uint64_t head = (16 - (d0 & 15)) & 15;
    const uint64_t nvec = (n - head) >> 4;
    const uint64_t tail = (n - head) & 15;
    if (tid < head) *reinterpret_cast<uint8_t *>(d0 + tid) = *reinterpret_cast<const uint8_t *>(s0 + tid);
    const uint64_t toff = head + (nvec << 4);
    if (tid < tail)
      *reinterpret_cast<uint8_t *>(d0 + toff + tid) = *reinterpret_cast<const uint8_t *>(s0 + toff + tid);
    copy_vectors<NT>(d0 + head, s0 + head, nvec, tid);
  } else {
    copy_span<NT>(d0, s0, n, tid, kThreads);
  }
}

// Payload bytes [p, p+take) of a pitched descriptor.
template <bool NT>
__device__ __forceinline__ void copy_rows(const Xfer &X, uint64_t p, uint64_t take, uint32_t tid) {
  const uint64_t rb = X.row_bytes;
  const uint64_t pend = p + take;
  const uint64_t r0 = p / rb;
  const uint64_t c0 = p - r0 * rb;
  const uint64_t rl = (pend - 1) / rb;
  const uint64_t cl = pend - rl * rb;  // one past the last column in the last row
  if (rb > 2048) {
    for (uint64_t r = r0; r <= rl; ++r) {
      const uint64_t ca = r == r0 ? c0 : 0, cb = r == rl ? cl : rb;
      copy_piece<NT>(X.dst + r * X.dst_pitch + ca, X.src + r * X.src_pitch + ca, cb - ca, tid);
    }
  } else {
    // short rows: a group of L lanes per row, several rows per pass
    const uint32_t L = rb <= 256 ? 16u : rb <= 512 ? 32u : rb <= 1024 ? 64u : 128u;
    const uint32_t groups = kThreads / L;
    const uint32_t g = tid / L, l = tid % L;
    for (uint64_t r = r0 + g; r <= rl; r += groups) {
      const uint64_t ca = r == r0 ? c0 : 0, cb = r == rl ? cl : rb;
      copy_span<NT>(X.dst + r * X.dst_pitch + ca, X.src + r * X.src_pitch + ca, cb - ca, l, L);
    }
  }
}

__device__ __forceinline__ uint64_t uniform64(uint64_t v) {
  uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
  uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return (uint64_t)hi << 32 | lo;
}

// The tile a ticket names: bytes [b0, b1) of function fl's stream (may be empty).
struct Tile {
  uint32_t fl;
  uint64_t k;
  uint64_t b0, b1;
};

__device__ __forceinline__ Tile tile_of(const ClassTable &T, uint64_t t) {
  uint64_t rank, ti;
  if (t < (1ull << 32)) {
    rank = (uint32_t)t / T.tiles_per_chunk;
    ti = (uint32_t)t - (uint32_t)rank * T.tiles_per_chunk;
  } else {
    rank = t / T.tiles_per_chunk;
    ti = t - rank * T.tiles_per_chunk;
  }
  const ChunkId id = decode_rank(T.phases, T.nphases, T.slots, T.funcs, rank);
  const uint64_t S = T.funcs[id.fl].stream_bytes;
  const uint64_t c0 = id.k * T.chunk_bytes;
  uint64_t lo = ti * T.tile_bytes, hi = lo + T.tile_bytes;
  if (hi > T.chunk_bytes) hi = T.chunk_bytes;
  Tile tl;
  tl.fl = id.fl;
  tl.k = id.k;
  tl.b0 = c0 + lo;
  tl.b1 = c0 + hi;
  if (tl.b1 > S) tl.b1 = S;
  if (tl.b0 > tl.b1) tl.b0 = tl.b1;
  return tl;
}

template <bool NT>
__global__ __launch_bounds__(kThreads) void ft_copy_kernel(ClassTable T) {
  __shared__ unsigned long long s_ticket[2];
  const uint32_t tid = threadIdx.x;
  if (tid == 0) s_ticket[0] = atomicAdd(T.ticket, 1ull);
  __syncthreads();
  uint64_t t = uniform64(s_ticket[0]);
  uint32_t buf = 0;
  while (t < T.ntickets) {
    // draw the next ticket now; its latency hides behind this tile's copy
    unsigned long long next = 0;
    if (tid == 0) next = atomicAdd(T.ticket, 1ull);
    uint64_t t_begin = 0;
    if (T.log) t_begin = wall_clock64();

    const Tile tl = tile_of(T, t);
    if (tl.b0 < tl.b1) {
      const Func fn = T.funcs[tl.fl];
      uint32_t x = find_xfer(T.xfers, fn, tl.b0);
      uint64_t pos = tl.b0;
      while (pos < tl.b1) {
        const Xfer X = T.xfers[x];
        const uint64_t p = pos - X.stream_off;
        const uint64_t size = X.row_bytes * X.rows;
        uint64_t take = size - p;
        if (take > tl.b1 - pos) take = tl.b1 - pos;
        if (X.rows == 1) copy_piece<NT>(X.dst + p, X.src + p, take, tid);
        else copy_rows<NT>(X, p, take, tid);
        pos += take;
        ++x;
      }
    }
    if (T.log) {
      // the tile counts as done when every store of the workgroup has been issued and
      // acknowledged
      __builtin_amdgcn_s_waitcnt(0);
      __syncthreads();
      if (tid == 0) {
        T.log[t].t_begin = t_begin;
        T.log[t].t_end = wall_clock64();
      }
    }
    if (tid == 0) s_ticket[buf ^ 1] = next;
    __syncthreads();
    buf ^= 1;
    t = uniform64(s_ticket[buf]);
  }
}

__global__ void ft_decode_kernel(ClassTable T, uint32_t *func_out, uint32_t *chunk_out, uint64_t cap) {
  uint64_t rank = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (rank >= T.nchunks || rank >= cap) return;
  const ChunkId id = decode_rank(T.phases, T.nphases, T.slots, T.funcs, rank);
  func_out[rank] = T.funcs[id.fl].func;
  chunk_out[rank] = (uint32_t)id.k;
}

__global__ __launch_bounds__(kThreads) void ft_plain_copy_kernel(u32x4 *dst, const u32x4 *src, uint64_t nvec) {
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

hipError_t launch_copy(const ClassTable &T, uint32_t workgroups, bool nontemporal, hipStream_t stream) {
  if (workgroups == 0) return hipErrorInvalidValue;
  if (nontemporal)
    hipLaunchKernelGGL(ft_copy_kernel<true>, dim3(workgroups), dim3(kThreads), 0, stream, T);
  else
    hipLaunchKernelGGL(ft_copy_kernel<false>, dim3(workgroups), dim3(kThreads), 0, stream, T);
  return hipGetLastError();
}

hipError_t launch_decode(const ClassTable &T, uint32_t *func_out, uint32_t *chunk_out, uint64_t cap,
                         hipStream_t stream) {
  uint64_t n = T.nchunks < cap ? T.nchunks : cap;
  if (n == 0) return hipSuccess;
  uint32_t blocks = (uint32_t)((n + 255) / 256);
  hipLaunchKernelGGL(ft_decode_kernel, dim3(blocks), dim3(256), 0, stream, T, func_out, chunk_out, cap);
  return hipGetLastError();
}

hipError_t launch_plain_copy(void *dst, const void *src, uint64_t bytes, uint32_t workgroups, hipStream_t stream) {
  if (bytes == 0) return hipSuccess;
  if (workgroups == 0) workgroups = 2048;
  hipLaunchKernelGGL(ft_plain_copy_kernel, dim3(workgroups), dim3(kThreads), 0, stream,
                     static_cast<u32x4 *>(dst), static_cast<const u32x4 *>(src), bytes >> 4);
  return hipGetLastError();
}

}  // namespace ft
