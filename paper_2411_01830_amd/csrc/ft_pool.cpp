#include "ft_pool.h"

#include <cstddef>

#include "../../include/faastube.h"

namespace ft {

int SlabPool::check_segment(const void *base, uint64_t bytes, uint64_t slab_bytes) {
  if (base == nullptr) return FT_EINVAL;
  if (slab_bytes == 0 || slab_bytes % 256 != 0) return FT_EINVAL;
  if (bytes == 0 || bytes % slab_bytes != 0) return FT_EINVAL;
  if (reinterpret_cast<uintptr_t>(base) % 256 != 0) return FT_EINVAL;
  return FT_OK;
}

int SlabPool::add_segment(void *base, uint64_t bytes) {
  int rc = check_segment(base, bytes, slab_);
  if (rc != FT_OK) return rc;
  Segment s;
  s.base = static_cast<char *>(base);
  s.bytes = bytes;
  s.first_slab = total_slabs_;
  s.nslabs = bytes / slab_;
  segs_.push_back(s);
  free_runs_[s.first_slab] = s.nslabs;  // kept apart from the previous segment's tail run
  total_slabs_ += s.nslabs;
  return FT_OK;
}

int SlabPool::drop_last_segment(void **base_out, uint64_t *bytes_out) {
  if (segs_.size() < 2) return FT_EINVAL;
  const Segment s = segs_.back();
  // a segment without allocations is exactly one free run
  auto it = free_runs_.find(s.first_slab);
  if (it == free_runs_.end() || it->second != s.nslabs) return FT_EBUSY;
  free_runs_.erase(it);
  segs_.pop_back();
  total_slabs_ -= s.nslabs;
  if (base_out) *base_out = s.base;
  if (bytes_out) *bytes_out = s.bytes;
  return FT_OK;
}

uint64_t SlabPool::live_bytes() const {
  uint64_t n = 0;
  for (const auto &kv : allocs_) n += kv.second.nslabs;
  return n * slab_;
}

const Segment *SlabPool::segment_of_slab(uint64_t slab) const {
  size_t lo = 0, hi = segs_.size();
  if (hi == 0 || slab >= total_slabs_) return nullptr;
  while (hi - lo > 1) {
    size_t mid = (lo + hi) / 2;
    if (segs_[mid].first_slab <= slab) lo = mid; else hi = mid;
  }
  return &segs_[lo];
}

int SlabPool::alloc(uint64_t nbytes, uint64_t *off_out) {
  if (nbytes == 0 || off_out == nullptr) return FT_EINVAL;
  uint64_t need = nbytes / slab_ + (nbytes % slab_ != 0);
  // free runs are keyed by first slab, so the first run that is long enough is the
  // lowest-indexed fit
  for (auto it = free_runs_.begin(); it != free_runs_.end(); ++it) {
    if (it->second < need) continue;
    uint64_t start = it->first, len = it->second;
    free_runs_.erase(it);
    if (len > need) free_runs_[start + need] = len - need;
    Allocation a;
    a.nslabs = need;
    a.busy = 0;
    a.serial = next_serial_++;
    allocs_[start * slab_] = a;
    *off_out = start * slab_;
    return FT_OK;
  }
  return FT_ENOMEM;
}

int SlabPool::free(uint64_t off, bool ordered) {
  auto it = allocs_.find(off);
  if (it == allocs_.end()) return FT_EINVAL;
  if (it->second.busy != 0 && !ordered) return FT_EBUSY;
  uint64_t start = off / slab_, len = it->second.nslabs;
  allocs_.erase(it);
  const Segment *seg = segment_of_slab(start);
  // merge with the free neighbours that lie in the same segment
  auto next = free_runs_.find(start + len);
  if (next != free_runs_.end() && start + len < seg->first_slab + seg->nslabs) {
    len += next->second;
    free_runs_.erase(next);
  }
  auto after = free_runs_.lower_bound(start);
  if (after != free_runs_.begin()) {
    auto prev = std::prev(after);
    if (prev->first + prev->second == start && start > seg->first_slab) {
      prev->second += len;
      return FT_OK;
    }
  }
  free_runs_[start] = len;
  return FT_OK;
}

Allocation *SlabPool::owner(uint64_t off, uint64_t extent, uint64_t *start_out) {
  auto it = allocs_.upper_bound(off);
  if (it == allocs_.begin()) return nullptr;
  --it;
  uint64_t a0 = it->first, a1 = a0 + it->second.nslabs * slab_;
  if (off < a0 || off >= a1 || extent > a1 - off) return nullptr;
  if (start_out) *start_out = a0;
  return &it->second;
}

Allocation *SlabPool::at(uint64_t start) {
  auto it = allocs_.find(start);
  return it == allocs_.end() ? nullptr : &it->second;
}

void *SlabPool::ptr(uint64_t off) const {
  const Segment *seg = segment_of_slab(off / slab_);
  if (!seg) return nullptr;
  return seg->base + (off - seg->first_slab * slab_);
}

}  // namespace ft
