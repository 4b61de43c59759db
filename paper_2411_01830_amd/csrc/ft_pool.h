// Host bookkeeping of the pooled GPU store (Sec. 7.1): segments of caller-owned
// device memory cut into slabs, first-fit runs, no device calls.
#pragma once
#include <stdint.h>
#include <map>
#include <vector>

namespace ft {

struct Segment {
  char *base;           // device pointer
  uint64_t bytes;
  uint64_t first_slab;  // index of its first slab in the logical space
  uint64_t nslabs;
};

struct Allocation {
  uint64_t nslabs;
  uint32_t busy;    // jobs not yet waited for that refer to it
  uint64_t serial;  // tells this allocation from an earlier one at the same offset
};

class SlabPool {
 public:
  // Argument rules of ft_pool_create; returns an FT_* code.
  static int check_segment(const void *base, uint64_t bytes, uint64_t slab_bytes);

  SlabPool(uint64_t slab_bytes) : slab_(slab_bytes) {}
  int add_segment(void *base, uint64_t bytes);
  // Drops the last segment if no allocation lies in it (FT_EBUSY otherwise; FT_EINVAL if
  // it is the only one): the pool never shrinks below its first segment.
  int drop_last_segment(void **base_out, uint64_t *bytes_out);
  uint64_t live_bytes() const;
  int alloc(uint64_t nbytes, uint64_t *off_out);
  // FT_EBUSY while a job that has not been waited for refers to the allocation, unless `ordered`:
  // then the caller vouches that whatever reuses the slabs is ordered after those jobs on the device.
  int free(uint64_t off, bool ordered = false);
  // Live allocation containing [off, off+extent), or nullptr. *start_out = its offset.
  Allocation *owner(uint64_t off, uint64_t extent, uint64_t *start_out);
  Allocation *at(uint64_t start);
  void *ptr(uint64_t off) const;
  uint64_t slab_bytes() const { return slab_; }
  uint64_t total_bytes() const { return total_slabs_ * slab_; }

 private:
  uint64_t slab_;
  uint64_t total_slabs_ = 0;
  uint64_t next_serial_ = 1;
  std::vector<Segment> segs_;
  std::map<uint64_t, uint64_t> free_runs_;   // first slab -> length; runs never cross a segment edge
  std::map<uint64_t, Allocation> allocs_;    // offset -> allocation
  const Segment *segment_of_slab(uint64_t slab) const;
};

}  // namespace ft
