// Sub-allocator over one caller-owned slab of GPU memory (paper section 1: unused GPU memory
// is pooled so that no driver allocation happens while the library runs).  Pure host logic:
// it hands out addresses and never dereferences them.
#pragma once
#include <cstddef>
#include <cstdint>
#include <map>

namespace dm {

class Pool {
public:
    static constexpr size_t kAlign = 256;
    Pool(void* base, size_t bytes);
    // nullptr when no free range is large enough.  Size 0 is treated as 1.
    void* alloc(size_t bytes);
    // p must come from alloc() of this pool; neighbours are merged.
    bool free(void* p);
    size_t in_use() const { return in_use_; }
    size_t high_water() const { return high_; }
    size_t capacity() const { return cap_; }
    size_t live_allocations() const { return used_.size(); }

private:
    uintptr_t base_;
    size_t cap_, in_use_ = 0, high_ = 0;
    std::map<uintptr_t, size_t> free_;  // offset -> length, non-adjacent
    std::map<uintptr_t, size_t> used_;  // offset -> length
};

}  // namespace dm
