#include "pool.hpp"

namespace dm {

static size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

Pool::Pool(void* base, size_t bytes)
{
    uintptr_t b = reinterpret_cast<uintptr_t>(base);
    uintptr_t aligned = round_up(b, kAlign);
    size_t lost = aligned - b;
    base_ = aligned;
    // the last kAlign bytes of the slab are never handed out: a 16-byte load that starts inside
    // the last allocation may run a few bytes past its end and must still hit owned memory
    cap_ = bytes > lost + kAlign ? (bytes - lost - kAlign) / kAlign * kAlign : 0;
    if (cap_) free_[0] = cap_;
}

void* Pool::alloc(size_t bytes)
{
    size_t need = round_up(bytes ? bytes : 1, kAlign);
    for (auto it = free_.begin(); it != free_.end(); ++it) {  // first fit, lowest address
        if (it->second < need) continue;
        uintptr_t off = it->first;
        size_t len = it->second;
        free_.erase(it);
        if (len > need) free_[off + need] = len - need;
        used_[off] = need;
        in_use_ += need;
        if (in_use_ > high_) high_ = in_use_;
        return reinterpret_cast<void*>(base_ + off);
    }
    return nullptr;
}

bool Pool::free(void* p)
{
    uintptr_t off = reinterpret_cast<uintptr_t>(p) - base_;
    auto u = used_.find(off);
    if (u == used_.end()) return false;
    size_t len = u->second;
    used_.erase(u);
    in_use_ -= len;
    auto next = free_.lower_bound(off);
    if (next != free_.end() && off + len == next->first) {  // merge with the range after
        len += next->second;
        next = free_.erase(next);
    }
    if (next != free_.begin()) {  // merge with the range before
        auto prev = std::prev(next);
        if (prev->first + prev->second == off) {
            prev->second += len;
            return true;
        }
    }
    free_[off] = len;
    return true;
}

}  // namespace dm
