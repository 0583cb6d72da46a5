// The block list of the striped arena: which stretches of a range of `bytes` are handed out.
// Host only, no device call: offsets are relative to the start of the range.  First fit; a
// freed block joins the free stretches on either side of it, so free stretches never adjoin.
#ifndef KDN_BLOCKLIST_H
#define KDN_BLOCKLIST_H

#include <algorithm>
#include <cstddef>
#include <iterator>
#include <map>

namespace kdn_impl {

class BlockList {
public:
    BlockList() = default;
    BlockList(size_t bytes, size_t align) : bytes_(bytes), align_(align)
    {
        if (bytes)
            free_at_[0] = bytes;
    }

    size_t bytes() const { return bytes_; }

    // Cuts `want` bytes (rounded up to the alignment) from the first free stretch that holds
    // them.  false if want is 0 or no stretch is long enough.
    bool take(size_t want, size_t *offset)
    {
        if (want == 0 || want > bytes_)
            return false;
        const size_t len = (want + align_ - 1) / align_ * align_;
        for (auto f = free_at_.begin(); f != free_at_.end(); ++f) {
            if (f->second < len)
                continue;
            const size_t off = f->first, had = f->second;
            free_at_.erase(f);
            if (had > len)
                free_at_[off + len] = had - len;
            used_at_[off] = len;
            *offset = off;
            return true;
        }
        return false;
    }

    // Gives a block back; false if `offset` is not the start of a block that is handed out.
    bool give(size_t offset)
    {
        auto u = used_at_.find(offset);
        if (u == used_at_.end())
            return false;
        size_t off = u->first, len = u->second;
        used_at_.erase(u);
        auto after = free_at_.lower_bound(off);
        if (after != free_at_.end() && after->first == off + len) { // joins the free stretch behind it
            len += after->second;
            after = free_at_.erase(after);
        }
        if (after != free_at_.begin()) {
            auto before = std::prev(after);
            if (before->first + before->second == off) { // and the one in front
                off = before->first;
                len += before->second;
                free_at_.erase(before);
            }
        }
        free_at_[off] = len;
        return true;
    }

    size_t in_use() const
    {
        size_t n = 0;
        for (const auto &kv : used_at_)
            n += kv.second;
        return n;
    }

    size_t largest_free() const
    {
        size_t m = 0;
        for (const auto &kv : free_at_)
            m = std::max(m, kv.second);
        return m;
    }

    size_t free_stretches() const { return free_at_.size(); }

private:
    size_t bytes_ = 0, align_ = 1;
    std::map<size_t, size_t> free_at_; // offset -> length, disjoint, never adjacent
    std::map<size_t, size_t> used_at_; // offset -> length
};

} // namespace kdn_impl
#endif // KDN_BLOCKLIST_H
