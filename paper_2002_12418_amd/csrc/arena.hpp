// One memory pool for a whole chain of operators (Section 3.2 of the MNN paper, "preparation-execution
// decoupling"): sizes and lifetimes of all buffers are known before anything runs, so the operators are
// walked in order without executing them, every buffer is taken from the pool at its first use and handed
// back after its last one, and the pool's high-water mark is what gets allocated once.  Host only.
#pragma once
#include <algorithm>
#include <utility>
#include <vector>

namespace mnnconv {

struct ArenaBuffer {
    long long bytes;   // >= 0
    int first, last;   // index of the first and the last operator that touches the buffer, first <= last
};

// Second placement rule, used as a cross-check on the walk: buffers in order of decreasing size, each at
// the lowest offset that is free over its whole lifetime.  It sees all lifetimes at once and so avoids the
// holes a strictly chronological walk can leave behind a buffer that is still alive.
inline long long place_by_size(const std::vector<ArenaBuffer>& bufs, const std::vector<long long>& size,
                               std::vector<long long>* offsets)
{
    const int n = (int)bufs.size();
    std::vector<int> order(n), placed;
    for (int i = 0; i < n; ++i) order[i] = i;
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return size[a] > size[b]; });
    offsets->assign(n, 0);
    long long pool = 0;
    for (int i : order) {
        if (size[i] == 0) continue;
        std::vector<std::pair<long long, long long>> busy;      // [begin, end) of placed buffers alive with i
        for (int j : placed)
            if (bufs[j].first <= bufs[i].last && bufs[i].first <= bufs[j].last)
                busy.push_back(std::make_pair((*offsets)[j], (*offsets)[j] + size[j]));
        std::sort(busy.begin(), busy.end());
        long long off = 0;
        for (const auto& iv : busy) {
            if (off + size[i] <= iv.first) break;
            off = std::max(off, iv.second);
        }
        (*offsets)[i] = off;
        pool = std::max(pool, off + size[i]);
        placed.push_back(i);
    }
    return pool;
}

// Writes one offset per buffer (multiples of `align`, a power of two) and the pool size.  Two buffers whose
// lifetimes intersect never overlap in memory.  Returns false on malformed input.
inline bool plan_arena(const std::vector<ArenaBuffer>& bufs, long long align, std::vector<long long>* offsets,
                       long long* total)
{
    if (align <= 0 || (align & (align - 1)) != 0 || !offsets || !total) return false;
    const int n = (int)bufs.size();
    offsets->assign(n, 0);
    *total = 0;
    int ops = 0;
    for (const ArenaBuffer& b : bufs) {
        if (b.bytes < 0 || b.first < 0 || b.last < b.first) return false;
        ops = std::max(ops, b.last + 1);
    }
    std::vector<long long> size(n);
    for (int i = 0; i < n; ++i) size[i] = (bufs[i].bytes + align - 1) / align * align;

    std::vector<std::pair<long long, long long>> holes;   // (offset, bytes), sorted by offset, never adjacent
    long long pool = 0;
    auto give_back = [&](long long off, long long bytes) {
        auto it = std::lower_bound(holes.begin(), holes.end(), std::make_pair(off, 0ll));
        it = holes.insert(it, std::make_pair(off, bytes));
        if (it + 1 != holes.end() && it->first + it->second == (it + 1)->first) {
            it->second += (it + 1)->second;
            it = holes.erase(it + 1) - 1;
        }
        if (it != holes.begin() && (it - 1)->first + (it - 1)->second == it->first) {
            (it - 1)->second += it->second;
            holes.erase(it);
        }
    };
    auto take = [&](long long bytes) -> long long {
        int best = -1;
        for (int h = 0; h < (int)holes.size(); ++h)
            if (holes[h].second >= bytes && (best < 0 || holes[h].second < holes[best].second)) best = h;
        if (best >= 0) {
            const long long off = holes[best].first;
            if (holes[best].second == bytes) holes.erase(holes.begin() + best);
            else { holes[best].first += bytes; holes[best].second -= bytes; }
            return off;
        }
        // nothing fits: grow the pool, starting inside a hole that touches its end
        long long off = pool;
        if (!holes.empty() && holes.back().first + holes.back().second == pool) {
            off = holes.back().first;
            holes.pop_back();
        }
        pool = off + bytes;
        return off;
    };

    std::vector<int> order(n);
    for (int i = 0; i < n; ++i) order[i] = i;
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return size[a] > size[b]; });
    for (int t = 0; t < ops; ++t) {
        for (int i = 0; i < n; ++i)
            if (size[i] > 0 && bufs[i].last == t - 1) give_back((*offsets)[i], size[i]);
        for (int i : order)
            if (size[i] > 0 && bufs[i].first == t) (*offsets)[i] = take(size[i]);
    }
    *total = pool;
    std::vector<long long> alt;
    const long long alt_pool = place_by_size(bufs, size, &alt);
    if (alt_pool < pool) {
        *offsets = alt;
        *total = alt_pool;
    }
    return true;
}

}  // namespace mnnconv
