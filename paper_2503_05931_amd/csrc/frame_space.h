// First-fit allocator over the frame axis of the cross-attention K/V cache
// (host side; used by the request queue).  Free intervals are kept sorted and
// merged, so with every request released the whole axis is one interval again:
// a request no longer than the axis can always be placed once nothing else runs.
#pragma once
#include <utility>
#include <vector>

namespace aed {

class FrameSpace {
public:
    explicit FrameSpace(int total) { free_.push_back({0, total}); }
    // first frame of a free run of n frames (n >= 1), or -1
    int take(int n) {
        for (size_t i = 0; i < free_.size(); ++i)
            if (free_[i].second >= n) {
                const int at = free_[i].first;
                free_[i].first += n;
                free_[i].second -= n;
                if (free_[i].second == 0) free_.erase(free_.begin() + i);
                return at;
            }
        return -1;
    }
    // give back exactly what take returned
    void give(int at, int n) {
        size_t i = 0;
        while (i < free_.size() && free_[i].first < at) ++i;
        free_.insert(free_.begin() + i, {at, n});
        if (i + 1 < free_.size() && free_[i].first + free_[i].second == free_[i + 1].first) {
            free_[i].second += free_[i + 1].second;
            free_.erase(free_.begin() + i + 1);
        }
        if (i > 0 && free_[i - 1].first + free_[i - 1].second == free_[i].first) {
            free_[i - 1].second += free_[i].second;
            free_.erase(free_.begin() + i);
        }
    }
    const std::vector<std::pair<int, int>>& free_runs() const { return free_; }  // (start, length), ascending

private:
    std::vector<std::pair<int, int>> free_;
};

}  // namespace aed
