// Offline cluster-combination selection of the paper's Sec. 4.2 (Algorithm 1), host only.
// A sample is the ordered list of clusters it activates.  Adding a prefix p whose parent is
// already cached (or that is a single cluster) raises the coverage by exactly the number of
// samples that start with p: each of them had len(p) - 1 leading hits and now has len(p).  So the
// greedy rounds are a best-first walk over the prefix tree by that count: a frontier ordered by
// (count descending, prefix ascending), O((prefixes + budget) log prefixes) instead of
// re-evaluating the coverage of every candidate every round.
#pragma once

#include <cstdint>
#include <map>
#include <set>
#include <vector>

namespace ax {

using ClusterSeq = std::vector<int32_t>;

struct SelectionResult {
    std::vector<ClusterSeq> chosen;       // in the order chosen
    std::vector<int64_t> coverage;        // coverage after each choice
};

inline SelectionResult select_combinations(const std::vector<ClusterSeq>& samples, int budget) {
    struct Node { int64_t count = 0; std::vector<ClusterSeq> children; };
    std::map<ClusterSeq, Node> tree;
    for (const ClusterSeq& s : samples) {
        ClusterSeq p;
        for (int32_t c : s) {
            ClusterSeq parent = p;
            p.push_back(c);
            Node& n = tree[p];
            if (n.count++ == 0 && !parent.empty()) tree[parent].children.push_back(p);
        }
    }
    struct Cand {
        int64_t count; const ClusterSeq* p;
        bool operator<(const Cand& o) const { return count != o.count ? count > o.count : *p < *o.p; }
    };
    std::set<Cand> frontier;
    for (auto& kv : tree)
        if (kv.first.size() == 1) frontier.insert({kv.second.count, &kv.first});
    SelectionResult r;
    int64_t cov = 0;
    for (int i = 0; i < budget && !frontier.empty(); ++i) {
        const Cand best = *frontier.begin();
        frontier.erase(frontier.begin());
        cov += best.count;
        r.chosen.push_back(*best.p);
        r.coverage.push_back(cov);
        for (const ClusterSeq& ch : tree[*best.p].children) {
            auto it = tree.find(ch);
            frontier.insert({it->second.count, &it->first});
        }
    }
    return r;
}

// Sum over the samples of the number of leading clusters found in `cached`.
inline int64_t coverage(const std::vector<ClusterSeq>& samples, const std::vector<ClusterSeq>& cached) {
    std::set<ClusterSeq> have(cached.begin(), cached.end());
    int64_t total = 0;
    for (const ClusterSeq& s : samples) {
        ClusterSeq p;
        size_t best = 0;
        for (int32_t c : s) {
            p.push_back(c);
            if (have.count(p)) best = p.size();
        }
        total += (int64_t)best;
    }
    return total;
}

}  // namespace ax
