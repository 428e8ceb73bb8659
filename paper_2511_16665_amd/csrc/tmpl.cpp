// Host side of sampled drafting: the static tree template.  The paper's sampled rollouts
// (temperature 0.9, Section 6.1) must stay lossless (Section 1, Section 3 principle (a)), which a
// tree whose shape depends on the drawn tokens would break; so the shape is fixed by the three
// tree parameters of Section 5.1 alone.  No GPU work; see include/tlt.h for the contract.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <map>
#include <queue>
#include <vector>

#include "../../include/tlt.h"

namespace {

// a node of the full topk-ary tree = the child ranks on the way down to it
struct Node {
    std::vector<uint8_t> ranks;
    double weight;   // log of prod_j a0 (1-a0)^(r_j), a0 = 0.6
};

double log_weight(const std::vector<uint8_t>& ranks) {
    int sum = 0;
    for (uint8_t r : ranks) sum += r;
    return (double)ranks.size() * std::log(0.6) + (double)sum * std::log(1.0 - 0.6);
}

// "a comes out of the queue after b": lower weight, then deeper, then the larger rank sequence
struct Later {
    bool operator()(const Node& a, const Node& b) const {
        if (a.weight != b.weight) return a.weight < b.weight;
        if (a.ranks.size() != b.ranks.size()) return a.ranks.size() > b.ranks.size();
        return a.ranks > b.ranks;
    }
};

}  // namespace

extern "C" int tlt_template_build(int topk, int depth, int n_verify, int32_t* parent, int32_t* rank,
                                  int32_t* node_depth, int32_t* n_nodes) {
    if (topk < 1 || topk > TLT_MAX_TOPK || depth < 0 || depth > TLT_MAX_DEPTH || n_verify < 1 || n_verify > TLT_MAX_TREE ||
        !parent || !rank || !node_depth || !n_nodes)
        return TLT_EINVAL;
    // best-first walk: a node's first child and next sibling both weigh less than the node, and every
    // node is reached through that relation, so popping n_verify-1 times yields the heaviest nodes
    std::priority_queue<Node, std::vector<Node>, Later> open;
    if (depth >= 1) open.push({{0}, log_weight({0})});
    std::vector<std::vector<uint8_t>> kept;
    while (!open.empty() && (int)kept.size() < n_verify - 1) {
        Node nd = open.top();
        open.pop();
        kept.push_back(nd.ranks);
        if ((int)nd.ranks.size() < depth) {
            std::vector<uint8_t> c = nd.ranks;
            c.push_back(0);
            open.push({c, log_weight(c)});
        }
        if (nd.ranks.back() + 1 < topk) {
            std::vector<uint8_t> s = nd.ranks;
            ++s.back();
            open.push({s, log_weight(s)});
        }
    }
    // number by depth, then parent number, then rank: parents precede children and a node's
    // children are consecutive, in rank order
    std::map<std::vector<uint8_t>, int> number;
    number[{}] = 0;
    parent[0] = -1;
    rank[0] = -1;
    node_depth[0] = 0;
    int n = 1;
    for (int d = 1; d <= depth; ++d) {
        std::vector<std::pair<std::pair<int, int>, const std::vector<uint8_t>*>> level;
        for (const auto& r : kept)
            if ((int)r.size() == d) {
                std::vector<uint8_t> up(r.begin(), r.end() - 1);
                level.push_back({{number.at(up), (int)r.back()}, &r});
            }
        std::sort(level.begin(), level.end(), [](const auto& a, const auto& b) { return a.first < b.first; });
        for (const auto& e : level) {
            number[*e.second] = n;
            parent[n] = e.first.first;
            rank[n] = e.first.second;
            node_depth[n] = d;
            ++n;
        }
    }
    *n_nodes = n;
    return TLT_OK;
}
