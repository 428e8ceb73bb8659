// Host-side model-free drafter (Section 5.3): per-prompt n-gram retrieval database and the
// confidence-ordered candidate tree built from it.  No GPU work; see include/tlt.h for the contract.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <limits>
#include <new>
#include <unordered_map>
#include <vector>

#include "../../include/tlt.h"

namespace {

struct Key {
    int64_t prompt;
    std::vector<int32_t> ctx;
    bool operator==(const Key& o) const { return prompt == o.prompt && ctx == o.ctx; }
};
struct KeyHash {
    size_t operator()(const Key& k) const {
        uint64_t h = 0x9e3779b97f4a7c15ull ^ (uint64_t)k.prompt;
        for (int32_t t : k.ctx) {
            h ^= (uint64_t)(uint32_t)t + 0x9e3779b97f4a7c15ull + (h << 6) + (h >> 2);
            h *= 0xff51afd7ed558ccdull;
        }
        return (size_t)h;
    }
};
struct Next {
    std::vector<std::pair<int32_t, int64_t>> items;   // (token, count), unordered
    int64_t total = 0;
};
struct Cont {
    int32_t token;
    double logp;
};
struct Cand {
    int32_t token;
    double score;
    int parent;                  // pool index, -1 for children of the root
    std::vector<int32_t> path;   // tokens from the root's child down to this candidate
};

}  // namespace

struct tlt_ngram {
    int n;
    std::unordered_map<Key, Next, KeyHash> table;

    // continuations of the longest seen suffix of ctx, best first (count desc, token asc), at most k of them
    void continuations(int64_t prompt, const std::vector<int32_t>& ctx, int k, std::vector<Cont>& out) const {
        out.clear();
        const int maxlen = std::min<int>(n - 1, (int)ctx.size());
        Key key;
        key.prompt = prompt;
        for (int len = maxlen; len >= 1; --len) {
            key.ctx.assign(ctx.end() - len, ctx.end());
            auto it = table.find(key);
            if (it == table.end() || it->second.items.empty()) continue;
            std::vector<std::pair<int32_t, int64_t>> ranked = it->second.items;
            std::sort(ranked.begin(), ranked.end(), [](const auto& a, const auto& b) {
                return a.second != b.second ? a.second > b.second : a.first < b.first;
            });
            for (size_t i = 0; i < ranked.size() && (int)i < k; ++i)
                out.push_back({ranked[i].first, std::log((double)ranked[i].second / (double)it->second.total)});
            return;
        }
    }
};

extern "C" {

int tlt_ngram_create(int order, tlt_ngram** out) {
    if (!out || order < 2 || order > 64) return TLT_EINVAL;
    tlt_ngram* db = new (std::nothrow) tlt_ngram();
    if (!db) return TLT_EINVAL;
    db->n = order;
    *out = db;
    return TLT_OK;
}

void tlt_ngram_destroy(tlt_ngram* db) { delete db; }

int tlt_ngram_insert(tlt_ngram* db, int64_t prompt_id, const int32_t* tokens, int len) {
    if (!db || (!tokens && len > 0) || len < 0) return TLT_EINVAL;
    Key key;
    key.prompt = prompt_id;
    for (int k = 1; k < db->n; ++k)
        for (int i = 0; i + k < len; ++i) {
            key.ctx.assign(tokens + i, tokens + i + k);
            Next& nx = db->table[key];
            const int32_t t = tokens[i + k];
            auto it = std::find_if(nx.items.begin(), nx.items.end(), [t](const auto& p) { return p.first == t; });
            if (it == nx.items.end())
                nx.items.emplace_back(t, 1);
            else
                ++it->second;
            ++nx.total;
        }
    return TLT_OK;
}

int tlt_ngram_propose(const tlt_ngram* db, int64_t prompt_id, const int32_t* context, int context_len, int depth, int topk,
                      int n_nodes, int32_t* token, int32_t* parent, float* score) {
    if (!db || !context || context_len < 1 || depth < 0 || topk < 1 || n_nodes < 1 || !token || !parent) return TLT_EINVAL;
    std::vector<int32_t> ctx(context, context + context_len);
    std::vector<Cand> pool;
    std::vector<int> frontier;
    std::vector<Cont> cont;
    if (depth >= 1) {
        db->continuations(prompt_id, ctx, topk, cont);
        for (const Cont& c : cont) {
            pool.push_back({c.token, c.logp, -1, {c.token}});
            frontier.push_back((int)pool.size() - 1);
        }
    }
    std::vector<int32_t> full;
    for (int level = 1; level < depth && !frontier.empty(); ++level) {
        const int base = (int)pool.size();
        for (int pi : frontier) {
            full = ctx;
            full.insert(full.end(), pool[pi].path.begin(), pool[pi].path.end());
            db->continuations(prompt_id, full, topk, cont);
            for (const Cont& c : cont) {
                std::vector<int32_t> path = pool[pi].path;
                path.push_back(c.token);
                pool.push_back({c.token, pool[pi].score + c.logp, pi, std::move(path)});
            }
        }
        std::vector<int> fresh;
        for (int i = base; i < (int)pool.size(); ++i) fresh.push_back(i);
        std::stable_sort(fresh.begin(), fresh.end(), [&](int a, int b) { return pool[a].score > pool[b].score; });
        if ((int)fresh.size() > topk) fresh.resize(topk);
        frontier = fresh;
    }
    std::vector<int> order(pool.size());
    for (size_t i = 0; i < pool.size(); ++i) order[i] = (int)i;
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return pool[a].score > pool[b].score; });
    if ((int)order.size() > n_nodes - 1) order.resize(n_nodes - 1);
    std::sort(order.begin(), order.end());
    std::vector<int> node_of(pool.size(), -1);
    int n = 0;
    token[n] = ctx.back();
    parent[n] = -1;
    if (score) score[n] = 0.f;
    ++n;
    for (int pi : order) {
        node_of[pi] = n;
        token[n] = pool[pi].token;
        parent[n] = pool[pi].parent < 0 ? 0 : node_of[pool[pi].parent];
        if (score) score[n] = (float)pool[pi].score;
        ++n;
    }
    // padding: children of the root with the smallest token ids it has no child for yet
    int32_t next_tok = 0;
    while (n < n_nodes) {
        bool used = false;
        for (int i = 1; i < n; ++i)
            if (parent[i] == 0 && token[i] == next_tok) used = true;
        if (!used) {
            token[n] = next_tok;
            parent[n] = 0;
            if (score) score[n] = -std::numeric_limits<float>::infinity();
            ++n;
        }
        ++next_tok;
    }
    return TLT_OK;
}

}  // extern "C"
