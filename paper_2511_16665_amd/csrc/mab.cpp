// Host-side strategy selector: the Bucketed-Epsilon-Greedy bandit of Algorithm 1 (Section 5.2) and
// the elastic activation threshold of Section 5.1.  No GPU work; see include/tlt.h for the contract.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <limits>
#include <new>
#include <vector>

#include "../../include/tlt.h"

namespace {

// last `cap` values, oldest overwritten first
struct Window {
    std::vector<double> buf;
    size_t cap = 0, head = 0, count = 0;
    void push(double x) {
        buf[(head + count) % cap] = x;
        if (count < cap)
            ++count;
        else
            head = (head + 1) % cap;
    }
    double median() const {
        if (count == 0) return std::numeric_limits<double>::infinity();
        std::vector<double> v(count);
        for (size_t i = 0; i < count; ++i) v[i] = buf[(head + i) % cap];
        std::sort(v.begin(), v.end());
        return (count & 1) ? v[count / 2] : (v[count / 2 - 1] + v[count / 2]) / 2.0;
    }
};

}  // namespace

struct tlt_mab {
    std::vector<tlt_strategy> strategies;
    std::vector<int32_t> thresholds;
    std::vector<std::vector<int>> groups;   // groups[i]: strategy indices with the i-th largest Tokens_to_Verify
    std::vector<Window> rewards, lengths;
    double epsilon;
    int sd_threshold;
};

extern "C" {

int tlt_mab_create(const tlt_strategy* strategies, int n_strategies, const int32_t* thresholds, int n_thresholds,
                   double epsilon, int window, int sd_threshold, tlt_mab** out) {
    if (!strategies || !thresholds || !out || n_strategies < 1 || n_thresholds < 1 || window < 1 || !(epsilon >= 0.0) ||
        !(epsilon <= 1.0) || sd_threshold < 1)
        return TLT_EINVAL;
    for (int i = 0; i + 1 < n_thresholds; ++i)
        if (thresholds[i] >= thresholds[i + 1]) return TLT_EINVAL;
    std::vector<int32_t> widths;
    for (int i = 0; i < n_strategies; ++i) {
        if (strategies[i].tokens_to_verify < 1 || strategies[i].draft_depth < 0 || strategies[i].topk < 0) return TLT_EINVAL;
        widths.push_back(strategies[i].tokens_to_verify);
    }
    std::sort(widths.begin(), widths.end(), [](int32_t a, int32_t b) { return a > b; });
    widths.erase(std::unique(widths.begin(), widths.end()), widths.end());
    if ((int)widths.size() != n_thresholds) return TLT_EINVAL;
    tlt_mab* m = new (std::nothrow) tlt_mab();
    if (!m) return TLT_EINVAL;
    m->strategies.assign(strategies, strategies + n_strategies);
    m->thresholds.assign(thresholds, thresholds + n_thresholds);
    m->groups.resize(widths.size());
    for (size_t g = 0; g < widths.size(); ++g)
        for (int i = 0; i < n_strategies; ++i)
            if (strategies[i].tokens_to_verify == widths[g]) m->groups[g].push_back(i);
    m->rewards.resize(n_strategies);
    m->lengths.resize(n_strategies);
    for (int i = 0; i < n_strategies; ++i) {
        m->rewards[i].buf.assign(window, 0.0);
        m->rewards[i].cap = window;
        m->lengths[i].buf.assign(window, 0.0);
        m->lengths[i].cap = window;
    }
    m->epsilon = epsilon;
    m->sd_threshold = sd_threshold;
    *out = m;
    return TLT_OK;
}

void tlt_mab_destroy(tlt_mab* mab) { delete mab; }

int tlt_mab_select(tlt_mab* mab, int batch_size, uint32_t u1, uint32_t u2, int32_t* strategy) {
    if (!mab || !strategy || batch_size < 0) return TLT_EINVAL;
    if (batch_size >= mab->sd_threshold) {
        *strategy = -1;
        return TLT_OK;
    }
    size_t bucket = 0;
    for (size_t j = 0; j < mab->thresholds.size(); ++j)
        if (batch_size >= mab->thresholds[j]) bucket = j;
    const std::vector<int>& cand = mab->groups[bucket];
    if (cand.size() == 1) {
        *strategy = cand[0];
        return TLT_OK;
    }
    const double u = ((double)u1 + 0.5) / 4294967296.0;
    if (u < mab->epsilon) {
        *strategy = cand[(size_t)(((uint64_t)u2 * (uint64_t)cand.size()) >> 32)];
        return TLT_OK;
    }
    int best = cand[0];
    double best_median = mab->rewards[best].median();
    for (size_t i = 1; i < cand.size(); ++i) {
        const double med = mab->rewards[cand[i]].median();
        if (med > best_median) {
            best = cand[i];
            best_median = med;
        }
    }
    *strategy = best;
    return TLT_OK;
}

int tlt_mab_record(tlt_mab* mab, int strategy, double elapsed_time, const int32_t* accept_lens, int batch_size,
                   double* a_bar, double* reward) {
    if (!mab || !accept_lens || strategy < 0 || strategy >= (int)mab->strategies.size() || batch_size < 1 ||
        !(elapsed_time > 0.0))
        return TLT_EINVAL;
    int64_t total = 0;
    for (int i = 0; i < batch_size; ++i) {
        if (accept_lens[i] < 0) return TLT_EINVAL;
        total += accept_lens[i];
    }
    const double a = (double)total / (double)batch_size + 1.0;
    const double r = a * (double)batch_size / elapsed_time;
    mab->rewards[strategy].push(r);
    mab->lengths[strategy].push(a);
    if (a_bar) *a_bar = a;
    if (reward) *reward = r;
    return TLT_OK;
}

int tlt_mab_median_reward(const tlt_mab* mab, int strategy, double* median, int32_t* count) {
    if (!mab || strategy < 0 || strategy >= (int)mab->strategies.size()) return TLT_EINVAL;
    if (median) *median = mab->rewards[strategy].median();
    if (count) *count = (int32_t)mab->rewards[strategy].count;
    return TLT_OK;
}

}  // extern "C"
