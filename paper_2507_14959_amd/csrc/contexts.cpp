// Host side of the selector: context construction from a co-occurrence matrix (Alg. 1, Sec. 3.4) and the three
// quality metrics of Sec. 3.4 (IntraCoherence, Eq. 6; AvgCoverage; SwitchPenalty).  Offline work on K <= 1024 labels:
// plain C++ on host memory, no device code.
#include <algorithm>
#include <cstdint>
#include <cstring>
#include <numeric>
#include <vector>

#include "../../include/poly.h"

namespace {

// a label set as a bit mask over K <= POLY_MAX_LABELS labels
struct LabelSet {
    uint64_t w[POLY_MAX_LABELS / 64];
    LabelSet() { std::memset(w, 0, sizeof(w)); }
    void add(int l) { w[l >> 6] |= 1ull << (l & 63); }
    bool has(int l) const { return (w[l >> 6] >> (l & 63)) & 1; }
    bool operator==(const LabelSet &o) const { return std::memcmp(w, o.w, sizeof(w)) == 0; }
    int size() const
    {
        int n = 0;
        for (uint64_t x : w) n += __builtin_popcountll(x);
        return n;
    }
};

}  // namespace

extern "C" int poly_build_contexts(const float *cooc, int K, int B, int M_max, int allow_overlap, uint8_t *group_membership,
                                   int32_t *n_contexts, int32_t *n_unplaced)
{
    if (!cooc || !group_membership || !n_contexts) return POLY_EINVAL;
    if (K <= 0 || K > POLY_MAX_LABELS || B <= 0 || M_max <= 0 || M_max > POLY_MAX_CONTEXTS) return POLY_EINVAL;
    auto co = [&](int i, int j) { return cooc[(size_t)i * K + j]; };

    // valid labels, most frequent first (stable: equal counts keep ascending ids)
    std::vector<int> visit;
    for (int l = 0; l < K; ++l)
        if (std::any_of(cooc + (size_t)l * K, cooc + (size_t)(l + 1) * K, [](float v) { return v != 0.f; })) visit.push_back(l);
    std::stable_sort(visit.begin(), visit.end(), [&](int a, int b) { return co(a, a) > co(b, b); });

    std::vector<LabelSet> ctx;
    LabelSet assigned;
    std::vector<int> nb;
    for (int l : visit) {
        if (!allow_overlap && assigned.has(l)) continue;
        // candidate neighbours: positive co-occurrence with l, still free when contexts may not overlap
        nb.clear();
        for (int j = 0; j < K; ++j)
            if (j != l && co(l, j) > 0.f && (allow_overlap || !assigned.has(j))) nb.push_back(j);
        const size_t take = std::min(nb.size(), (size_t)(B - 1));
        std::partial_sort(nb.begin(), nb.begin() + take, nb.end(),
                          [&](int a, int b) { return co(l, a) != co(l, b) ? co(l, a) > co(l, b) : a < b; });
        LabelSet c;
        c.add(l);
        for (size_t i = 0; i < take; ++i) c.add(nb[i]);
        if ((int)ctx.size() < M_max && std::find(ctx.begin(), ctx.end(), c) == ctx.end()) {
            ctx.push_back(c);
            if (!allow_overlap)
                for (size_t i = 0; i < sizeof(c.w) / sizeof(c.w[0]); ++i) assigned.w[i] |= c.w[i];
        }
    }

    // labels that ended up in no context go where they fit best among the contexts that still have room
    int left_out = 0;
    std::vector<int> fill(ctx.size());
    for (size_t c = 0; c < ctx.size(); ++c) fill[c] = ctx[c].size();
    for (int l : visit) {
        if (std::any_of(ctx.begin(), ctx.end(), [&](const LabelSet &c) { return c.has(l); })) continue;
        int best = -1;
        double best_fit = 0.0;
        for (size_t c = 0; c < ctx.size(); ++c) {
            if (fill[c] >= B) continue;
            double fit = 0.0;
            for (int j = 0; j < K; ++j)
                if (ctx[c].has(j)) fit += (double)co(l, j);
            if (best < 0 || fit > best_fit) { best = (int)c; best_fit = fit; }
        }
        if (best < 0) { ++left_out; continue; }
        ctx[best].add(l);
        ++fill[best];
    }

    std::memset(group_membership, 0, (size_t)M_max * K);
    for (size_t c = 0; c < ctx.size(); ++c)
        for (int l = 0; l < K; ++l) group_membership[c * K + l] = ctx[c].has(l) ? 1 : 0;
    *n_contexts = (int32_t)ctx.size();
    if (n_unplaced) *n_unplaced = left_out;
    return POLY_OK;
}

extern "C" int poly_intra_coherence(const float *cooc, int K, double norm, const uint8_t *group_membership, int M, double *out)
{
    if (!cooc || !group_membership || !out || K <= 0 || M < 0 || norm == 0.0) return POLY_EINVAL;
    double total = 0.0;
    std::vector<int> labels;
    for (int c = 0; c < M; ++c) {
        labels.clear();
        for (int l = 0; l < K; ++l)
            if (group_membership[(size_t)c * K + l]) labels.push_back(l);
        const size_t n = labels.size();
        if (n < 2) continue;                       // no pair: contributes nothing
        double pairs = 0.0;
        for (size_t a = 0; a < n; ++a)
            for (size_t b = 0; b < n; ++b)
                if (a != b) pairs += (double)cooc[(size_t)labels[a] * K + labels[b]];
        total += pairs / norm / (double)(n * (n - 1));
    }
    *out = M > 0 ? total / M : 0.0;
    return POLY_OK;
}

extern "C" int poly_stream_metrics(const int32_t *row_offsets, const int32_t *adapter_ids, int F, int M, double *avg_coverage,
                                   int64_t *switch_penalty)
{
    if (!row_offsets || F < 0 || M <= 0 || M > POLY_MAX_CONTEXTS || !avg_coverage || !switch_penalty) return POLY_EINVAL;
    if (F > 0 && row_offsets[F] > 0 && !adapter_ids) return POLY_EINVAL;
    uint64_t prev = 0;
    int64_t switches = 0;
    for (int t = 0; t < F; ++t) {
        if (row_offsets[t] > row_offsets[t + 1] || row_offsets[t] < 0) return POLY_ERANGE;
        uint64_t cur = 0;                          // S_t as a set: the order inside a frame does not count as a change
        for (int i = row_offsets[t]; i < row_offsets[t + 1]; ++i) {
            if (adapter_ids[i] < 0 || adapter_ids[i] >= M) return POLY_ERANGE;
            cur |= 1ull << adapter_ids[i];
        }
        if (t > 0 && cur != prev) ++switches;
        prev = cur;
    }
    *avg_coverage = F > 0 ? (double)(row_offsets[F] - row_offsets[0]) / F : 0.0;
    *switch_penalty = switches;
    return POLY_OK;
}
