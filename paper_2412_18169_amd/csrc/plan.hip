// Host-side planning routines around the attention path (no device work):
//   * the cost model of a chunk and of a microbatch (Section 4.3, Eq. 1-3) and its least-squares fit,
//   * the lookahead batch formulation (Section 4.3): recursive halving of the queued tokens into
//     cost-balanced microbatches,
//   * drop-plan generation (Section 4.1, Algorithm 1): merge the two smallest instance groups until the memory
//     demand is met; each merge drops one redundant copy of the parameters.
#include <math.h>

#include <algorithm>
#include <queue>
#include <vector>

#include "kun_internal.h"

namespace {

typedef long double ld;

inline double pairs(int64_t p, int64_t c) { return (double)p * (double)c + ((double)c * (double)c + (double)c) / 2.0; }

struct Sums {            // attention pairs, tokens and live chunks of a span of the queue
    double a = 0, c = 0;
    int n = 0;
};

inline double cost_of(const kun_cost_model& m, const Sums& s) {
    return s.n == 0 ? 0.0 : m.alpha * s.a + m.beta * s.c + m.gamma;
}

// One microbatch -> two, in queue order.  The cost of the left part grows and that of the right part
// shrinks with every token moved left, so the position with the smallest difference is next to the
// sign change of (left - right); among equal differences the earliest position wins.
void split(const kun_cost_model& m, const std::vector<kun_chunk>& b, std::vector<kun_chunk>& left,
           std::vector<kun_chunk>& right) {
    left.clear();
    right.clear();
    Sums all;
    for (const kun_chunk& ch : b) {
        all.a += pairs(ch.prior, ch.tokens);
        all.c += ch.tokens;
        all.n += 1;
    }
    if (all.n == 0) return;
    // f(i, k): left = chunks before i plus the first k tokens of chunk i
    auto diff = [&](const Sums& before, const kun_chunk& ch, int64_t k, int n_after) {
        Sums l = before, r;
        if (k > 0) {
            l.a += pairs(ch.prior, k);
            l.c += k;
            l.n += 1;
        }
        r.a = all.a - l.a;
        r.c = all.c - l.c;
        r.n = n_after + (k < ch.tokens ? 1 : 0);
        return cost_of(m, l) - cost_of(m, r);
    };
    Sums before;
    size_t i = 0;
    for (; i < b.size(); ++i) {                          // first chunk at whose end left >= right
        if (diff(before, b[i], b[i].tokens, (int)(b.size() - i - 1)) >= 0.0 || i + 1 == b.size()) break;
        before.a += pairs(b[i].prior, b[i].tokens);
        before.c += b[i].tokens;
        before.n += 1;
    }
    const kun_chunk& ch = b[i];
    const int n_after = (int)(b.size() - i - 1);
    int64_t lo = 0, hi = ch.tokens;                      // smallest k with diff >= 0 (hi if none)
    while (lo < hi) {
        const int64_t mid = lo + (hi - lo) / 2;
        if (diff(before, ch, mid, n_after) >= 0.0) hi = mid;
        else lo = mid + 1;
    }
    int64_t k = lo;
    if (k > 0 && fabs(diff(before, ch, k - 1, n_after)) <= fabs(diff(before, ch, k, n_after))) k -= 1;
    // k == 0 at chunk i is the same cut as k == tokens at chunk i - 1, which comes first
    for (size_t j = 0; j < i; ++j) left.push_back(b[j]);
    if (k > 0) left.push_back(kun_chunk{ch.request, ch.prior, (int32_t)k});
    if (k < ch.tokens) right.push_back(kun_chunk{ch.request, (int32_t)(ch.prior + k), (int32_t)(ch.tokens - k)});
    for (size_t j = i + 1; j < b.size(); ++j) right.push_back(b[j]);
}

int64_t tokens_of(const std::vector<kun_chunk>& b) {
    int64_t t = 0;
    for (const kun_chunk& ch : b) t += ch.tokens;
    return t;
}

}  // namespace

extern "C" {

double kun_cost_chunk(const kun_cost_model* m, int64_t prior, int64_t tokens) {
    if (!m || prior < 0 || tokens < 0) return NAN;
    return m->alpha * pairs(prior, tokens) + m->beta * (double)tokens + m->gamma;
}

double kun_cost_microbatch(const kun_cost_model* m, const kun_chunk* chunks, int n) {
    if (!m || n < 0 || (n > 0 && !chunks)) return NAN;
    Sums s;
    for (int i = 0; i < n; ++i) {
        if (chunks[i].tokens <= 0) continue;
        s.a += pairs(chunks[i].prior, chunks[i].tokens);
        s.c += chunks[i].tokens;
        s.n += 1;
    }
    return cost_of(*m, s);
}

int kun_cost_fit(const kun_chunk* chunks, const int32_t* mb_start, int n_microbatches, const double* seconds,
                 kun_cost_model* out) {
    if (!chunks || !mb_start || !seconds || !out || n_microbatches < 3) return KUN_ERR_INVALID_ARG;
    // normal equations of  t = alpha * A + beta * C + gamma  with the columns scaled to unit maximum
    std::vector<ld> A(n_microbatches), C(n_microbatches);
    ld sa = 0, sc = 0;
    for (int k = 0; k < n_microbatches; ++k) {
        if (mb_start[k + 1] < mb_start[k]) return KUN_ERR_INVALID_ARG;
        ld a = 0, c = 0;
        for (int i = mb_start[k]; i < mb_start[k + 1]; ++i) {
            if (chunks[i].tokens <= 0) continue;
            a += pairs(chunks[i].prior, chunks[i].tokens);
            c += chunks[i].tokens;
        }
        A[k] = a;
        C[k] = c;
        sa = std::max(sa, a);
        sc = std::max(sc, c);
    }
    if (sa == 0 || sc == 0) return KUN_ERR_INVALID_ARG;
    ld M[3][4] = {};
    for (int k = 0; k < n_microbatches; ++k) {
        const ld row[3] = {A[k] / sa, C[k] / sc, 1};
        for (int r = 0; r < 3; ++r) {
            for (int c = 0; c < 3; ++c) M[r][c] += row[r] * row[c];
            M[r][3] += row[r] * seconds[k];
        }
    }
    for (int col = 0; col < 3; ++col) {                  // Gauss-Jordan with partial pivoting
        int piv = col;
        for (int r = col + 1; r < 3; ++r)
            if (fabsl(M[r][col]) > fabsl(M[piv][col])) piv = r;
        if (fabsl(M[piv][col]) < 1e-18L) return KUN_ERR_INVALID_ARG;     // the samples do not determine the model
        for (int c = 0; c < 4; ++c) std::swap(M[col][c], M[piv][c]);
        for (int r = 0; r < 3; ++r) {
            if (r == col) continue;
            const ld f = M[r][col] / M[col][col];
            for (int c = col; c < 4; ++c) M[r][c] -= f * M[col][c];
        }
    }
    out->alpha = (double)(M[0][3] / M[0][0] / sa);
    out->beta = (double)(M[1][3] / M[1][1] / sc);
    out->gamma = (double)(M[2][3] / M[2][2]);
    return KUN_OK;
}

int kun_lookahead(const kun_cost_model* m, const kun_chunk* queue, int n, int min_tokens, int max_microbatches,
                  kun_chunk* out_chunks, int chunk_capacity, int32_t* out_mb_start, int mb_capacity,
                  int* n_microbatches, int* n_chunks) {
    if (!m || n < 0 || (n > 0 && !queue) || min_tokens < 1 || max_microbatches < 0 || !out_chunks ||
        !out_mb_start || !n_microbatches || !n_chunks || chunk_capacity < 0 || mb_capacity < 1)
        return KUN_ERR_INVALID_ARG;
    if (m->alpha < 0 || m->beta < 0 || m->gamma < 0) return KUN_ERR_INVALID_ARG;
    std::vector<std::vector<kun_chunk>> level(1), next;
    for (int i = 0; i < n; ++i) {
        if (queue[i].tokens < 0 || queue[i].prior < 0) return KUN_ERR_INVALID_ARG;
        if (queue[i].tokens > 0) level[0].push_back(queue[i]);
    }
    std::vector<kun_chunk> l, r;
    for (;;) {                                           // one level of halving per pass
        if (max_microbatches && 2 * level.size() > (size_t)max_microbatches) break;
        next.clear();
        bool changed = false;
        for (const std::vector<kun_chunk>& b : level) {
            split(*m, b, l, r);
            if (tokens_of(l) >= min_tokens && tokens_of(r) >= min_tokens) {
                next.push_back(l);
                next.push_back(r);
                changed = true;
            } else {
                next.push_back(b);
            }
        }
        if (!changed) break;
        if (max_microbatches && next.size() > (size_t)max_microbatches) break;
        level.swap(next);
    }
    size_t total = 0;
    for (const auto& b : level) total += b.size();
    if (level.size() > (size_t)mb_capacity || total > (size_t)chunk_capacity) return KUN_ERR_TOO_SMALL;
    int o = 0;
    for (size_t k = 0; k < level.size(); ++k) {
        out_mb_start[k] = o;
        for (const kun_chunk& ch : level[k]) out_chunks[o++] = ch;
    }
    out_mb_start[level.size()] = o;
    *n_microbatches = (int)level.size();
    *n_chunks = o;
    return KUN_OK;
}

int kun_drop_plan(int n_instances, const int32_t* initial_group, int num_layers, int64_t layer_bytes,
                  int64_t demand_bytes, int32_t* group_of_instance, int32_t* kept_first, int32_t* kept_end,
                  int64_t* dropped_bytes, int32_t* merge_members, int32_t* merge_sizes, int* n_merges,
                  int64_t* freed_bytes, int* demand_met) {
    if (n_instances < 1 || num_layers < 1 || layer_bytes < 1 || demand_bytes < 0 || !group_of_instance ||
        !kept_first || !kept_end || !dropped_bytes || !n_merges || !freed_bytes || !demand_met)
        return KUN_ERR_INVALID_ARG;
    const int N = n_instances;
    // groups as linked lists of instances (constant-time merge); `head` doubles as the group's name
    std::vector<int> next(N, -1), tail(N), size(N, 0), head_of(N, -1);
    std::vector<int> heads;
    if (initial_group) {
        std::vector<int> first(N, -1);
        for (int i = 0; i < N; ++i) {
            const int g = initial_group[i];
            if (g < 0 || g >= N) return KUN_ERR_INVALID_ARG;
            if (first[g] < 0) {
                first[g] = i;
                tail[i] = i;
                heads.push_back(i);
            } else {
                next[tail[first[g]]] = i;
                tail[first[g]] = i;
            }
            size[first[g]] += 1;
        }
        // creation order of the initial groups: by group number
        std::sort(heads.begin(), heads.end(), [&](int a, int b) { return initial_group[a] < initial_group[b]; });
    } else {
        for (int i = 0; i < N; ++i) {
            tail[i] = i;
            size[i] = 1;
            heads.push_back(i);
        }
    }
    struct Entry {
        int size, order, head;
        bool operator>(const Entry& o) const { return size != o.size ? size > o.size : order > o.order; }
    };
    std::priority_queue<Entry, std::vector<Entry>, std::greater<Entry>> q;
    int order = 0;
    for (int h : heads) q.push(Entry{size[h], order++, h});
    const int64_t copy_bytes = (int64_t)num_layers * layer_bytes;
    int64_t freed = 0;
    int merges = 0;
    while (freed < demand_bytes && q.size() >= 2) {
        const Entry a = q.top(); q.pop();
        const Entry b = q.top(); q.pop();
        if (merge_members) {
            merge_members[2 * merges] = a.head;
            merge_members[2 * merges + 1] = b.head;
        }
        if (merge_sizes) {
            merge_sizes[2 * merges] = a.size;
            merge_sizes[2 * merges + 1] = b.size;
        }
        next[tail[a.head]] = b.head;                     // b's list goes behind a's
        tail[a.head] = tail[b.head];
        size[a.head] = a.size + b.size;
        q.push(Entry{a.size + b.size, order++, a.head});
        freed += copy_bytes;
        ++merges;
    }
    // final groups, numbered by their smallest instance; stage j of a group is its j-th smallest instance
    std::vector<std::vector<int>> groups;
    while (!q.empty()) {
        std::vector<int> g;
        for (int i = q.top().head; i >= 0; i = next[i]) g.push_back(i);
        std::sort(g.begin(), g.end());
        groups.push_back(g);
        q.pop();
    }
    std::sort(groups.begin(), groups.end(), [](const std::vector<int>& a, const std::vector<int>& b) { return a[0] < b[0]; });
    for (size_t gi = 0; gi < groups.size(); ++gi) {
        const int64_t g = (int64_t)groups[gi].size();
        for (int64_t j = 0; j < g; ++j) {
            const int inst = groups[gi][j];
            group_of_instance[inst] = (int32_t)gi;
            kept_first[inst] = (int32_t)(j * num_layers / g);
            kept_end[inst] = (int32_t)((j + 1) * num_layers / g);
            dropped_bytes[inst] = (int64_t)(num_layers - (kept_end[inst] - kept_first[inst])) * layer_bytes;
        }
    }
    *n_merges = merges;
    *freed_bytes = freed;
    *demand_met = freed >= demand_bytes;
    return KUN_OK;
}

}  // extern "C"
