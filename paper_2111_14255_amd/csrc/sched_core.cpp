// Host-only scheduling layer: T(G, rho), launch order, schedule search.
// Paper: Sec. III-B (Eqs. 3-6), Sec. III-C (Eq. 8, Alg. 1), Sec. III-D (BFS issue).
#include "internal.h"

#include <algorithm>
#include <cmath>
#include <cstring>

namespace mt {

thread_local std::string g_last_error;

int32_t fail(int32_t code, const std::string &msg) {
    g_last_error = msg;
    return code;
}

// A row of pointers is valid when it is non-decreasing and stays inside [0, len].
int32_t validate_pointers(int32_t n_tenants, const int32_t *lens, int32_t n_stages, const int32_t *pointers) {
    if (n_tenants < 1 || n_tenants > MT_MAX_TENANTS) return fail(MT_ERR_INVALID_SCHEDULE, "tenant count out of range");
    if (n_stages < 1 || n_stages > MT_MAX_STAGES) return fail(MT_ERR_INVALID_SCHEDULE, "stage count out of range");
    const int P = n_stages - 1;
    if (P > 0 && !pointers) return fail(MT_ERR_INVALID_ARG, "pointers is NULL");
    for (int i = 0; i < n_tenants; ++i) {
        int prev = 0;
        for (int j = 0; j < P; ++j) {
            int v = pointers[i * P + j];
            if (v < prev) return fail(MT_ERR_INVALID_SCHEDULE, "pointer row " + std::to_string(i) + " is not non-decreasing");
            if (v > lens[i]) return fail(MT_ERR_INVALID_SCHEDULE, "pointer beyond the end of sequence " + std::to_string(i));
            prev = v;
        }
    }
    return MT_OK;
}

// Stage s of tenant i launches operators [rho[i][s-1], rho[i][s]) with rho[i][-1] = 0 and rho[i][P] = len_i.
void expand_pointers(int32_t n_tenants, const int32_t *lens, int32_t n_stages, const int32_t *pointers,
                     int32_t *slices) {
    const int P = n_stages - 1;
    for (int s = 0; s < n_stages; ++s)
        for (int i = 0; i < n_tenants; ++i) {
            int b = s == 0 ? 0 : pointers[i * P + s - 1];
            int e = s == P ? lens[i] : pointers[i * P + s];
            slices[(s * n_tenants + i) * 2 + 0] = b;
            slices[(s * n_tenants + i) * 2 + 1] = e;
        }
}

// Which stream each tenant with work is issued on.  With at least as many streams as such tenants every tenant keeps
// its own stream (Sec. III-B, Eq. 2).  With fewer, the streams in use are those of tenant indices 0 .. c - 1 and the
// tenants are dealt to them longest first: in descending order of the operator count of their slice (ties: lower
// tenant index first) each goes to the stream that holds the fewest operators so far (ties: lowest stream).
void stream_map(int32_t n_tenants, const int32_t *slices, int32_t concurrency, int32_t *host_stream) {
    std::vector<int> active;
    for (int i = 0; i < n_tenants; ++i) {
        host_stream[i] = -1;
        if (slices[2 * i + 1] > slices[2 * i]) active.push_back(i);
    }
    if (active.empty()) return;
    const int c = std::max(1, concurrency);
    if (c >= (int)active.size()) {
        for (int t : active) host_stream[t] = t;
        return;
    }
    auto ops = [&](int t) { return slices[2 * t + 1] - slices[2 * t]; };
    std::stable_sort(active.begin(), active.end(), [&](int a, int b) { return ops(a) > ops(b); });
    std::vector<int64_t> load(c, 0);
    for (int t : active) {
        int best = 0;
        for (int k = 1; k < c; ++k)
            if (load[k] < load[best]) best = k;
        host_stream[t] = best;
        load[best] += ops(t);
    }
}

std::vector<IssueItem> issue_order(int32_t n_tenants, const int32_t *slices, int32_t concurrency, int32_t order) {
    int32_t hs[MT_MAX_TENANTS];
    stream_map(n_tenants, slices, concurrency, hs);
    std::vector<std::vector<IssueItem>> queue(n_tenants);
    for (int t = 0; t < n_tenants; ++t) {
        if (hs[t] < 0) continue;
        for (int i = slices[2 * t]; i < slices[2 * t + 1]; ++i) queue[hs[t]].push_back({hs[t], t, i});
    }
    std::vector<IssueItem> out;
    if (order == MT_ISSUE_DFS) {
        for (auto &q : queue) out.insert(out.end(), q.begin(), q.end());
        return out;
    }
    for (size_t depth = 0;; ++depth) {
        bool any = false;
        for (auto &q : queue)
            if (depth < q.size()) {
                out.push_back(q[depth]);
                any = true;
            }
        if (!any) break;
    }
    return out;
}

// splitmix64 finaliser, chained over the counter words.
static inline uint64_t mix64(uint64_t z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

uint64_t counter_draw(uint64_t seed, uint64_t a, uint64_t b, uint64_t c, uint64_t d) {
    uint64_t h = mix64(seed);
    h = mix64(h ^ a);
    h = mix64(h ^ b);
    h = mix64(h ^ c);
    h = mix64(h ^ d);
    return h;
}

static void even_split(int n_tenants, const int32_t *lens, int P, int32_t *rho) {
    for (int i = 0; i < n_tenants; ++i)
        for (int j = 0; j < P; ++j) rho[i * P + j] = (int32_t)(((int64_t)lens[i] * (j + 1) + P) / (P + 1));
}

struct Recorder {
    int32_t *rec_pointers;
    double *rec_cost;
    int32_t cap, n, width;
    std::vector<int32_t> best;
    double best_cost;
    bool have;
    void add(const int32_t *rho, double c) {
        if (rec_pointers && rec_cost && n < cap) {
            std::memcpy(rec_pointers + (size_t)n * width, rho, sizeof(int32_t) * width);
            rec_cost[n] = c;
        }
        ++n;
        if (!have || c < best_cost) {   // strict: the earliest minimum wins
            best.assign(rho, rho + width);
            best_cost = c;
            have = true;
        }
    }
};

int32_t search_pointers(int32_t n_tenants, const int32_t *lens, const mt_search_opts *o, mt_cost_fn cost, void *user,
                        int32_t *best_pointers, double *best_cost, int32_t *rec_pointers, double *rec_cost,
                        int32_t max_records, int32_t *n_records) {
    if (!lens || !o || !cost || !best_pointers) return fail(MT_ERR_INVALID_ARG, "NULL argument");
    if (n_tenants < 1 || n_tenants > MT_MAX_TENANTS) return fail(MT_ERR_INVALID_ARG, "tenant count out of range");
    if (o->n_stages < 1 || o->n_stages > MT_MAX_STAGES) return fail(MT_ERR_INVALID_ARG, "stage count out of range");
    if (o->rounds < 1 || o->candidates < 1) return fail(MT_ERR_INVALID_ARG, "rounds and candidates must be >= 1");
    for (int i = 0; i < n_tenants; ++i)
        if (lens[i] < 0) return fail(MT_ERR_INVALID_ARG, "negative sequence length");
    const int P = o->n_stages - 1;
    const int width = std::max(1, n_tenants * P);
    Recorder rec{rec_pointers, rec_cost, max_records, 0, n_tenants * P, {}, 0.0, false};
    std::vector<int32_t> rho(width, 0), cand(width, 0), row(std::max(1, P));

    if (o->seed_baselines && P > 0) {
        for (int i = 0; i < n_tenants; ++i)
            for (int j = 0; j < P; ++j) cand[i * P + j] = lens[i];     // everything in stage 1
        rec.add(cand.data(), cost(cand.data(), user));
        even_split(n_tenants, lens, P, cand.data());
        rec.add(cand.data(), cost(cand.data(), user));
    }
    if (o->algo == MT_SEARCH_COORDINATE) {
        even_split(n_tenants, lens, P, rho.data());
        for (int r = 0; r < o->rounds; ++r)
            for (int i = 0; i < n_tenants; ++i) {
                std::vector<int32_t> best_row(std::max(1, P));
                double best_lat = 0;
                for (int m = 0; m < o->candidates; ++m) {
                    for (int j = 0; j < P; ++j)
                        row[j] = (int32_t)(counter_draw(o->seed, r, i, m, j) % (uint64_t)(lens[i] + 1));
                    std::sort(row.begin(), row.begin() + P);
                    cand = rho;
                    for (int j = 0; j < P; ++j) cand[i * P + j] = row[j];
                    double lat = cost(cand.data(), user);
                    rec.add(cand.data(), lat);
                    if (m == 0 || lat < best_lat) {
                        best_lat = lat;
                        best_row = row;
                    }
                }
                for (int j = 0; j < P; ++j) rho[i * P + j] = best_row[j];   // argmin over this row's candidates
            }
    } else if (o->algo == MT_SEARCH_RANDOM) {
        const int64_t evals = (int64_t)o->rounds * n_tenants * o->candidates;
        for (int64_t e = 0; e < evals; ++e) {
            bool feasible = true;
            for (int i = 0; i < n_tenants && feasible; ++i) {
                int prev = 0;
                for (int j = 0; j < P; ++j) {
                    int v = (int)(counter_draw(o->seed, (uint64_t)e, i, 0x52, j) % (uint64_t)(lens[i] + 1));
                    cand[i * P + j] = v;
                    if (v < prev) feasible = false;   // infeasible matrices are filtered out
                    prev = v;
                }
            }
            if (!feasible) continue;
            rec.add(cand.data(), cost(cand.data(), user));
        }
    } else {
        return fail(MT_ERR_INVALID_ARG, "unknown search algorithm");
    }
    if (n_records) *n_records = rec.n;
    if (!rec.have) return fail(MT_ERR_INVALID_SCHEDULE, "search evaluated no feasible schedule");
    if (n_tenants * P > 0) std::memcpy(best_pointers, rec.best.data(), sizeof(int32_t) * n_tenants * P);   // one stage: nothing to copy
    if (best_cost) *best_cost = rec.best_cost;
    return MT_OK;
}

// Play-off over the record memory (an addition to Alg. 1, whose last step returns the best record as profiled once).
// Candidates: the top_k distinct matrices by (profiled cost, position in the record memory), then the matrix with every
// operator in stage 1 unless it is one of them.  Each is measured again with `cost` (which the caller makes a longer
// measurement); the lowest wins, the earlier candidate on ties.
int32_t playoff_pointers(int32_t n_tenants, const int32_t *lens, int32_t n_stages, const int32_t *rec_pointers,
                         const double *rec_cost, int32_t n_records, int32_t top_k, mt_cost_fn cost, void *user,
                         int32_t *best_pointers, double *best_cost, int32_t *n_evaluated) {
    if (!lens || !cost || !best_pointers || !best_cost) return fail(MT_ERR_INVALID_ARG, "NULL argument");
    if (n_tenants < 1 || n_tenants > MT_MAX_TENANTS) return fail(MT_ERR_INVALID_ARG, "tenant count out of range");
    if (n_stages < 1 || n_stages > MT_MAX_STAGES) return fail(MT_ERR_INVALID_ARG, "stage count out of range");
    if (n_records < 0 || (n_records > 0 && (!rec_pointers || !rec_cost))) return fail(MT_ERR_INVALID_ARG, "bad record memory");
    const int P = n_stages - 1;
    const int width = n_tenants * P;
    std::vector<int32_t> order(n_records);
    for (int j = 0; j < n_records; ++j) order[j] = j;
    std::stable_sort(order.begin(), order.end(), [&](int32_t x, int32_t y) { return rec_cost[x] < rec_cost[y]; });
    std::vector<std::vector<int32_t>> cands;
    auto known = [&](const std::vector<int32_t> &m) { return std::find(cands.begin(), cands.end(), m) != cands.end(); };
    for (int32_t j : order) {
        std::vector<int32_t> m(rec_pointers + (size_t)j * width, rec_pointers + (size_t)(j + 1) * width);
        if (!known(m)) cands.push_back(std::move(m));
        if ((int)cands.size() >= std::max(1, top_k)) break;
    }
    std::vector<int32_t> one(width);
    for (int i = 0; i < n_tenants; ++i)
        for (int j = 0; j < P; ++j) one[i * P + j] = lens[i];
    if (!known(one)) cands.push_back(one);
    int best = -1;
    double best_c = 0;
    for (size_t c = 0; c < cands.size(); ++c) {
        const double v = cost(cands[c].data(), user);
        if (best < 0 || v < best_c) { best = (int)c; best_c = v; }     // strict: the earlier candidate wins a tie
    }
    if (width > 0) std::memcpy(best_pointers, cands[best].data(), sizeof(int32_t) * width);
    *best_cost = best_c;
    if (n_evaluated) *n_evaluated = (int32_t)cands.size();
    return MT_OK;
}

int32_t proportional_cu_share(int32_t n_tenants, int32_t cu_count, const double *weight, int32_t *share) {
    if (!weight || !share) return fail(MT_ERR_INVALID_ARG, "NULL argument");
    if (n_tenants < 1 || n_tenants > MT_MAX_TENANTS || cu_count < 8)
        return fail(MT_ERR_INVALID_ARG, "bad tenant count or CU count");
    double total = 0;
    for (int i = 0; i < n_tenants; ++i) {
        if (!(weight[i] >= 0)) return fail(MT_ERR_INVALID_ARG, "weights must be non-negative");
        total += weight[i];
    }
    const int unit = cu_count / 8;
    std::vector<int32_t> units(n_tenants, 1);            // every tenant owns at least one eighth
    const int spare = 8 - n_tenants;
    if (spare > 0 && total > 0) {
        std::vector<double> frac(n_tenants);
        int given = 0;
        for (int i = 0; i < n_tenants; ++i) {
            const double quota = (double)spare * weight[i] / total;
            const int whole = (int)std::floor(quota);
            units[i] += whole;
            given += whole;
            frac[i] = quota - (double)whole;
        }
        for (; given < spare; ++given) {                 // largest remainder first, lower index on ties
            int pick = 0;
            for (int i = 1; i < n_tenants; ++i)
                if (frac[i] > frac[pick]) pick = i;
            units[pick] += 1;
            frac[pick] = -1.0;
        }
    } else if (spare > 0) {
        for (int k = 0; k < spare; ++k) units[k % n_tenants] += 1;
    }
    for (int i = 0; i < n_tenants; ++i) share[i] = units[i] * unit;
    return MT_OK;
}

int32_t search_cu_share(int32_t n_tenants, int32_t cu_count, int32_t rounds, mt_share_cost_fn cost, void *user,
                        int32_t *best_share, double *best_cost) {
    if (!cost || !best_share || !best_cost) return fail(MT_ERR_INVALID_ARG, "NULL argument");
    if (n_tenants < 1 || n_tenants > MT_MAX_TENANTS || cu_count < 8 || rounds < 1)
        return fail(MT_ERR_INVALID_ARG, "bad tenant count, CU count or rounds");
    std::vector<int32_t> cur(best_share, best_share + n_tenants), cand(n_tenants, 0);
    for (int i = 0; i < n_tenants; ++i)
        if (cur[i] < 0 || cur[i] > cu_count) return fail(MT_ERR_INVALID_ARG, "start share out of range");
    double best = *best_cost;
    for (int r = 0; r < rounds; ++r)
        for (int i = 0; i < n_tenants; ++i)
            for (int k = 1; k <= 7; ++k) {
                cand = cur;
                cand[i] = k * cu_count / 8;
                if (cand[i] == cur[i]) continue;
                const double c = cost(cand.data(), user);
                if (c < best) {
                    best = c;
                    cur = cand;
                }
            }
    std::memcpy(best_share, cur.data(), sizeof(int32_t) * n_tenants);
    *best_cost = best;
    return MT_OK;
}

int32_t search_wave_priority(int32_t n_tenants, int32_t rounds, mt_share_cost_fn cost, void *user, int32_t *best_prio,
                             double *best_cost) {
    if (!cost || !best_prio || !best_cost) return fail(MT_ERR_INVALID_ARG, "NULL argument");
    if (n_tenants < 1 || n_tenants > MT_MAX_TENANTS || rounds < 1) return fail(MT_ERR_INVALID_ARG, "bad tenant count or rounds");
    std::vector<int32_t> cur(best_prio, best_prio + n_tenants), cand(n_tenants, 0);
    for (int i = 0; i < n_tenants; ++i)
        if (cur[i] < -1 || cur[i] > 3) return fail(MT_ERR_INVALID_ARG, "start priority out of range");
    double best = *best_cost;
    for (int r = 0; r < rounds; ++r) {
        bool changed = false;
        for (int i = 0; i < n_tenants; ++i)
            for (int v = -1; v <= 3; ++v) {
                cand = cur;
                cand[i] = v;
                if (v == cur[i]) continue;
                const double c = cost(cand.data(), user);
                if (c < best) {
                    best = c;
                    cur = cand;
                    changed = true;
                }
            }
        if (!changed) break;
    }
    std::memcpy(best_prio, cur.data(), sizeof(int32_t) * n_tenants);
    *best_cost = best;
    return MT_OK;
}

}  // namespace mt

extern "C" {

int32_t mt_search_wave_priority(int32_t n_tenants, int32_t rounds, mt_share_cost_fn prio_cost, void *user, int32_t *best_prio,
                                double *best_cost) {
    return mt::search_wave_priority(n_tenants, rounds, prio_cost, user, best_prio, best_cost);
}

int32_t mt_proportional_cu_share(int32_t n_tenants, int32_t cu_count, const double *weight, int32_t *share) {
    return mt::proportional_cu_share(n_tenants, cu_count, weight, share);
}

int32_t mt_search_cu_share(int32_t n_tenants, int32_t cu_count, int32_t rounds, mt_share_cost_fn share_cost, void *user,
                           int32_t *best_share, double *best_cost) {
    return mt::search_cu_share(n_tenants, cu_count, rounds, share_cost, user, best_share, best_cost);
}

const char *mt_last_error(void) { return mt::g_last_error.c_str(); }

int32_t mt_expand_pointers(int32_t n_tenants, const int32_t *lens, int32_t n_stages, const int32_t *pointers,
                           int32_t *slices_out) {
    if (!lens || !slices_out) return mt::fail(MT_ERR_INVALID_ARG, "NULL argument");
    int32_t rc = mt::validate_pointers(n_tenants, lens, n_stages, pointers);
    if (rc != MT_OK) return rc;
    mt::expand_pointers(n_tenants, lens, n_stages, pointers, slices_out);
    return MT_OK;
}

int32_t mt_issue_order_of_stage(int32_t n_tenants, const int32_t *slices, int32_t concurrency, int32_t order,
                                int32_t *order_out, int32_t *n_out) {
    if (!slices || !order_out || !n_out) return mt::fail(MT_ERR_INVALID_ARG, "NULL argument");
    if (n_tenants < 1 || n_tenants > MT_MAX_TENANTS) return mt::fail(MT_ERR_INVALID_ARG, "tenant count out of range");
    if (concurrency < 1) return mt::fail(MT_ERR_INVALID_SCHEDULE, "concurrency must be >= 1");
    if (order != MT_ISSUE_BFS && order != MT_ISSUE_DFS) return mt::fail(MT_ERR_INVALID_ARG, "unknown issue order");
    for (int i = 0; i < n_tenants; ++i)
        if (slices[2 * i] < 0 || slices[2 * i + 1] < slices[2 * i]) return mt::fail(MT_ERR_INVALID_ARG, "bad slice");
    auto v = mt::issue_order(n_tenants, slices, concurrency, order);
    for (size_t k = 0; k < v.size(); ++k) {
        order_out[3 * k + 0] = v[k].stream;
        order_out[3 * k + 1] = v[k].tenant;
        order_out[3 * k + 2] = v[k].op;
    }
    *n_out = (int32_t)v.size();
    return MT_OK;
}

int32_t mt_playoff_pointers(int32_t n_tenants, const int32_t *lens, int32_t n_stages, const int32_t *rec_pointers,
                            const double *rec_cost, int32_t n_records, int32_t top_k, mt_cost_fn cost, void *user,
                            int32_t *best_pointers, double *best_cost, int32_t *n_evaluated) {
    return mt::playoff_pointers(n_tenants, lens, n_stages, rec_pointers, rec_cost, n_records, top_k, cost, user,
                                best_pointers, best_cost, n_evaluated);
}

int32_t mt_search_pointers(int32_t n_tenants, const int32_t *lens, const mt_search_opts *opts, mt_cost_fn cost,
                           void *user, int32_t *best_pointers, double *best_cost, int32_t *rec_pointers,
                           double *rec_cost, int32_t max_records, int32_t *n_records) {
    return mt::search_pointers(n_tenants, lens, opts, cost, user, best_pointers, best_cost, rec_pointers, rec_cost,
                               max_records, n_records);
}

}  // extern "C"
