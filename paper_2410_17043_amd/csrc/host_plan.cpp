// Host-side planners: transmission order of one all-to-all (Sec. 4.2, 5.2,
// Appendix A/B) and expert colocation by bottleneck matching (Sec. 6.2).
// Plain C++; nothing here touches the GPU.  Planning is offline (Sec. 2.4), its
// results are inputs of moe_dispatch.
#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>
#include <queue>
#include <vector>

#include "common.h"

namespace {

using Mat = std::vector<std::vector<double>>;

int check_traffic(const char* who, int32_t n, const int64_t* D, const double* B) {
    if (!D) return moe_set_error(MOE_EINVAL, "%s: D is NULL", who);
    if (n < 1 || n > MOE_MAX_G) return moe_set_error(MOE_ESHAPE, "%s: n must be in 1..%d", who, MOE_MAX_G);
    for (int64_t i = 0; i < (int64_t)n * n; ++i)
        if (D[i] < 0) return moe_set_error(MOE_EINVAL, "%s: negative traffic entry", who);
    if (B)
        for (int i = 0; i < n; ++i)
            if (!(B[i] > 0.0) || !std::isfinite(B[i])) return moe_set_error(MOE_EINVAL, "%s: link rates must be positive", who);
    return MOE_OK;
}

// p_ij = d_ij / min(B_i, B_j) off the diagonal (Appendix B; B = 1 is Sec. 4.2).
Mat scaled(int n, const int64_t* D, const double* B) {
    Mat P(n, std::vector<double>(n, 0.0));
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < n; ++j)
            if (i != j) P[i][j] = (double)D[i * n + j] / (B ? std::min(B[i], B[j]) : 1.0);
    return P;
}

double max_line_sum(const Mat& P) {
    const int n = (int)P.size();
    double m = 0.0;
    for (int i = 0; i < n; ++i) {
        double r = 0.0, c = 0.0;
        for (int j = 0; j < n; ++j) { r += P[i][j]; c += P[j][i]; }
        m = std::max(m, std::max(r, c));
    }
    return m;
}

// Kuhn's augmenting paths on a boolean support; returns the number of matched senders.
struct Matcher {
    int n;
    const std::vector<std::vector<char>>& adj;
    std::vector<int> match_recv;
    std::vector<char> seen;
    Matcher(int n_, const std::vector<std::vector<char>>& a) : n(n_), adj(a), match_recv(n_, -1), seen(n_, 0) {}
    bool augment(int i) {
        for (int j = 0; j < n; ++j) {
            if (adj[i][j] && !seen[j]) {
                seen[j] = 1;
                if (match_recv[j] < 0 || augment(match_recv[j])) { match_recv[j] = i; return true; }
            }
        }
        return false;
    }
    int run() {
        int m = 0;
        for (int i = 0; i < n; ++i) {
            std::fill(seen.begin(), seen.end(), 0);
            if (augment(i)) ++m;
        }
        return m;
    }
};

struct Round { std::vector<int32_t> dst; double tau; };

// Appendix A: pad P to equal row/column sums, peel permutations, strip the padding.
std::vector<Round> plan_rounds(const Mat& P, double bm) {
    const int n = (int)P.size();
    std::vector<Round> out;
    if (bm <= 0.0) return out;
    const double eps = bm * 1e-12;
    Mat Dp = P, left = P;
    {   // step 1: artificial traffic X >= 0, deficits matched from the top-left corner
        std::vector<double> r(n), c(n);
        for (int i = 0; i < n; ++i) {
            double rs = 0.0, cs = 0.0;
            for (int j = 0; j < n; ++j) { rs += P[i][j]; cs += P[j][i]; }
            r[i] = std::max(0.0, bm - rs);
            c[i] = std::max(0.0, bm - cs);
        }
        int i = 0, j = 0;
        while (i < n && j < n) {
            const double q = std::min(r[i], c[j]);
            Dp[i][j] += q;
            r[i] -= q;
            c[j] -= q;
            if (r[i] <= eps) ++i; else ++j;
        }
    }
    std::vector<std::vector<char>> adj(n, std::vector<char>(n));
    auto emit = [&](const std::vector<int>& match_recv, bool padded) {
        std::vector<int> sigma(n, -1);
        for (int j = 0; j < n; ++j)
            if (match_recv[j] >= 0) sigma[match_recv[j]] = j;
        double tau = -1.0;
        for (int i = 0; i < n; ++i)
            if (sigma[i] >= 0) {
                const double v = padded ? Dp[i][sigma[i]] : left[i][sigma[i]];
                tau = (tau < 0.0) ? v : std::min(tau, v);
            }
        Round rd;
        rd.tau = tau;
        rd.dst.assign(n, -1);
        for (int i = 0; i < n; ++i) {
            const int j = sigma[i];
            if (j < 0) continue;
            if (padded) { Dp[i][j] -= tau; if (Dp[i][j] <= eps) Dp[i][j] = 0.0; }
            const double use = std::min(left[i][j], tau);
            if (use > eps) rd.dst[i] = j;
            left[i][j] -= use;
            if (left[i][j] <= eps) left[i][j] = 0.0;
        }
        out.push_back(rd);
    };
    // step 2: every slot is a full permutation while the padded matrix is not empty
    for (int it = 0; it < n * n + 8; ++it) {
        bool any = false;
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < n; ++j) { adj[i][j] = Dp[i][j] > eps; any |= (bool)adj[i][j]; }
        if (!any) break;
        Matcher m(n, adj);
        if (m.run() < n) break;                   // only possible through rounding residue
        emit(m.match_recv, true);
    }
    // rounding residue of heterogeneous rates: deliver whatever real traffic is left
    for (int it = 0; it < n * n + 8; ++it) {
        bool any = false;
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < n; ++j) { adj[i][j] = left[i][j] > eps; any |= (bool)adj[i][j]; }
        if (!any) break;
        Matcher m(n, adj);
        m.run();
        emit(m.match_recv, false);
    }
    return out;
}

using Timeline = std::vector<std::pair<double, double>>;   // sorted busy intervals

double earliest_fit(const Timeline& busy, double t, double p) {
    for (const auto& iv : busy) {
        if (t + p <= iv.first) break;
        if (iv.second > t) t = iv.second;
    }
    return t;
}

// Algorithm 1, greedy reading: bottleneck GPU first, then GPUs by remaining row
// sum; each flow goes into the earliest gap free on the sender's and the
// receiver's timeline.
void plan_order(const Mat& P, std::vector<int32_t>& dest_order, std::vector<double>& start, double* makespan) {
    const int n = (int)P.size();
    Mat rem = P;
    std::vector<Timeline> sb(n), rb(n);
    start.assign((size_t)n * n, -1.0);
    std::vector<double> rows(n, 0.0), cols(n, 0.0);
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < n; ++j) { rows[i] += P[i][j]; cols[j] += P[i][j]; }
    auto earliest = [&](int i, int j) {
        double t = 0.0;
        const double p = rem[i][j];
        for (;;) {
            const double t1 = earliest_fit(sb[i], t, p);
            const double t2 = earliest_fit(rb[j], t1, p);
            if (t2 == t1) return t1;
            t = t2;
        }
    };
    double end = 0.0;
    auto place = [&](int i, int j, double t0) {
        const double p = rem[i][j];
        start[(size_t)i * n + j] = t0;
        sb[i].emplace_back(t0, t0 + p);
        std::sort(sb[i].begin(), sb[i].end());
        rb[j].emplace_back(t0, t0 + p);
        std::sort(rb[j].begin(), rb[j].end());
        rem[i][j] = 0.0;
        end = std::max(end, t0 + p);
    };
    int b = 0;
    for (int i = 1; i < n; ++i)
        if (std::max(rows[i], cols[i]) > std::max(rows[b], cols[b])) b = i;
    double t = 0.0;
    for (int peer = 0; peer < n; ++peer) {
        const int i = rows[b] >= cols[b] ? b : peer, j = rows[b] >= cols[b] ? peer : b;
        if (rem[i][j] > 0.0) { const double p = rem[i][j]; place(i, j, t); t += p; }
    }
    auto row_left = [&](int i) { double s = 0.0; for (int j = 0; j < n; ++j) s += rem[i][j]; return s; };
    for (;;) {
        std::vector<int> by(n);
        std::vector<double> rl(n);
        bool any = false;
        for (int i = 0; i < n; ++i) { by[i] = i; rl[i] = row_left(i); any |= rl[i] > 0.0; }
        if (!any) break;
        std::stable_sort(by.begin(), by.end(), [&](int a, int c) { return rl[a] > rl[c]; });
        for (int i : by) {
            for (;;) {
                int bj = -1;
                double bt = 0.0;
                for (int j = 0; j < n; ++j) {
                    if (!(rem[i][j] > 0.0)) continue;
                    const double tj = earliest(i, j);
                    const bool better = bj < 0 || tj < bt || (tj == bt && (cols[j] > cols[bj] || (cols[j] == cols[bj] && rem[i][j] > rem[i][bj])));
                    if (better) { bj = j; bt = tj; }
                }
                if (bj < 0) break;
                place(i, bj, bt);
            }
        }
    }
    dest_order.assign((size_t)n * n, 0);
    for (int i = 0; i < n; ++i) {
        std::vector<int> real, empty;
        for (int j = 0; j < n; ++j) {
            if (start[(size_t)i * n + j] >= 0.0) real.push_back(j);
            else if (j != i) empty.push_back(j);
        }
        std::stable_sort(real.begin(), real.end(), [&](int a, int c) { return start[(size_t)i * n + a] < start[(size_t)i * n + c]; });
        int p = 0;
        for (int j : real) dest_order[(size_t)i * n + p++] = j;
        for (int j : empty) dest_order[(size_t)i * n + p++] = j;
        dest_order[(size_t)i * n + p] = i;
    }
    *makespan = end;
}

// Completion time when GPU i sends to order[i*n ..] one destination after another on the big switch of
// Sec. 2.4: a receiver with m incoming flows gives each B_recv / m, a flow runs at min(B_send, share).
double simulate_order(int n, const int64_t* D, const double* B, const int32_t* order) {
    std::vector<int> pos(n, 0), cur(n, -1), fan(n);
    std::vector<double> left(n, 0.0), rate(n, 0.0);
    auto next_flow = [&](int i) {
        cur[i] = -1;
        while (pos[i] < n) {
            const int j = order[i * n + pos[i]++];
            if (j != i && D[i * n + j] > 0) { cur[i] = j; left[i] = (double)D[i * n + j]; break; }
        }
    };
    for (int i = 0; i < n; ++i) next_flow(i);
    double t = 0.0;
    for (;;) {
        std::fill(fan.begin(), fan.end(), 0);
        bool any = false;
        for (int i = 0; i < n; ++i)
            if (cur[i] >= 0) { ++fan[cur[i]]; any = true; }
        if (!any) break;
        double dt = -1.0;
        for (int i = 0; i < n; ++i) {
            if (cur[i] < 0) continue;
            const double bs = B ? B[i] : 1.0, br = B ? B[cur[i]] : 1.0;
            rate[i] = std::min(bs, br / fan[cur[i]]);
            const double need = left[i] / rate[i];
            dt = (dt < 0.0) ? need : std::min(dt, need);
        }
        t += dt;
        for (int i = 0; i < n; ++i) {
            if (cur[i] < 0) continue;
            left[i] -= rate[i] * dt;
            if (left[i] <= 1e-9 * (double)D[i * n + cur[i]]) next_flow(i);
        }
    }
    return t;
}

// Row i of a whole-flow order: the given non-empty flows, then the empty destinations, then i itself.
void fill_order_row(int n, int i, const std::vector<int>& real, int32_t* row) {
    std::vector<char> used(n, 0);
    int p = 0;
    for (int j : real) { row[p++] = j; used[j] = 1; }
    for (int j = 0; j < n; ++j)
        if (j != i && !used[j]) row[p++] = j;
    row[p] = i;
}

// Whole-flow order read off the rounds of Appendix A: destinations in the order of their first round.
void order_from_rounds(int n, const std::vector<Round>& rounds, std::vector<int32_t>& order) {
    order.assign((size_t)n * n, 0);
    for (int i = 0; i < n; ++i) {
        std::vector<int> real;
        std::vector<char> seen(n, 0);
        for (const Round& rd : rounds) {
            const int j = rd.dst[i];
            if (j >= 0 && !seen[j]) { seen[j] = 1; real.push_back(j); }
        }
        fill_order_row(n, i, real, &order[(size_t)i * n]);
    }
}

// Whole-flow order built while the transfer is played forward under the sharing rule of simulate_order:
// a GPU with nothing in flight starts the flow whose receiver has the fewest incoming flows at that moment
// (a free port if there is one: no contention at the receiving side, Theorem 2), then the largest flow, then
// the lowest destination; GPUs deciding at the same instant go by descending traffic left to send.
void order_by_list(int n, const int64_t* D, const double* B, std::vector<int32_t>& order) {
    std::vector<std::vector<int64_t>> todo(n, std::vector<int64_t>(n, 0));
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < n; ++j)
            if (i != j) todo[i][j] = D[i * n + j];
    std::vector<std::vector<int>> seq(n);
    std::vector<int> cur(n, -1), fan(n), idle;
    std::vector<double> left(n, 0.0), rate(n, 0.0), to_send(n);
    for (;;) {
        idle.clear();
        for (int i = 0; i < n; ++i) {
            int64_t s = 0;
            for (int j = 0; j < n; ++j) s += todo[i][j];
            to_send[i] = (double)s / (B ? B[i] : 1.0);
            if (cur[i] < 0 && s > 0) idle.push_back(i);
        }
        std::stable_sort(idle.begin(), idle.end(), [&](int a, int c) { return to_send[a] > to_send[c]; });
        for (int i : idle) {
            std::fill(fan.begin(), fan.end(), 0);
            for (int s = 0; s < n; ++s)
                if (cur[s] >= 0) ++fan[cur[s]];
            int bj = -1;
            for (int j = 0; j < n; ++j) {
                if (todo[i][j] <= 0) continue;
                if (bj < 0 || fan[j] < fan[bj] || (fan[j] == fan[bj] && todo[i][j] > todo[i][bj])) bj = j;
            }
            cur[i] = bj;
            left[i] = (double)todo[i][bj];
            todo[i][bj] = 0;
            seq[i].push_back(bj);
        }
        std::fill(fan.begin(), fan.end(), 0);
        bool any = false;
        for (int i = 0; i < n; ++i)
            if (cur[i] >= 0) { ++fan[cur[i]]; any = true; }
        if (!any) break;
        double dt = -1.0;
        for (int i = 0; i < n; ++i) {
            if (cur[i] < 0) continue;
            rate[i] = std::min(B ? B[i] : 1.0, (B ? B[cur[i]] : 1.0) / fan[cur[i]]);
            const double need = left[i] / rate[i];
            dt = (dt < 0.0) ? need : std::min(dt, need);
        }
        for (int i = 0; i < n; ++i) {
            if (cur[i] < 0) continue;
            left[i] -= rate[i] * dt;
            if (left[i] <= 1e-9 * (double)D[i * n + cur[i]]) cur[i] = -1;
        }
    }
    order.assign((size_t)n * n, 0);
    for (int i = 0; i < n; ++i) fill_order_row(n, i, seq[i], &order[(size_t)i * n]);
}

constexpr double kImproveMargin = 1e-9;      // an exchange must gain more than this fraction of the time

// Hill climbing: two neighbouring non-empty flows of a GPU are exchanged and the exchange is kept when the
// simulated completion time drops by more than kImproveMargin of its value; at most 64 n exchanges are tried.
double improve_order(int n, const int64_t* D, const double* B, std::vector<int32_t>& order) {
    std::vector<int> n_real(n, 0);
    for (int i = 0; i < n; ++i) {
        std::vector<int> real;
        for (int p = 0; p < n; ++p) {
            const int j = order[(size_t)i * n + p];
            if (j != i && D[i * n + j] > 0) real.push_back(j);
        }
        n_real[i] = (int)real.size();
        fill_order_row(n, i, real, &order[(size_t)i * n]);
    }
    double best = simulate_order(n, D, B, order.data());
    int budget = 64 * n;
    bool changed = true;
    while (changed && budget > 0) {
        changed = false;
        for (int i = 0; i < n; ++i)
            for (int p = 0; p + 1 < n_real[i] && budget > 0; ++p) {
                --budget;
                std::swap(order[(size_t)i * n + p], order[(size_t)i * n + p + 1]);
                const double v = simulate_order(n, D, B, order.data());
                if (v < best * (1.0 - kImproveMargin)) { best = v; changed = true; }
                else std::swap(order[(size_t)i * n + p], order[(size_t)i * n + p + 1]);
            }
    }
    return best;
}

// Hopcroft-Karp on the edges of weight <= limit; left side na, right side nb.
struct HopcroftKarp {
    int na, nb;
    const std::vector<int64_t>& W;
    int64_t limit;
    std::vector<int> ml, mr, dist;
    HopcroftKarp(int a, int b, const std::vector<int64_t>& w, int64_t lim)
        : na(a), nb(b), W(w), limit(lim), ml(a, -1), mr(b, -1), dist(a, 0) {}
    bool ok(int i, int j) const { return W[(size_t)i * nb + j] <= limit; }
    bool bfs() {
        std::queue<int> q;
        for (int i = 0; i < na; ++i) {
            if (ml[i] < 0) { dist[i] = 0; q.push(i); } else dist[i] = -1;
        }
        bool found = false;
        while (!q.empty()) {
            const int i = q.front();
            q.pop();
            for (int j = 0; j < nb; ++j) {
                if (!ok(i, j)) continue;
                const int i2 = mr[j];
                if (i2 < 0) found = true;
                else if (dist[i2] < 0) { dist[i2] = dist[i] + 1; q.push(i2); }
            }
        }
        return found;
    }
    bool dfs(int i) {
        for (int j = 0; j < nb; ++j) {
            if (!ok(i, j)) continue;
            const int i2 = mr[j];
            if (i2 < 0 || (dist[i2] == dist[i] + 1 && dfs(i2))) { ml[i] = j; mr[j] = i; return true; }
        }
        dist[i] = -1;
        return false;
    }
    int run() {
        int m = 0;
        while (bfs())
            for (int i = 0; i < na; ++i)
                if (ml[i] < 0 && dfs(i)) ++m;
        return m;
    }
};

}  // namespace

extern "C" void aurora_schedule_free(aurora_schedule* s) {
    if (!s) return;
    free(s->duration);
    free(s->dst);
    free(s->dest_order);
    free(s->alg1_order);
    free(s->start);
    memset(s, 0, sizeof(*s));
}

extern "C" int aurora_order(int32_t n, const int64_t* D, const double* B, aurora_schedule* out) {
    if (!out) return moe_set_error(MOE_EINVAL, "aurora_order: out is NULL");
    memset(out, 0, sizeof(*out));
    int rc = check_traffic("aurora_order", n, D, B);
    if (rc != MOE_OK) return rc;
    try {
        const Mat P = scaled(n, D, B);
        out->n = n;
        out->bmax = max_line_sum(P);
        double pb = 0.0;
        for (int i = 0; i < n; ++i) {
            double r = 0.0, c = 0.0;
            for (int j = 0; j < n; ++j)
                if (i != j) { r += (double)D[i * n + j]; c += (double)D[j * n + i]; }
            pb = std::max(pb, std::max(r, c) / (B ? B[i] : 1.0));
        }
        out->port_bound = pb;
        const std::vector<Round> rounds = plan_rounds(P, out->bmax);
        std::vector<int32_t> order, by_rounds, by_list, by_shift((size_t)n * n);
        std::vector<double> start;
        plan_order(P, order, start, &out->makespan_order);
        // the order for the send buffer: the best of four whole-flow orders when run back to back (an earlier
        // candidate stays unless a later one is better by more than the margin), then adjacent exchanges
        order_from_rounds(n, rounds, by_rounds);
        order_by_list(n, D, B, by_list);
        for (int i = 0; i < n; ++i) {                            // shifted order: in step s GPU i sends to (i + s) mod n
            for (int sft = 1; sft < n; ++sft) by_shift[(size_t)i * n + sft - 1] = (i + sft) % n;
            by_shift[(size_t)i * n + n - 1] = i;
        }
        const std::vector<int32_t>* cand[4] = {&order, &by_rounds, &by_list, &by_shift};
        int pick = 0;
        for (int c = 0; c < 4; ++c) {
            out->candidate_time[c] = simulate_order(n, D, B, cand[c]->data());
            if (c > 0 && out->candidate_time[c] < out->candidate_time[pick] * (1.0 - kImproveMargin)) pick = c;
        }
        std::vector<int32_t> chosen = *cand[pick];
        out->order_source = pick;
        out->order_time = improve_order(n, D, B, chosen);
        out->n_rounds = (int32_t)rounds.size();
        out->duration = (double*)malloc(sizeof(double) * std::max<size_t>(1, rounds.size()));
        out->dst = (int32_t*)malloc(sizeof(int32_t) * std::max<size_t>(1, rounds.size() * n));
        out->dest_order = (int32_t*)malloc(sizeof(int32_t) * (size_t)n * n);
        out->alg1_order = (int32_t*)malloc(sizeof(int32_t) * (size_t)n * n);
        out->start = (double*)malloc(sizeof(double) * (size_t)n * n);
        if (!out->duration || !out->dst || !out->dest_order || !out->alg1_order || !out->start) {
            aurora_schedule_free(out);
            return moe_set_error(MOE_ENOMEM, "aurora_order: host allocation failed");
        }
        double total = 0.0;
        for (size_t r = 0; r < rounds.size(); ++r) {
            out->duration[r] = rounds[r].tau;
            total += rounds[r].tau;
            memcpy(out->dst + r * n, rounds[r].dst.data(), sizeof(int32_t) * n);
        }
        out->makespan_rounds = total;
        memcpy(out->dest_order, chosen.data(), sizeof(int32_t) * (size_t)n * n);
        memcpy(out->alg1_order, order.data(), sizeof(int32_t) * (size_t)n * n);
        memcpy(out->start, start.data(), sizeof(double) * (size_t)n * n);
    } catch (const std::bad_alloc&) {
        aurora_schedule_free(out);
        return moe_set_error(MOE_ENOMEM, "aurora_order: host allocation failed");
    }
    return MOE_OK;
}

extern "C" int aurora_chunks(const aurora_schedule* s, const int64_t* D, const double* B, int32_t g, int32_t* chunk_dest,
                             int32_t* chunk_rows, int32_t* n_chunks) {
    if (!s || !chunk_dest || !chunk_rows || !n_chunks) return moe_set_error(MOE_EINVAL, "aurora_chunks: NULL argument");
    const int n = s->n;
    int rc = check_traffic("aurora_chunks", n, D, B);
    if (rc != MOE_OK) return rc;
    if (g < 0 || g >= n) return moe_set_error(MOE_ESHAPE, "aurora_chunks: g = %d outside [0, %d)", g, n);
    if (!s->dst || !s->duration) return moe_set_error(MOE_EINVAL, "aurora_chunks: schedule holds no rounds");
    // Per destination: scaled real traffic not yet sent, tokens already put into chunks, last chunk.
    double left[MOE_MAX_G], total[MOE_MAX_G], rate[MOE_MAX_G];
    int64_t sent[MOE_MAX_G];
    int last[MOE_MAX_G];
    for (int j = 0; j < n; ++j) {
        rate[j] = B ? std::min(B[g], B[j]) : 1.0;
        total[j] = (j == g) ? 0.0 : (double)D[(size_t)g * n + j] / rate[j];
        left[j] = total[j];
        sent[j] = 0;
        last[j] = -1;
    }
    int nc = 0;
    for (int r = 0; r < s->n_rounds; ++r) {
        const int j = s->dst[(size_t)r * n + g];
        if (j < 0 || j >= n || j == g) continue;
        left[j] -= std::min(left[j], s->duration[r]);        // real traffic first, as in the rounds themselves
        int64_t cum = (int64_t)std::floor((total[j] - left[j]) * rate[j] + 1e-6);
        cum = std::min<int64_t>(cum, D[(size_t)g * n + j]);
        if (cum > sent[j]) {
            chunk_dest[nc] = j;
            chunk_rows[nc] = (int32_t)(cum - sent[j]);
            last[j] = nc++;
            sent[j] = cum;
        }
    }
    for (int j = 0; j < n; ++j) {                            // whatever floating point left over joins the last chunk
        const int64_t miss = (j == g) ? 0 : D[(size_t)g * n + j] - sent[j];
        if (miss > 0) {
            if (last[j] < 0) return moe_set_error(MOE_ESHAPE, "aurora_chunks: the schedule never sends %d -> %d; made from another matrix?", g, j);
            chunk_rows[last[j]] += (int32_t)miss;
        }
    }
    *n_chunks = nc;
    return MOE_OK;
}

extern "C" int aurora_simulate(int32_t n, const int64_t* D, const double* B, const int32_t* order, double* time_out) {
    if (!order || !time_out) return moe_set_error(MOE_EINVAL, "aurora_simulate: NULL argument");
    int rc = check_traffic("aurora_simulate", n, D, B);
    if (rc != MOE_OK) return rc;
    for (int i = 0; i < n; ++i) {
        bool seen[MOE_MAX_G] = {false};
        for (int p = 0; p < n; ++p) {
            const int j = order[i * n + p];
            if (j < 0 || j >= n || seen[j]) return moe_set_error(MOE_ESHAPE, "aurora_simulate: order row %d is not a permutation", i);
            seen[j] = true;
        }
    }
    try {
        *time_out = simulate_order(n, D, B, order);
    } catch (const std::bad_alloc&) {
        return moe_set_error(MOE_ENOMEM, "aurora_simulate: host allocation failed");
    }
    return MOE_OK;
}

extern "C" int colocate_match(int32_t na, int32_t nb, const int64_t* Da, const int64_t* Db, int32_t* pair,
                              double* bottleneck) {
    if (!Da || !Db || !pair || !bottleneck) return moe_set_error(MOE_EINVAL, "colocate_match: NULL argument");
    if (na < 1 || nb < na || nb > MOE_MAX_E) return moe_set_error(MOE_ESHAPE, "colocate_match: need 1 <= na <= nb <= %d", MOE_MAX_E);
    for (int64_t i = 0; i < (int64_t)na * na; ++i)
        if (Da[i] < 0) return moe_set_error(MOE_EINVAL, "colocate_match: negative entry in Da");
    for (int64_t i = 0; i < (int64_t)nb * nb; ++i)
        if (Db[i] < 0) return moe_set_error(MOE_EINVAL, "colocate_match: negative entry in Db");
    try {
        auto sums = [](int n, const int64_t* D, std::vector<int64_t>& send, std::vector<int64_t>& recv) {
            send.assign(n, 0);
            recv.assign(n, 0);
            for (int i = 0; i < n; ++i)
                for (int j = 0; j < n; ++j)
                    if (i != j) { send[i] += D[i * n + j]; recv[j] += D[i * n + j]; }
        };
        std::vector<int64_t> sa, ra, sb, rb;
        sums(na, Da, sa, ra);
        sums(nb, Db, sb, rb);
        std::vector<int64_t> W((size_t)na * nb);
        for (int i = 0; i < na; ++i)
            for (int j = 0; j < nb; ++j) W[(size_t)i * nb + j] = std::max(sa[i] + sb[j], ra[i] + rb[j]);
        std::vector<int64_t> sorted = W;
        std::sort(sorted.begin(), sorted.end());
        sorted.erase(std::unique(sorted.begin(), sorted.end()), sorted.end());
        size_t lo = 0, hi = sorted.size() - 1;       // the largest weight always admits a full matching
        while (lo < hi) {
            const size_t mid = (lo + hi) / 2;
            HopcroftKarp hk(na, nb, W, sorted[mid]);
            if (hk.run() == na) hi = mid; else lo = mid + 1;
        }
        HopcroftKarp hk(na, nb, W, sorted[lo]);
        if (hk.run() != na) return moe_set_error(MOE_EINTERNAL, "colocate_match: no matching at the largest weight");
        for (int i = 0; i < na; ++i) pair[i] = hk.ml[i];
        *bottleneck = (double)sorted[lo];
    } catch (const std::bad_alloc&) {
        return moe_set_error(MOE_ENOMEM, "colocate_match: host allocation failed");
    }
    return MOE_OK;
}

// ---------------------------------------------------------------------------------------------
// Theorem 3 (Sec. 5.1): the expert with the r-th largest load on the GPU with the r-th highest
// performance; ties keep the lower index first on both sides.
extern "C" int aurora_assign(int32_t n, const int64_t* load, const double* perf, int32_t* expert_to_gpu) {
    if (!load || !perf || !expert_to_gpu) return moe_set_error(MOE_EINVAL, "aurora_assign: NULL argument");
    if (n < 1 || n > MOE_MAX_E) return moe_set_error(MOE_ESHAPE, "aurora_assign: need 1 <= n <= %d", MOE_MAX_E);
    for (int i = 0; i < n; ++i) {
        if (load[i] < 0) return moe_set_error(MOE_EINVAL, "aurora_assign: negative load");
        if (!(perf[i] > 0.0) || !std::isfinite(perf[i])) return moe_set_error(MOE_EINVAL, "aurora_assign: performance must be finite and > 0");
    }
    try {
        std::vector<int> experts(n), gpus(n);
        for (int i = 0; i < n; ++i) experts[i] = gpus[i] = i;
        std::stable_sort(experts.begin(), experts.end(), [&](int a, int b) { return load[a] > load[b]; });
        std::stable_sort(gpus.begin(), gpus.end(), [&](int a, int b) { return perf[a] > perf[b]; });
        for (int r = 0; r < n; ++r) expert_to_gpu[experts[r]] = gpus[r];
    } catch (const std::bad_alloc&) {
        return moe_set_error(MOE_ENOMEM, "aurora_assign: host allocation failed");
    }
    return MOE_OK;
}

namespace {

// Perfect matching rows -> columns of an n x n weight table that minimises the largest weight used:
// binary search over the sorted distinct weights (as ranks), Hopcroft-Karp as the feasibility test.
int bottleneck_perfect(int n, const double* W, int32_t* col_of_row, double* value) {
    std::vector<double> vals(W, W + (size_t)n * n);
    std::sort(vals.begin(), vals.end());
    vals.erase(std::unique(vals.begin(), vals.end()), vals.end());
    std::vector<int64_t> rank((size_t)n * n);
    for (size_t i = 0; i < rank.size(); ++i) rank[i] = std::lower_bound(vals.begin(), vals.end(), W[i]) - vals.begin();
    size_t lo = 0, hi = vals.size() - 1;             // every edge allowed: a perfect matching exists
    while (lo < hi) {
        const size_t mid = (lo + hi) / 2;
        HopcroftKarp hk(n, n, rank, (int64_t)mid);
        if (hk.run() == n) hi = mid; else lo = mid + 1;
    }
    HopcroftKarp hk(n, n, rank, (int64_t)lo);
    if (hk.run() != n) return moe_set_error(MOE_EINTERNAL, "bottleneck matching: no perfect matching at the largest weight");
    for (int i = 0; i < n; ++i) col_of_row[i] = hk.ml[i];
    *value = vals[lo];
    return MOE_OK;
}

int check_weights(const char* who, size_t count, const double* W) {
    for (size_t i = 0; i < count; ++i)
        if (!std::isfinite(W[i])) return moe_set_error(MOE_EINVAL, "%s: weight %zu is not finite", who, i);
    return MOE_OK;
}

}  // namespace

extern "C" int aurora_bottleneck_assign(int32_t n, const double* W, int32_t* item_of_gpu, double* bottleneck) {
    if (!W || !item_of_gpu || !bottleneck) return moe_set_error(MOE_EINVAL, "aurora_bottleneck_assign: NULL argument");
    if (n < 1 || n > MOE_MAX_E) return moe_set_error(MOE_ESHAPE, "aurora_bottleneck_assign: need 1 <= n <= %d", MOE_MAX_E);
    int rc = check_weights("aurora_bottleneck_assign", (size_t)n * n, W);
    if (rc != MOE_OK) return rc;
    try {
        return bottleneck_perfect(n, W, item_of_gpu, bottleneck);
    } catch (const std::bad_alloc&) {
        return moe_set_error(MOE_ENOMEM, "aurora_bottleneck_assign: host allocation failed");
    }
}

extern "C" int colocate_hetero_match(int32_t n, const int64_t* Da, const int64_t* Db, const double* time3, int32_t* pair,
                                     int32_t* gpu_of_pair, double* value) {
    if (!Da || !Db || !time3 || !pair || !gpu_of_pair || !value)
        return moe_set_error(MOE_EINVAL, "colocate_hetero_match: NULL argument");
    if (n < 1 || n > MOE_MAX_G) return moe_set_error(MOE_ESHAPE, "colocate_hetero_match: need 1 <= n <= %d", MOE_MAX_G);
    int rc = check_weights("colocate_hetero_match", (size_t)n * n * n, time3);
    if (rc != MOE_OK) return rc;
    double traffic_bottleneck = 0.0;
    rc = colocate_match(n, n, Da, Db, pair, &traffic_bottleneck);       // stage one: experts against experts, traffic only
    if (rc != MOE_OK) return rc;
    try {
        std::vector<double> W((size_t)n * n);                           // stage two: GPUs against the pairs found
        for (int g = 0; g < n; ++g)
            for (int i = 0; i < n; ++i) W[(size_t)g * n + i] = time3[((size_t)g * n + i) * n + pair[i]];
        std::vector<int32_t> item(n);
        rc = bottleneck_perfect(n, W.data(), item.data(), value);
        if (rc != MOE_OK) return rc;
        for (int g = 0; g < n; ++g) gpu_of_pair[item[g]] = g;
    } catch (const std::bad_alloc&) {
        return moe_set_error(MOE_ENOMEM, "colocate_hetero_match: host allocation failed");
    }
    return MOE_OK;
}

extern "C" int aurora_layer_time(int32_t n, const double* G, const double* N, const double* F, const double* C,
                                 const double* A, double* t_out) {
    if (!G || !N || !F || !C || !A || !t_out) return moe_set_error(MOE_EINVAL, "aurora_layer_time: NULL argument");
    if (n < 1) return moe_set_error(MOE_ESHAPE, "aurora_layer_time: need n >= 1");
    double gn = G[0] + N[0], fc = F[0] + C[0], a = A[0];
    for (int i = 1; i < n; ++i) {
        gn = std::max(gn, G[i] + N[i]);
        fc = std::max(fc, F[i] + C[i]);
        a = std::max(a, A[i]);
    }
    *t_out = gn + fc + a;
    return MOE_OK;
}

extern "C" int aurora_colocated_time(double Ga, double Gb, double Fa, double Fb, double Aa, double Ab, double Na, double Nb,
                                     double NaNb, aurora_coloc_times* out) {
    if (!out) return moe_set_error(MOE_EINVAL, "aurora_colocated_time: NULL argument");
    const double in[9] = {Ga, Gb, Fa, Fb, Aa, Ab, Na, Nb, NaNb};
    for (double v : in)
        if (!(v >= 0.0) || !std::isfinite(v)) return moe_set_error(MOE_EINVAL, "aurora_colocated_time: durations must be finite and >= 0");
    // the second all-to-all is the first one reversed: same stand-alone and aggregated durations
    const double Ca = Na, Cb = Nb, CaCb = NaNb;
    out->Gb = Gb;
    out->Na = Na;
    out->Fa = std::max(Gb, Na) + Fa;
    out->Nb = std::max(NaNb, Gb + Nb);
    out->Fb = std::max(out->Fa, out->Nb) + Fb;
    out->Ca = std::max(NaNb + Ca, out->Fa + Ca);
    out->Aa = std::max(out->Fb, out->Ca) + Aa;
    out->Cb = std::max(NaNb + CaCb, out->Fb + Cb);
    out->Ab = std::max(out->Aa, out->Cb) + Ab;
    out->Ga = out->Ab + Ga;
    out->t = out->Ga;
    return MOE_OK;
}
