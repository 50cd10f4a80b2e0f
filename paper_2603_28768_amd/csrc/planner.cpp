// Host-side replica planner (craft_plan and its accessors).
//
// Sec. 4.2 of the paper: estimate what replicas buy (Alg. 1's load model), decide how
// many each layer gets under the memory budget, fix how many experts each rank holds per
// layer (Alg. 3), then place expert copies on ranks greedily (Sec. 4.2.2).
#include <algorithm>
#include <cmath>
#include <cstring>
#include <limits>
#include <memory>
#include <new>
#include <numeric>

#include "plan_internal.h"

namespace {

typedef __int128 wide_t;

struct Copy {
    int64_t weight;
    int32_t expert;
    int32_t index;
};

// Which expert receives the next replica: the one whose load per existing copy is
// largest (exact cross-multiplied comparison, first such expert on ties).  Experts that
// already have one copy per rank are passed over.  -1 when none is left.
int32_t hottest_per_copy(const int64_t *ws, const std::vector<int32_t> &copies, int32_t D) {
    int32_t pick = -1;
    for (int32_t e = 0; e < (int32_t)copies.size(); ++e) {
        if (copies[e] >= D) continue;
        if (pick < 0) { pick = e; continue; }
        wide_t lhs = (wide_t)ws[e] * copies[pick];
        wide_t rhs = (wide_t)ws[pick] * copies[e];
        if (lhs > rhs) pick = e;
    }
    return pick;
}

// Alg. 3 starts every layer from floor(total / D); when no Alg. 3 result exists yet (the
// estimate of Alg. 1 is taken before it), the remainder goes to the first ranks.
std::vector<int32_t> even_capacity(int32_t total, int32_t D) {
    std::vector<int32_t> cap(D, total / D);
    for (int32_t g = 0; g < total % D; ++g) cap[g] += 1;
    return cap;
}

// Sec. 4.2.2 step 5: heaviest copy first onto the least-loaded rank that has room; a rank
// already holding the same expert is avoided while another choice exists.  Per-copy
// weight is Alg. 1's floor(W / copies).
struct Placement {
    std::vector<std::vector<std::pair<int32_t, int32_t>>> held;  // per rank: (expert, copy)
    std::vector<int64_t> load;
};

Placement place_copies(const int64_t *ws, const std::vector<int32_t> &copies,
                       const std::vector<int32_t> &cap) {
    const int32_t E = (int32_t)copies.size(), D = (int32_t)cap.size();
    std::vector<Copy> items;
    for (int32_t e = 0; e < E; ++e)
        for (int32_t q = 0; q < copies[e]; ++q) items.push_back({ws[e] / copies[e], e, q});
    std::stable_sort(items.begin(), items.end(), [](const Copy &a, const Copy &b) {
        if (a.weight != b.weight) return a.weight > b.weight;
        if (a.expert != b.expert) return a.expert < b.expert;
        return a.index < b.index;
    });
    Placement out;
    out.held.resize(D);
    out.load.assign(D, 0);
    std::vector<int32_t> room(cap);
    std::vector<char> holds((size_t)D * E, 0);
    for (const Copy &it : items) {
        int32_t target = -1;
        for (int pass = 0; pass < 2 && target < 0; ++pass) {
            for (int32_t g = 0; g < D; ++g) {
                if (room[g] <= 0) continue;
                if (pass == 0 && holds[(size_t)g * E + it.expert]) continue;
                if (target < 0 || out.load[g] < out.load[target] ||
                    (out.load[g] == out.load[target] && room[g] > room[target]))
                    target = g;
            }
        }
        out.held[target].push_back({it.expert, it.index});
        holds[(size_t)target * E + it.expert] = 1;
        out.load[target] += it.weight;
        room[target] -= 1;
    }
    return out;
}

int64_t max_rank_load(const int64_t *ws, const std::vector<int32_t> &copies, int32_t D) {
    int32_t total = std::accumulate(copies.begin(), copies.end(), 0);
    Placement p = place_copies(ws, copies, even_capacity(total, D));
    return *std::max_element(p.load.begin(), p.load.end());
}

// Alg. 3.  total[l] = physical experts of layer l.  A[l][g] = experts on rank g.
std::vector<std::vector<int32_t>> interleaved_capacity(const std::vector<int32_t> &total, int32_t D) {
    const int32_t L = (int32_t)total.size();
    std::vector<std::vector<int32_t>> A(L, std::vector<int32_t>(D));
    std::vector<int64_t> held(D, 0);
    for (int32_t l = 0; l < L; ++l)
        for (int32_t g = 0; g < D; ++g) { A[l][g] = total[l] / D; held[g] += A[l][g]; }
    for (int32_t l = 0; l < L; ++l) {
        const int32_t extra = total[l] % D;
        if (extra == 0) continue;
        std::vector<int64_t> sorted(held);
        std::nth_element(sorted.begin(), sorted.begin() + (extra - 1), sorted.end());
        const int64_t cutoff = sorted[extra - 1];
        std::vector<int32_t> chosen, tied;
        for (int32_t g = 0; g < D; ++g) {
            if (held[g] < cutoff) chosen.push_back(g);
            else if (held[g] == cutoff) tied.push_back(g);
        }
        const int32_t want = extra - (int32_t)chosen.size();
        // evenly spread over the tied ranks: positions floor(i * n / want), the spacing of
        // the paper's worked example (four tied devices, two extras -> devices 0 and 2)
        for (int32_t i = 0; i < want; ++i)
            chosen.push_back(tied[(size_t)((int64_t)i * (int64_t)tied.size() / want)]);
        for (int32_t g : chosen) { A[l][g] += 1; held[g] += 1; }
    }
    return A;
}

// Objective 0.  One replica at a time to the layer whose estimated maximum rank load drops
// most per byte; steps without gain are still taken while something fits the budget.
void unit_greedy(const std::vector<int64_t> &ws, int32_t L, int32_t E, int32_t D,
                 const std::vector<int64_t> &cost, int64_t budget, std::vector<int32_t> &x,
                 std::vector<std::vector<int32_t>> &copies, std::vector<int32_t> &order) {
    std::vector<int64_t> now(L), next(L, 0);
    std::vector<std::vector<int32_t>> next_copies(L);
    std::vector<char> have_next(L, 0);
    for (int32_t l = 0; l < L; ++l) now[l] = max_rank_load(&ws[(size_t)l * E], copies[l], D);
    int64_t spent = 0;
    const int64_t cap_per_layer = (int64_t)E * (D - 1);
    for (;;) {
        int32_t pick = -1;
        for (int32_t l = 0; l < L; ++l) {
            if (cost[l] > budget - spent || x[l] >= cap_per_layer) continue;
            if (!have_next[l]) {
                next_copies[l] = copies[l];
                int32_t e = hottest_per_copy(&ws[(size_t)l * E], next_copies[l], D);
                if (e < 0) continue;
                next_copies[l][e] += 1;
                next[l] = max_rank_load(&ws[(size_t)l * E], next_copies[l], D);
                have_next[l] = 1;
            }
            if (pick < 0) { pick = l; continue; }
            // (now - next) / cost, larger first; then larger current maximum; then lower layer
            wide_t lhs = (wide_t)(now[l] - next[l]) * cost[pick];
            wide_t rhs = (wide_t)(now[pick] - next[pick]) * cost[l];
            if (lhs > rhs || (lhs == rhs && now[l] > now[pick])) pick = l;
        }
        if (pick < 0) break;
        x[pick] += 1;
        spent += cost[pick];
        copies[pick].swap(next_copies[pick]);
        now[pick] = next[pick];
        have_next[pick] = 0;
        order.push_back(pick);
    }
}

// Alg. 1.  For r = 0 and r = 1, 2, 4, .. <= D: place the layer once on the summed loads with
// r replicas, then replay every batch under that placement (a copy of expert e carries
// floor(W[b][l][e] / copies[e])) and average (mean rank load) / (maximum rank load) over the
// batches.  base[l] = that mean at r = 0; gain[i][l] = mean at counts[i] minus base[l] (the
// listing's scalar `base` is assigned from BAL[l], so it is read per layer).  A batch that
// sends nothing to the layer scores 1.
void replay_benefit(const int64_t *load, int64_t B, const std::vector<int64_t> &ws, int32_t L,
                    int32_t E, int32_t D, craft_plan_t &plan) {
    plan.benefit_counts.clear();
    for (int64_t r = 1; r <= D && r <= (int64_t)E * (D - 1); r *= 2)
        plan.benefit_counts.push_back((int32_t)r);
    const size_t K = plan.benefit_counts.size();
    plan.benefit_base.assign(L, 0.0);
    plan.benefit_gain.assign(K * (size_t)L, 0.0);
    std::vector<int64_t> G(D);
    for (int32_t l = 0; l < L; ++l) {
        const int64_t *wl = &ws[(size_t)l * E];
        std::vector<int32_t> copies(E, 1);
        int32_t have = 0;
        for (size_t i = 0; i <= K; ++i) {
            const int32_t r = i == 0 ? 0 : plan.benefit_counts[i - 1];
            for (; have < r; ++have) copies[hottest_per_copy(wl, copies, D)] += 1;
            Placement pl = place_copies(wl, copies, even_capacity(E + r, D));
            double bal = 0.0;
            for (int64_t b = 0; b < B; ++b) {
                const int64_t *wb = load + ((size_t)b * L + l) * E;
                int64_t mx = 0, sum = 0;
                for (int32_t g = 0; g < D; ++g) {
                    int64_t v = 0;
                    for (auto &ec : pl.held[g]) v += wb[ec.first] / copies[ec.first];
                    mx = std::max(mx, v);
                    sum += v;
                }
                bal += mx == 0 ? 1.0 : ((double)sum / (double)D) / (double)mx;
            }
            const double mean = bal / (double)B;
            if (i == 0) plan.benefit_base[l] = mean;
            else plan.benefit_gain[(i - 1) * (size_t)L + l] = mean - plan.benefit_base[l];
        }
    }
}

// Alg. 2 for every capacity 0..C: value[c] = largest total gain of one count per layer from
// {0} + counts that sums to exactly c; reach[c] = whether any selection does.  Counts are
// tried in ascending order and only a strictly larger value replaces the incumbent, so ties
// keep "no replica", then the smaller count.  choice[l][c] = count taken by layer l-1.
struct Knapsack {
    std::vector<double> value;
    std::vector<char> reach;
    std::vector<std::vector<int32_t>> choice;
};
Knapsack knapsack(const craft_plan_t &plan, int32_t L, int64_t C) {
    const size_t K = plan.benefit_counts.size();
    Knapsack k;
    k.value.assign(C + 1, 0.0);
    k.reach.assign(C + 1, 0);
    k.reach[0] = 1;
    k.choice.assign(L + 1, std::vector<int32_t>(C + 1, 0));
    std::vector<double> nv(C + 1);
    std::vector<char> nr(C + 1);
    for (int32_t l = 1; l <= L; ++l) {
        for (int64_t c = 0; c <= C; ++c) {
            nv[c] = k.value[c];
            nr[c] = k.reach[c];
            for (size_t i = 0; i < K; ++i) {
                const int64_t r = plan.benefit_counts[i];
                if (c < r || !k.reach[c - r]) continue;
                const double cand = k.value[c - r] + plan.benefit_gain[i * (size_t)L + (l - 1)];
                if (!nr[c] || cand > nv[c]) { nv[c] = cand; nr[c] = 1; k.choice[l][c] = (int32_t)r; }
            }
        }
        k.value.swap(nv);
        k.reach.swap(nr);
    }
    return k;
}

// Sec. 4.2.1 steps 2 and 3.  The replica total is the budget (capped at what the candidate
// counts can hold), or with auto_r the multiple R * D <= budget with the highest total gain
// per replica (ties: smaller R); a total no selection reaches falls back to the next lower
// one that is reachable.  Then Alg. 2's back-trace.
void knapsack_allocation(craft_plan_t &plan, int32_t L, int32_t D, int64_t budget, bool auto_r,
                         std::vector<int32_t> &x) {
    x.assign(L, 0);
    if (plan.benefit_counts.empty()) return;
    int64_t cap = std::min<int64_t>(budget, (int64_t)L * plan.benefit_counts.back());
    Knapsack k = knapsack(plan, L, cap);
    if (auto_r) {
        int64_t best_R = 0;
        double best = 0.0;
        for (int64_t R = 1; R * D <= cap; ++R) {
            if (!k.reach[R * D]) continue;
            const double per = k.value[R * D] / (double)(R * D);
            if (best_R == 0 || per > best) { best_R = R; best = per; }
        }
        cap = best_R * D;
        plan.auto_R = (int32_t)best_R;
    }
    while (!k.reach[cap]) cap -= 1;
    plan.total_gain = k.value[cap];
    int64_t c = cap;
    for (int32_t l = L; l >= 1; --l) {
        const int32_t r = k.choice[l][c];
        x[l - 1] = r;
        c -= r;
    }
}

}  // namespace

size_t craft_tables_words(int32_t E, int32_t S) {
    size_t hdr = sizeof(craft_tables_header) / sizeof(int32_t);
    return hdr + (size_t)E + (size_t)(E + 1) + 3 * (size_t)S;
}

void craft_tables_build(const craft_layer_plan &lp, int32_t E, int32_t rank, int32_t *buf) {
    const int32_t S = (int32_t)lp.slot_expert.size();
    craft_tables_header h;
    std::memset(&h, 0, sizeof(h));
    h.E = E;
    h.S = S;
    h.s_lo = lp.rank_slot_off[rank];
    h.s_hi = lp.rank_slot_off[rank + 1];
    int32_t w = (int32_t)(sizeof(h) / sizeof(int32_t));
    h.off_copies = w; w += E;
    h.off_efirst = w; w += E + 1;
    h.off_eslots = w; w += S;
    h.off_slot_expert = w; w += S;
    h.off_slot_copy = w; w += S;
    h.total_words = w;
    std::memcpy(buf, &h, sizeof(h));
    int32_t *copies = buf + h.off_copies, *efirst = buf + h.off_efirst;
    int32_t *eslots = buf + h.off_eslots, *sexp = buf + h.off_slot_expert;
    int32_t *scopy = buf + h.off_slot_copy;
    for (int32_t e = 0; e < E; ++e) copies[e] = lp.copies[e];
    efirst[0] = 0;
    for (int32_t e = 0; e < E; ++e) efirst[e + 1] = efirst[e] + copies[e];
    std::vector<int32_t> seen(E, 0);
    for (int32_t p = 0; p < S; ++p) {
        const int32_t e = lp.slot_expert[p];
        sexp[p] = e;
        scopy[p] = seen[e];
        eslots[efirst[e] + seen[e]] = p;
        seen[e] += 1;
    }
}

extern "C" {

const char *craft_status_str(craft_status s) {
    switch (s) {
        case CRAFT_OK: return "ok";
        case CRAFT_EINVAL: return "invalid argument";
        case CRAFT_ENOMEM: return "out of host memory";
        case CRAFT_EHIP: return "HIP runtime error";
        case CRAFT_EWORKSPACE: return "workspace too small";
        case CRAFT_EINFEASIBLE: return "request exceeds a fixed limit of the library";
    }
    return "unknown status";
}

craft_status craft_plan(const craft_plan_params *pp, craft_plan_t **out) {
    if (!pp || !out) return CRAFT_EINVAL;
    *out = nullptr;
    const int32_t L = pp->L, E = pp->E, D = pp->D;
    if (L <= 0 || E <= 0 || D <= 0 || pp->B <= 0 || !pp->load || pp->budget_bytes < 0)
        return CRAFT_EINVAL;
    if (pp->objective < 0 || pp->objective > 2) return CRAFT_EINVAL;
    if ((int64_t)E * D > (int64_t)1 << 30) return CRAFT_EINVAL;
    std::vector<int64_t> cost(L, 1);
    if (pp->bytes_per_replica)
        for (int32_t l = 0; l < L; ++l) {
            if (pp->bytes_per_replica[l] <= 0) return CRAFT_EINVAL;
            cost[l] = pp->bytes_per_replica[l];
        }
    // objectives 1 and 2 count replicas, as the paper does: one size for every layer
    if (pp->objective != 0)
        for (int32_t l = 1; l < L; ++l)
            if (cost[l] != cost[0]) return CRAFT_EINVAL;
    for (size_t i = 0, n = (size_t)pp->B * L * E; i < n; ++i)
        if (pp->load[i] < 0) return CRAFT_EINVAL;
    try {
        // Alg. 1: W_s = W summed over batches
        std::vector<int64_t> ws((size_t)L * E, 0);
        for (int64_t b = 0; b < pp->B; ++b)
            for (int32_t l = 0; l < L; ++l)
                for (int32_t e = 0; e < E; ++e)
                    ws[(size_t)l * E + e] += pp->load[((size_t)b * L + l) * E + e];

        std::unique_ptr<struct craft_plan> plan(new struct craft_plan());
        plan->L = L; plan->E = E; plan->D = D; plan->gpus_per_node = pp->gpus_per_node;
        plan->ranks.reset(new craft_rank_state[(size_t)L * D]);

        std::vector<std::vector<int32_t>> copies(L, std::vector<int32_t>(E, 1));
        std::vector<int32_t> x(L, 0);
        if (pp->objective == 0) {
            unit_greedy(ws, L, E, D, cost, pp->budget_bytes, x, copies, plan->order);
        } else {
            const int64_t budget = pp->budget_bytes / cost[0];
            if (pp->objective == 1) {
                replay_benefit(pp->load, pp->B, ws, L, E, D, *plan);
                knapsack_allocation(*plan, L, D, budget, pp->auto_r != 0, x);
            } else {
                const int64_t n = std::min<int64_t>(budget / L, (int64_t)E * (D - 1));
                x.assign(L, (int32_t)n);
            }
            for (int32_t l = 0; l < L; ++l)
                for (int32_t i = 0; i < x[l]; ++i)
                    copies[l][hottest_per_copy(&ws[(size_t)l * E], copies[l], D)] += 1;
        }

        // Alg. 3 on the physical expert counts, then the final placement per layer
        std::vector<int32_t> total(L);
        for (int32_t l = 0; l < L; ++l) total[l] = E + x[l];
        std::vector<std::vector<int32_t>> A = interleaved_capacity(total, D);
        plan->layers.resize(L);
        for (int32_t l = 0; l < L; ++l) {
            craft_layer_plan &lp = plan->layers[l];
            lp.n_replicas = x[l];
            lp.copies = copies[l];
            Placement pl = place_copies(&ws[(size_t)l * E], copies[l], A[l]);
            lp.rank_slot_off.assign(1, 0);
            for (int32_t g = 0; g < D; ++g) {
                std::sort(pl.held[g].begin(), pl.held[g].end());
                for (auto &ec : pl.held[g]) lp.slot_expert.push_back(ec.first);
                lp.rank_slot_off.push_back((int32_t)lp.slot_expert.size());
            }
            lp.rank_load = pl.load;
            lp.expert_load.assign(ws.begin() + (size_t)l * E, ws.begin() + (size_t)(l + 1) * E);
            int64_t mx = 0, sum = 0;
            for (int64_t v : pl.load) { mx = std::max(mx, v); sum += v; }
            lp.est_max_rank_load = mx;
            lp.est_balancedness = mx == 0 ? 1.0 : ((double)sum / (double)D) / (double)mx;
        }
        *out = plan.release();
        return CRAFT_OK;
    } catch (const std::bad_alloc &) {
        return CRAFT_ENOMEM;
    }
}

void craft_plan_destroy(craft_plan_t *plan) { delete plan; }

craft_status craft_plan_summary(const craft_plan_t *plan, int32_t *L, int32_t *E, int32_t *D,
                                int64_t *total_replicas, double *replication_factor,
                                double *memory_saving_vs_uniform) {
    if (!plan) return CRAFT_EINVAL;
    int64_t total = 0;
    for (const auto &lp : plan->layers) total += lp.n_replicas;
    if (L) *L = plan->L;
    if (E) *E = plan->E;
    if (D) *D = plan->D;
    if (total_replicas) *total_replicas = total;
    if (replication_factor) *replication_factor = (double)total / (double)plan->D;
    if (memory_saving_vs_uniform)
        *memory_saving_vs_uniform = total ? (double)plan->L * (double)plan->D / (double)total
                                          : std::numeric_limits<double>::infinity();
    return CRAFT_OK;
}

craft_status craft_plan_layer_info(const craft_plan_t *plan, int32_t layer, int32_t *n_replicas,
                                   int32_t *n_slots, double *est_balancedness,
                                   int64_t *est_max_rank_load) {
    if (!plan || layer < 0 || layer >= plan->L) return CRAFT_EINVAL;
    const craft_layer_plan &lp = plan->layers[layer];
    if (n_replicas) *n_replicas = lp.n_replicas;
    if (n_slots) *n_slots = (int32_t)lp.slot_expert.size();
    if (est_balancedness) *est_balancedness = lp.est_balancedness;
    if (est_max_rank_load) *est_max_rank_load = lp.est_max_rank_load;
    return CRAFT_OK;
}

craft_status craft_plan_layer_tables(const craft_plan_t *plan, int32_t layer, int32_t *copies,
                                     int32_t *slot_expert, int32_t *rank_slot_off,
                                     int64_t *rank_load) {
    if (!plan || layer < 0 || layer >= plan->L) return CRAFT_EINVAL;
    const craft_layer_plan &lp = plan->layers[layer];
    if (copies) std::copy(lp.copies.begin(), lp.copies.end(), copies);
    if (slot_expert) std::copy(lp.slot_expert.begin(), lp.slot_expert.end(), slot_expert);
    if (rank_slot_off) std::copy(lp.rank_slot_off.begin(), lp.rank_slot_off.end(), rank_slot_off);
    if (rank_load) std::copy(lp.rank_load.begin(), lp.rank_load.end(), rank_load);
    return CRAFT_OK;
}

craft_status craft_plan_greedy_order(const craft_plan_t *plan, int32_t *layers, int64_t cap,
                                     int64_t *n) {
    if (!plan || !n || cap < 0 || (cap > 0 && !layers)) return CRAFT_EINVAL;
    *n = (int64_t)plan->order.size();
    for (int64_t i = 0; i < std::min(*n, cap); ++i) layers[i] = plan->order[(size_t)i];
    return CRAFT_OK;
}

craft_status craft_plan_benefit(const craft_plan_t *plan, int32_t *n_counts, int32_t *counts,
                                double *base, double *gain, double *total_gain, int32_t *auto_R) {
    if (!plan) return CRAFT_EINVAL;
    const size_t K = plan->benefit_counts.size();
    if (n_counts) *n_counts = (int32_t)K;
    if (counts) std::copy(plan->benefit_counts.begin(), plan->benefit_counts.end(), counts);
    if (base) std::copy(plan->benefit_base.begin(), plan->benefit_base.end(), base);
    if (gain) std::copy(plan->benefit_gain.begin(), plan->benefit_gain.end(), gain);
    if (total_gain) *total_gain = plan->total_gain;
    if (auto_R) *auto_R = plan->auto_R;
    return CRAFT_OK;
}

craft_status craft_plan_rank_rows(const craft_plan_t *plan, int32_t layer, const int64_t *counts,
                                  int64_t *rows, int32_t *heaviest) {
    if (!plan || layer < 0 || layer >= plan->L || !counts) return CRAFT_EINVAL;
    const craft_layer_plan &lp = plan->layers[layer];
    const int32_t S = (int32_t)lp.slot_expert.size();
    std::vector<int32_t> seen(plan->E, 0);
    std::vector<int64_t> per_rank(plan->D, 0);
    int32_t g = 0;
    for (int32_t p = 0; p < S; ++p) {
        while (p >= lp.rank_slot_off[g + 1]) ++g;
        const int32_t e = lp.slot_expert[p];
        const int64_t n = counts[e], c = lp.copies[e], q = seen[e]++;
        if (n < 0) return CRAFT_EINVAL;
        per_rank[g] += n > q ? (n - q + c - 1) / c : 0;   // tokens i < n with i mod c == q
    }
    int32_t top = 0;
    for (int32_t r = 1; r < plan->D; ++r)
        if (per_rank[r] > per_rank[top]) top = r;
    if (rows) std::copy(per_rank.begin(), per_rank.end(), rows);
    if (heaviest) *heaviest = top;
    return CRAFT_OK;
}

craft_status craft_plan_diff(const craft_plan_t *old_plan, const craft_plan_t *new_plan,
                             int32_t layer, int32_t rank, int32_t *reuse, int32_t *n_fetch,
                             int32_t *n_drop) {
    if (!old_plan || !new_plan) return CRAFT_EINVAL;
    if (old_plan->L != new_plan->L || old_plan->E != new_plan->E || old_plan->D != new_plan->D)
        return CRAFT_EINVAL;
    if (layer < 0 || layer >= new_plan->L || rank < 0 || rank >= new_plan->D) return CRAFT_EINVAL;
    const craft_layer_plan &a = old_plan->layers[layer], &b = new_plan->layers[layer];
    const int32_t a_lo = a.rank_slot_off[rank], a_hi = a.rank_slot_off[rank + 1];
    const int32_t b_lo = b.rank_slot_off[rank], b_hi = b.rank_slot_off[rank + 1];
    // both runs ascend by expert: one merge pass pairs equal experts in order
    int32_t i = a_lo, fetch = 0, kept = 0;
    for (int32_t j = b_lo; j < b_hi; ++j) {
        while (i < a_hi && a.slot_expert[i] < b.slot_expert[j]) ++i;
        const bool hit = i < a_hi && a.slot_expert[i] == b.slot_expert[j];
        if (reuse) reuse[j - b_lo] = hit ? i - a_lo : -1;
        if (hit) { ++i; ++kept; } else ++fetch;
    }
    if (n_fetch) *n_fetch = fetch;
    if (n_drop) *n_drop = (a_hi - a_lo) - kept;
    return CRAFT_OK;
}

craft_status craft_plan_tables_bytes(const craft_plan_t *plan, int32_t layer, int32_t rank,
                                     size_t *bytes) {
    if (!plan || !bytes || layer < 0 || layer >= plan->L || rank < 0 || rank >= plan->D)
        return CRAFT_EINVAL;
    *bytes = craft_tables_words(plan->E, (int32_t)plan->layers[layer].slot_expert.size()) *
             sizeof(int32_t);
    return CRAFT_OK;
}

}  // extern "C"
