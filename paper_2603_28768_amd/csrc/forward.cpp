// Device-side entry points of the C ABI: argument checks, workspace layout, launches.
#include <algorithm>
#include <atomic>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <memory>
#include <mutex>
#include <queue>
#include <vector>

#include "kernels.h"

namespace {

using namespace craft;

inline hipStream_t as_stream(void *s) { return static_cast<hipStream_t>(s); }
inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---- workspace layout of one forward -------------------------------------------------
struct Layout {
    size_t ctrl, ids, w, lrank, dest, src, hist, chunk_tot, chunk_base, gate_logits, gate_ws, gate_ws_bytes, counts, slot_cnt, slot_off, mt_start, order, act, y, total;
    int64_t max_rows, NB;
};

int cached_num_cu();

size_t gate_workspace_bytes(int32_t dtype, int64_t T, int32_t H, int32_t E) {
    int nxf = 1, nsplit = 1;
    if (dtype == CRAFT_BF16 && T > 0) router_logits_shape(T, H, E, cached_num_cu(), true, &nxf, &nsplit);
    return nsplit > 1 ? (size_t)nsplit * (size_t)T * (size_t)E * sizeof(float) : 0;
}

Layout make_layout(int64_t T, int32_t k, int32_t E, int32_t S, int32_t nslots, int32_t H, int32_t I,
                   int32_t dtype, int64_t max_rows_arg, bool own_gate) {
    Layout L;
    const int64_t A = T * k;
    const size_t es = dtype == CRAFT_BF16 ? 2 : 4;
    const int64_t worst = T * std::min<int64_t>(k, nslots);
    L.max_rows = max_rows_arg > 0 ? std::min(max_rows_arg, worst) : worst;
    L.NB = (T + kTokPerBlock - 1) / kTokPerBlock;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = round_up(off + bytes, 256); return o; };
    L.ctrl = take(CTRL_WORDS * 4);
    L.ids = take((size_t)A * 4);
    L.w = take((size_t)A * 4);
    L.lrank = take((size_t)A);
    L.dest = take((size_t)A * 4);
    L.src = take((size_t)A * 4);
    L.hist = take((size_t)L.NB * E * 4);
    const size_t chunks = (size_t)(L.NB + kScanChunk - 1) / kScanChunk;
    L.chunk_tot = take(chunks * E * 4);
    L.chunk_base = take(chunks * E * 4);
    // scores and the split gate's partial scores, when the forward runs the gating network
    L.gate_ws_bytes = own_gate ? gate_workspace_bytes(dtype, T, H, E) : 0;
    L.gate_logits = take(own_gate ? (size_t)T * E * 4 : 0);
    L.gate_ws = take(L.gate_ws_bytes);
    L.counts = take((size_t)E * 4);
    L.slot_cnt = take((size_t)S * 4);
    L.slot_off = take((size_t)(S + 1) * 4);
    L.mt_start = take((size_t)(nslots + 1) * 4 * 2);
    L.order = take((size_t)(nslots + 1) * 4);
    L.act = take((size_t)L.max_rows * I * es);
    L.y = take((size_t)L.max_rows * H * es);
    L.total = off;
    return L;
}

// ---- kernel timing ---------------------------------------------------------------------
struct Timing {
    std::mutex mu;
    int level = 0;
    std::vector<hipEvent_t> ev;      // pairs
    std::vector<int> kind;           // kernel id of each recorded pair
    size_t used = 0;                 // pairs recorded since the last read
} g_timing;

struct ScopedEvent {
    hipStream_t s;
    hipEvent_t stop = nullptr;
    ScopedEvent(int kernel, hipStream_t stream) : s(stream) {
        Timing &t = g_timing;
        if (t.level == 0 || (t.level == 1 && kernel != CRAFT_K_GATEUP)) return;
        std::lock_guard<std::mutex> lk(t.mu);
        if ((t.used + 1) * 2 > t.ev.size()) return;
        hipEvent_t start = t.ev[t.used * 2];
        stop = t.ev[t.used * 2 + 1];
        t.kind[t.used] = kernel;
        t.used += 1;
        (void)hipEventRecord(start, s);
    }
    ~ScopedEvent() {
        if (stop) (void)hipEventRecord(stop, s);
    }
};

int cached_num_cu() {
    static int n = 0;
    if (n == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
            n = prop.multiProcessorCount;
        if (n <= 0) n = 256;
    }
    return n;
}

// ---- row-tile height of the packed FFN ---------------------------------------------------
// A row-tile may have 4 to 8 fragments of 32 rows.  Taller tiles reuse a weight fragment more
// often, but the tiles of the busy slots must also come out as whole rounds over the CUs: 176
// tiles of 8 fragments on 256 CUs take as long as 256 would.  The height is chosen per GEMM by
// playing the launch through on the host: expected rows per slot from the profiled loads the
// plan was made from (scaled to this batch), tiles handed to the first free CU in list order,
// with a tile costing a fixed part (starting it and streaming its weight block through one
// CU) plus a part per fragment.  The constants are fitted to tile timings on MI355X under
// full load; replayed against measured sweeps of the height on three workloads the model
// picks the fastest or second-fastest height each time.
double ffn_makespan(const std::vector<double> &slot_rows, int32_t frags, bool even, int64_t nt,
                    double fixed_us, double frag_us, bool riders, double rider_us, int32_t cus) {
    // the tile list as the kernel walks it: busy slots first (rows sorted, busiest first)
    std::vector<double> cost;
    int64_t ncold = 0, ncold2 = 0;
    for (double r : slot_rows) {
        const int64_t F = (int64_t)((r + 31.0) / 32.0);
        if (F <= 0) continue;
        if (r <= (double)kColdRows) { ncold += 1; ncold2 += F > 1 ? 1 : 0; continue; }
        const int64_t m = (F + frags - 1) / frags;
        for (int64_t n = 0; n < nt; ++n)
            for (int64_t i = 0; i < m; ++i) {
                const int64_t f = even ? (i + 1) * F / m - i * F / m : std::min<int64_t>(frags, F - i * frags);
                cost.push_back(fixed_us + frag_us * (double)f);
            }
    }
    // rider units go to the first tiles, one each (see kRiderHostFrags)
    const int64_t units2 = ncold2 * 4 * nt, units = units2 + (ncold - ncold2) * 2 * nt;
    int64_t carried = riders && frags <= kRiderHostFrags ? std::min<int64_t>((int64_t)cost.size(), units) : 0;
    if (carried < units2) carried = carried / (4 * nt) * (4 * nt);
    for (int64_t u = 0; u < carried; ++u) cost[(size_t)u] += rider_us;
    // what is left of the cold slots: half-width tiles, about half the cost
    const int64_t left2 = carried <= units2 ? ncold2 - carried / (4 * nt) : 0;
    const int64_t left1 = carried <= units2 ? (ncold - ncold2) * 2 * nt : units - carried;
    for (int64_t i = 0; i < left2 * 2 * nt; ++i) cost.push_back(4.0 + 0.5 * (fixed_us + frag_us * 2.0));
    for (int64_t i = 0; i < left1; ++i) cost.push_back(4.0 + 0.5 * (fixed_us + frag_us));
    std::priority_queue<double, std::vector<double>, std::greater<double>> free_at;
    for (int32_t i = 0; i < cus; ++i) free_at.push(0.0);
    double end = 0.0;
    for (double c : cost) {
        const double t = free_at.top() + c;
        free_at.pop();
        free_at.push(t);
        end = std::max(end, t);
    }
    return end;
}

struct tile_choice { int32_t frags[2]; bool riders[2]; };

tile_choice choose_tiles(const craft_plan_t *plan, int32_t layer, int32_t rank, int64_t T, int32_t k,
                         int32_t H, int32_t I, int32_t cus) {
    const craft_layer_plan &lp = plan->layers[layer];
    tile_choice best{{kFragsPacked, kFragsPacked}, {false, false}};
    double total = 0.0;
    for (int64_t v : lp.expert_load) total += (double)v;
    if (total <= 0.0 || T <= 0) return best;
    std::vector<double> rows;
    for (int32_t p = lp.rank_slot_off[rank]; p < lp.rank_slot_off[rank + 1]; ++p) {
        const int32_t e = lp.slot_expert[p];
        // a slot expected to see a fraction of a row is counted with one: it costs a tile per
        // column block as soon as a single token reaches it
        const double est = (double)(lp.expert_load[e] / lp.copies[e]) * (double)T * k / total;
        rows.push_back(est >= 0.2 ? std::max(1.0, est) : 0.0);
    }
    std::sort(rows.begin(), rows.end(), std::greater<double>());
    for (int kind = 0; kind < 2; ++kind) {
        const int64_t K = kind == 0 ? H : I, N = kind == 0 ? I : H;
        const int64_t nt = kind == 0 ? (N + 127) / 128 : (N + 255) / 256;
        // microseconds per tile under full load, linear in the contraction length K; from
        // per-tile device timestamps at K = 4096 and 7168 (gate/up) and 1536 and 2048 (down)
        const double fixed_us = kind == 0 ? 20.0 + 0.0055 * (double)K : 21.0 + 0.0020 * (double)K;
        const double frag_us = kind == 0 ? 1.5 + 0.00182 * (double)K : 0.1 + 0.00234 * (double)K;
        // A rider's weights come through the same path from L2 as the tile's own operands, and
        // that path is what bounds a tile under full load: the rider costs its bytes (5 KB per
        // step against the tile's 8 + fragments) rather than its one MFMA in 2 * fragments + 1.
        const double rider_us = 4.0 + 0.004 * (double)K;
        // Only where the busy slots' tiles make up a round or two does their count decide the
        // time; over many rounds the tallest tile (most reuse per weight fragment, fewest
        // fixed costs) wins by itself, and there the model is not trusted to say otherwise.
        int64_t tall_tiles = 0;
        for (double r : rows)
            if (r > (double)kColdRows) tall_tiles += (((int64_t)((r + 31.0) / 32.0) + kFragsPacked - 1) / kFragsPacked) * nt;
        if (tall_tiles > 2 * (int64_t)cus) continue;
        double best_t = 0.0;
        for (int32_t f = kFragsPacked; f >= 4; --f)
            for (int even = 0; even < 2; ++even)
                for (int riders = 0; riders < (f <= kRiderHostFrags ? 2 : 1); ++riders) {
                    const double t = ffn_makespan(rows, f, even != 0, nt, fixed_us, frag_us, riders != 0, rider_us, cus);
                    if ((f == kFragsPacked && !even) || t < best_t * 0.98) {    // a change has to earn it
                        best_t = t;
                        best.frags[kind] = even ? -f : f;
                        best.riders[kind] = riders != 0;
                    }
                }
    }
    return best;
}

// The choice for (layer, rank, T, k, H, I) is made once and kept with the plan: later forwards
// of the same shape find it by walking a short insert-only list, without a lock.
tile_choice tiles_for(const craft_plan_t *plan, int32_t layer, int32_t rank, const craft_fwd_args *a,
                      bool packed) {
    if (a->dtype != CRAFT_BF16) return {{kFragsF32, kFragsF32}, {false, false}};
    if (!packed) return {{kFragsBf16, kFragsBf16}, {false, false}};
    craft_rank_state &rs = plan->state(layer, rank);
    auto find = [&]() -> const craft_tile_choice * {
        for (const craft_tile_choice *t = rs.tiles.load(std::memory_order_acquire); t; t = t->next)
            if (t->T == a->T && t->k == a->k && t->H == a->H && t->I == a->I) return t;
        return nullptr;
    };
    const craft_tile_choice *hit = find();
    if (!hit) {
        std::lock_guard<std::mutex> lk(rs.mu);
        hit = find();
        if (!hit) {
            const tile_choice c = choose_tiles(plan, layer, rank, a->T, a->k, a->H, a->I, cached_num_cu());
            craft_tile_choice *n = new craft_tile_choice{a->T, a->k, a->H, a->I, {c.frags[0], c.frags[1]},
                                                         {c.riders[0], c.riders[1]},
                                                         rs.tiles.load(std::memory_order_relaxed)};
            rs.tiles.store(n, std::memory_order_release);
            hit = n;
        }
    }
    tile_choice c{{hit->frags[0], hit->frags[1]}, {hit->riders[0], hit->riders[1]}};
    // the caller's own heights: riders wherever such tiles can carry them, unless told
    const int32_t rows_arg[2] = {a->tile_rows_gateup, a->tile_rows_down};
    const int32_t riders_arg[2] = {a->riders_gateup, a->riders_down};
    for (int kind = 0; kind < 2; ++kind) {
        if (rows_arg[kind]) { c.frags[kind] = rows_arg[kind] / 32; c.riders[kind] = true; }
        if (riders_arg[kind]) c.riders[kind] = riders_arg[kind] > 0;
        c.riders[kind] = c.riders[kind] && std::abs(c.frags[kind]) <= kRiderHostFrags;
    }
    return c;
}

craft_status check_fwd(const craft_plan_t *plan, int32_t layer, int32_t rank, const craft_fwd_args *a) {
    if (!plan || !a || layer < 0 || layer >= plan->L || rank < 0 || rank >= plan->D) return CRAFT_EINVAL;
    if (a->dtype != CRAFT_F32 && a->dtype != CRAFT_BF16) return CRAFT_EINVAL;
    if (a->T < 0 || a->H <= 0 || a->I <= 0 || a->k <= 0 || a->k > 64 || a->k > plan->E) return CRAFT_EINVAL;
    if (plan->E > 1024 || a->max_rows < 0) return CRAFT_EINVAL;
    for (int32_t r : {a->tile_rows_gateup, a->tile_rows_down})
        if (r != 0 && (r % 32 || r < 128 || r > 256)) return CRAFT_EINVAL;
    for (int32_t r : {a->riders_gateup, a->riders_down})
        if (r < -1 || r > 1) return CRAFT_EINVAL;
    if (a->T * (int64_t)a->k >= ((int64_t)1 << 31)) return CRAFT_EINVAL;
    const int unit = a->dtype == CRAFT_BF16 ? 8 : 4;
    if (a->H % unit || a->I % unit) return CRAFT_EINVAL;
    const craft_layer_plan &lp = plan->layers[layer];
    const int32_t nslots = lp.rank_slot_off[rank + 1] - lp.rank_slot_off[rank];
    if (nslots > 1024) return CRAFT_EINVAL;
    return CRAFT_OK;
}

}  // namespace

extern "C" {

craft_status craft_router_logits_workspace(int32_t dtype, int64_t T, int32_t H, int32_t E,
                                           size_t *bytes) {
    if (!bytes || (dtype != CRAFT_F32 && dtype != CRAFT_BF16)) return CRAFT_EINVAL;
    if (T < 0 || H <= 0 || E <= 0 || E > 1024 || (dtype == CRAFT_BF16 && H % 8)) return CRAFT_EINVAL;
    *bytes = gate_workspace_bytes(dtype, T, H, E);
    return CRAFT_OK;
}

craft_status craft_router_logits(int32_t dtype, const void *x, const void *w_router, int64_t T,
                                 int32_t H, int32_t E, float *logits, void *workspace,
                                 size_t workspace_bytes, void *stream) {
    if (dtype != CRAFT_F32 && dtype != CRAFT_BF16) return CRAFT_EINVAL;
    if (T < 0 || H <= 0 || E <= 0 || E > 1024 || (dtype == CRAFT_BF16 && H % 8)) return CRAFT_EINVAL;
    if (T * (int64_t)E >= ((int64_t)1 << 40)) return CRAFT_EINVAL;
    if (T == 0) return CRAFT_OK;
    if (!x || !w_router || !logits || !aligned(x, 16) || !aligned(w_router, 16) || !aligned(logits, 4))
        return CRAFT_EINVAL;
    if (workspace && !aligned(workspace, 16)) return CRAFT_EINVAL;
    size_t need = 0;
    craft_status st = craft_router_logits_workspace(dtype, T, H, E, &need);
    if (st != CRAFT_OK) return st;
    const bool split = workspace && need > 0 && workspace_bytes >= need;
    RouterArgs ra{dtype, x, w_router, T, H, E, logits, cached_num_cu(),
                  split ? static_cast<float *>(workspace) : nullptr, 1};
    return launch_router_logits(ra, as_stream(stream)) == hipSuccess ? CRAFT_OK : CRAFT_EHIP;
}

craft_status craft_route_topk(const float *logits, int64_t T, int32_t E, int32_t k,
                              int32_t renormalize, int32_t *ids, float *w, void *stream) {
    if (T < 0 || E <= 0 || E > 1024 || k <= 0 || k > E || k > 64) return CRAFT_EINVAL;
    if (T == 0) return CRAFT_OK;
    if (!logits || !ids || !w || !aligned(logits, 4) || !aligned(ids, 4) || !aligned(w, 4)) return CRAFT_EINVAL;
    RouteArgs ra{logits, T, E, k, renormalize ? 1 : 0, ids, w, nullptr, nullptr, nullptr};
    return launch_route(ra, as_stream(stream)) == hipSuccess ? CRAFT_OK : CRAFT_EHIP;
}

craft_status craft_expert_load(const int32_t *topk_ids, int32_t L, int64_t T, int32_t k, int32_t E,
                               int64_t batch_tokens, int64_t *counts, void *stream) {
    if (L <= 0 || T < 0 || k <= 0 || E <= 0 || E > 4096 || batch_tokens <= 0) return CRAFT_EINVAL;
    if (T == 0) return CRAFT_OK;
    if (!topk_ids || !counts || !aligned(topk_ids, 16) || !aligned(counts, 8)) return CRAFT_EINVAL;
    LoadArgs la{topk_ids, L, k, E, T, batch_tokens, (T + batch_tokens - 1) / batch_tokens, counts};
    return launch_expert_load(la, as_stream(stream)) == hipSuccess ? CRAFT_OK : CRAFT_EHIP;
}

craft_status craft_load_accumulate(const int32_t *counts, int64_t n, int64_t *window, void *stream) {
    if (n < 0 || n > ((int64_t)1 << 40)) return CRAFT_EINVAL;
    if (n == 0) return CRAFT_OK;
    if (!counts || !window || !aligned(counts, 4) || !aligned(window, 8)) return CRAFT_EINVAL;
    return launch_load_accumulate(counts, n, window, as_stream(stream)) == hipSuccess ? CRAFT_OK
                                                                                        : CRAFT_EHIP;
}

craft_status craft_plan_tables_upload(craft_plan_t *plan, int32_t layer, int32_t rank,
                                      void *dev_tables, size_t bytes, void *stream) {
    if (!plan || !dev_tables || layer < 0 || layer >= plan->L || rank < 0 || rank >= plan->D)
        return CRAFT_EINVAL;
    if (!aligned(dev_tables, 256)) return CRAFT_EINVAL;
    const craft_layer_plan &lp = plan->layers[layer];
    const size_t words = craft_tables_words(plan->E, (int32_t)lp.slot_expert.size());
    if (bytes < words * sizeof(int32_t)) return CRAFT_EWORKSPACE;
    craft_rank_state &rs = plan->state(layer, rank);
    try {
        {
            // the host copy of the tables is built once and stays with the plan, so the copy
            // below may still be in flight when this call returns
            std::lock_guard<std::mutex> lk(rs.mu);
            if (rs.host_tables.empty()) {
                std::vector<int32_t> host(words);
                craft_tables_build(lp, plan->E, rank, host.data());
                rs.host_tables.swap(host);
            }
        }
        std::lock_guard<std::mutex> lk(plan->reg_mutex);
        auto it = plan->reg_of.find(dev_tables);
        const bool same = it != plan->reg_of.end() && it->second->layer == layer && it->second->rank == rank;
        if (it != plan->reg_of.end() && !same) {
            // the buffer held another rank's tables: its old entry goes blank
            it->second->dev.store(nullptr, std::memory_order_release);
            plan->reg_of.erase(it);
        }
        if (hipMemcpyAsync(dev_tables, rs.host_tables.data(), words * sizeof(int32_t), hipMemcpyHostToDevice,
                           as_stream(stream)) != hipSuccess)
            return CRAFT_EHIP;
        if (!same) {
            craft_table_reg *n = new craft_table_reg{{dev_tables}, rs.regs.load(std::memory_order_relaxed), layer, rank};
            rs.regs.store(n, std::memory_order_release);
            plan->reg_of.emplace(dev_tables, n);
        }
    } catch (const std::bad_alloc &) {
        return CRAFT_ENOMEM;
    }
    return CRAFT_OK;
}

craft_status craft_pack_weights_bytes(int32_t dtype, int32_t H, int32_t I, size_t *gateup_bytes,
                                      size_t *down_bytes) {
    if (dtype != CRAFT_BF16 || H <= 0 || I <= 0 || H % 8 || I % 8 || !gateup_bytes || !down_bytes)
        return CRAFT_EINVAL;
    packed_sizes(H, I, gateup_bytes, down_bytes);
    return CRAFT_OK;
}

craft_status craft_pack_weights(int32_t dtype, int32_t H, int32_t I, const void *w_gate,
                                const void *w_up, const void *w_down, void *packed_gateup,
                                void *packed_down, void *stream) {
    if (dtype != CRAFT_BF16 || H <= 0 || I <= 0 || H % 8 || I % 8) return CRAFT_EINVAL;
    if (!w_gate || !w_up || !w_down || !packed_gateup || !packed_down) return CRAFT_EINVAL;
    if (!aligned(w_gate, 16) || !aligned(w_up, 16) || !aligned(w_down, 16) ||
        !aligned(packed_gateup, 16) || !aligned(packed_down, 16))
        return CRAFT_EINVAL;
    return launch_pack(H, I, w_gate, w_up, w_down, packed_gateup, packed_down, as_stream(stream)) ==
                   hipSuccess ? CRAFT_OK : CRAFT_EHIP;
}

craft_status craft_quantize_e4m3(const void *w, int64_t rows, int32_t K, uint8_t *codes, float *scale,
                                 void *stream) {
    if (rows < 0 || K <= 0 || K % 8) return CRAFT_EINVAL;
    if (rows == 0) return CRAFT_OK;
    if (!w || !codes || !scale || !aligned(w, 16) || !aligned(codes, 8) || !aligned(scale, 4))
        return CRAFT_EINVAL;
    return launch_quantize_e4m3(w, rows, K, codes, scale, as_stream(stream)) == hipSuccess ? CRAFT_OK
                                                                                             : CRAFT_EHIP;
}

craft_status craft_pack_weights_e4m3_bytes(int32_t H, int32_t I, size_t *gateup_bytes,
                                           size_t *down_bytes) {
    if (H <= 0 || I <= 0 || H % 8 || I % 8 || !gateup_bytes || !down_bytes) return CRAFT_EINVAL;
    packed_sizes_e4m3(H, I, gateup_bytes, down_bytes);
    return CRAFT_OK;
}

craft_status craft_pack_weights_e4m3(int32_t H, int32_t I, const uint8_t *gate_codes,
                                     const uint8_t *up_codes, const uint8_t *down_codes,
                                     const float *gate_scale, const float *up_scale,
                                     const float *down_scale, void *packed_gateup,
                                     void *packed_down, void *stream) {
    if (H <= 0 || I <= 0 || H % 8 || I % 8) return CRAFT_EINVAL;
    if (!gate_codes || !up_codes || !down_codes || !gate_scale || !up_scale || !down_scale ||
        !packed_gateup || !packed_down)
        return CRAFT_EINVAL;
    if (!aligned(gate_codes, 8) || !aligned(up_codes, 8) || !aligned(down_codes, 8) ||
        !aligned(packed_gateup, 16) || !aligned(packed_down, 16))
        return CRAFT_EINVAL;
    return launch_pack_e4m3(H, I, gate_codes, up_codes, down_codes, gate_scale, up_scale, down_scale,
                            packed_gateup, packed_down, as_stream(stream)) == hipSuccess ? CRAFT_OK
                                                                                          : CRAFT_EHIP;
}

craft_status craft_moe_rank_forward_workspace(const craft_plan_t *plan, int32_t layer, int32_t rank,
                                              const craft_fwd_args *a, size_t *bytes) {
    if (!bytes) return CRAFT_EINVAL;
    craft_status st = check_fwd(plan, layer, rank, a);
    if (st != CRAFT_OK) return st;
    const craft_layer_plan &lp = plan->layers[layer];
    const int32_t nslots = lp.rank_slot_off[rank + 1] - lp.rank_slot_off[rank];
    Layout L = make_layout(a->T, a->k, plan->E, (int32_t)lp.slot_expert.size(), nslots, a->H, a->I,
                           a->dtype, a->max_rows, a->logits == nullptr);
    *bytes = L.total;
    return CRAFT_OK;
}

}  // extern "C"

namespace {

// Scratch for craft_moe_rank_forward_static: device memory that lives in the library's code
// object, one copy per GPU.  In host code this name only stands for the symbol; the address
// on a given device comes from hipGetSymbolAddress (static_scratch below) and only that
// pointer is ever handed to a kernel or a copy.
constexpr size_t kStaticScratchBytes = (size_t)CRAFT_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_on_device[kMaxDevices];

// The array's address on the current device; resolved at the first call on each device.
craft_status static_scratch(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return CRAFT_EHIP;
    void *p = g_scratch_on_device[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return CRAFT_EHIP;
        g_scratch_on_device[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return CRAFT_OK;
}

// One forward on `workspace` (the caller's, or the library's static scratch); `a` has passed
// check_fwd.
craft_status forward_on(const craft_plan_t *plan, int32_t layer, int32_t rank, const craft_fwd_args *a,
                        void *workspace, size_t workspace_bytes, void *stream) {
    if (!workspace || !aligned(workspace, 256) || !a->tables) return CRAFT_EINVAL;
    {
        // the tables must be a buffer this plan filled for this (layer, rank)
        bool known = false;
        for (const craft_table_reg *r = plan->state(layer, rank).regs.load(std::memory_order_acquire); r && !known;
             r = r->next)
            known = r->dev.load(std::memory_order_relaxed) == a->tables;
        if (!known) return CRAFT_EINVAL;
    }
    const craft_layer_plan &lp = plan->layers[layer];
    const int32_t E = plan->E, S = (int32_t)lp.slot_expert.size();
    const int32_t s_lo = lp.rank_slot_off[rank], s_hi = lp.rank_slot_off[rank + 1];
    const int32_t nslots = s_hi - s_lo;
    const bool own_gate = a->logits == nullptr;
    Layout L = make_layout(a->T, a->k, E, S, nslots, a->H, a->I, a->dtype, a->max_rows, own_gate);
    if (workspace_bytes < L.total) return CRAFT_EWORKSPACE;
    if (a->T > 0) {
        if (!a->x || !a->out || (own_gate && !a->w_router)) return CRAFT_EINVAL;
        if (!aligned(a->x, 16) || !aligned(a->out, 16)) return CRAFT_EINVAL;
        if (own_gate ? !aligned(a->w_router, 16) : !aligned(a->logits, 4)) return CRAFT_EINVAL;
        const bool packed = a->w_gateup_packed && a->w_down_packed;
        if ((a->w_gateup_packed != nullptr) != (a->w_down_packed != nullptr)) return CRAFT_EINVAL;
        if (packed && a->dtype != CRAFT_BF16) return CRAFT_EINVAL;
        if (a->weight_format != CRAFT_W_BF16 && a->weight_format != CRAFT_W_E4M3) return CRAFT_EINVAL;
        if (a->weight_format == CRAFT_W_E4M3 && !packed) return CRAFT_EINVAL;
        if (nslots > 0 && !packed && (!a->w_gate || !a->w_up || !a->w_down)) return CRAFT_EINVAL;
        // the packed kernels address token rows of x and the fragments of one packed matrix by
        // 32-bit byte offsets from a base
        if (packed) {
            const int64_t limit = (int64_t)1 << 32;
            size_t gub = 0, dnb = 0;
            if (a->weight_format == CRAFT_W_E4M3) packed_sizes_e4m3(a->H, a->I, &gub, &dnb);
            else packed_sizes(a->H, a->I, &gub, &dnb);
            if (a->T * (int64_t)a->H * 2 >= limit || (int64_t)gub >= limit || (int64_t)dnb >= limit) return CRAFT_EINVAL;
        }
    }
    hipStream_t s = as_stream(stream);
    unsigned char *ws = static_cast<unsigned char *>(workspace);
    int32_t *ctrl = reinterpret_cast<int32_t *>(ws + L.ctrl);
    int32_t *ids = reinterpret_cast<int32_t *>(ws + L.ids);
    float *w = reinterpret_cast<float *>(ws + L.w);
    uint8_t *lrank = ws + L.lrank;
    int32_t *dest = reinterpret_cast<int32_t *>(ws + L.dest);
    int32_t *src = reinterpret_cast<int32_t *>(ws + L.src);
    int32_t *hist = reinterpret_cast<int32_t *>(ws + L.hist);
    int32_t *chunk_tot = reinterpret_cast<int32_t *>(ws + L.chunk_tot);
    int32_t *chunk_base = reinterpret_cast<int32_t *>(ws + L.chunk_base);
    const bool chunked = L.NB > kScanChunk;
    int32_t *counts = reinterpret_cast<int32_t *>(ws + L.counts);
    int32_t *slot_cnt = reinterpret_cast<int32_t *>(ws + L.slot_cnt);
    int32_t *slot_off = reinterpret_cast<int32_t *>(ws + L.slot_off);
    int32_t *mt_start = reinterpret_cast<int32_t *>(ws + L.mt_start);
    int32_t *order = reinterpret_cast<int32_t *>(ws + L.order);
    const bool packed = a->w_gateup_packed && a->w_down_packed;
    const tile_choice tiles = tiles_for(plan, layer, rank, a, packed);
    const int32_t *tables = static_cast<const int32_t *>(a->tables);

    // 0 gating network, unless the scores are handed in
    const float *logits = a->logits;
    if (own_gate && a->T > 0) {
        ScopedEvent ev(CRAFT_K_GATE, s);
        float *own = reinterpret_cast<float *>(ws + L.gate_logits);
        RouterArgs ga{a->dtype, a->x, a->w_router, a->T, a->H, E, own, cached_num_cu(),
                      L.gate_ws_bytes ? reinterpret_cast<float *>(ws + L.gate_ws) : nullptr, 1};
        if (launch_router_logits(ga, s) != hipSuccess) return CRAFT_EHIP;
        logits = own;
    }
    // 1 route (+ per-block ranks and counts); user copies of ids / weights are written by the
    // same kernel when asked for, so route straight into them and alias the workspace views
    int32_t *ids_out = a->ids ? a->ids : ids;
    float *w_out = a->topk_w ? a->topk_w : w;
    {
        ScopedEvent ev(CRAFT_K_ROUTE, s);
        RouteArgs ra{logits, a->T, E, a->k, a->renormalize ? 1 : 0, ids_out, w_out, lrank, hist, ctrl};
        if (launch_route(ra, s) != hipSuccess) return CRAFT_EHIP;
    }
    // 2 per-expert totals, slot offsets, tile table
    {
        ScopedEvent ev(CRAFT_K_SCAN, s);
        ScanArgs sa{hist, chunk_tot, chunk_base, (int32_t)L.NB, E, tables, S, s_lo, s_hi, L.max_rows,
                    counts, slot_cnt, slot_off, ctrl, a->counts, a->slot_cnt, a->slot_off};
        if (launch_scan(sa, s) != hipSuccess) return CRAFT_EHIP;
    }
    // 3 dispatch permutation (and, beside it, the tile tables of the two GEMMs)
    {
        ScopedEvent ev(CRAFT_K_DISPATCH, s);
        DispatchArgs da{ids_out, lrank, hist, chunked ? chunk_base : nullptr, a->T, a->k, E, tables, slot_off, dest, src,
                        a->dest, a->src, slot_cnt, s_lo, s_hi, tiles.frags[0], tiles.frags[1],
                        tiles.riders[0] ? (a->I + 127) / 128 : 0, tiles.riders[1] ? (a->H + 255) / 256 : 0,
                        mt_start, order, ctrl};
        if (launch_dispatch(da, s) != hipSuccess) return CRAFT_EHIP;
    }
    // 4 grouped FFN
    FfnArgs fa{a->dtype, a->H, a->I, a->k, s_lo, nslots, a->x, src, slot_off, mt_start, order, ctrl,
               a->w_gate, a->w_up, a->w_down, a->w_gateup_packed, a->w_down_packed,
               ws + L.act, ws + L.y, L.max_rows, cached_num_cu(), a->weight_format == CRAFT_W_E4M3 ? 1 : 0,
               tiles.frags[0], tiles.frags[1]};
    if (a->T > 0) {
        {
            ScopedEvent ev(CRAFT_K_GATEUP, s);
            if ((packed ? launch_gateup_packed(fa, s) : launch_gateup(fa, s)) != hipSuccess)
                return CRAFT_EHIP;
        }
        {
            ScopedEvent ev(CRAFT_K_DOWN, s);
            if ((packed ? launch_down_packed(fa, s) : launch_down(fa, s)) != hipSuccess)
                return CRAFT_EHIP;
        }
    }
    // 5 combine
    {
        ScopedEvent ev(CRAFT_K_COMBINE, s);
        CombineArgs ca{a->dtype, a->T, a->k, a->H, ws + L.y, dest, w_out, slot_off, s_lo, s_hi, ctrl, a->out};
        if (launch_combine(ca, s) != hipSuccess) return CRAFT_EHIP;
    }
    return CRAFT_OK;
}

}  // namespace

extern "C" {

craft_status craft_moe_rank_forward(const craft_plan_t *plan, int32_t layer, int32_t rank,
                                    const craft_fwd_args *a, void *stream) {
    craft_status st = check_fwd(plan, layer, rank, a);
    if (st != CRAFT_OK) return st;
    return forward_on(plan, layer, rank, a, a->workspace, a->workspace_bytes, stream);
}

craft_status craft_moe_rank_forward_static(const craft_plan_t *plan, int32_t layer, int32_t rank,
                                           const craft_fwd_args *a, void *stream) {
    craft_status st = check_fwd(plan, layer, rank, a);
    if (st != CRAFT_OK) return st;
    // sizes first (host arithmetic only): a request that does not fit is refused before any
    // device is touched
    const craft_layer_plan &lp = plan->layers[layer];
    const int32_t nslots = lp.rank_slot_off[rank + 1] - lp.rank_slot_off[rank];
    const Layout L = make_layout(a->T, a->k, plan->E, (int32_t)lp.slot_expert.size(), nslots, a->H, a->I,
                                 a->dtype, a->max_rows, a->logits == nullptr);
    if (L.total > kStaticScratchBytes) return CRAFT_EINFEASIBLE;
    void *ws = nullptr;
    st = static_scratch(&ws);
    if (st != CRAFT_OK) return st;
    return forward_on(plan, layer, rank, a, ws, kStaticScratchBytes, stream);
}

craft_status craft_moe_rank_forward_tiles(const craft_plan_t *plan, int32_t layer, int32_t rank,
                                          const craft_fwd_args *a, int32_t *rows_gateup,
                                          int32_t *rows_down, int32_t *riders_gateup,
                                          int32_t *riders_down) {
    craft_status st = check_fwd(plan, layer, rank, a);
    if (st != CRAFT_OK) return st;
    const bool packed = a->w_gateup_packed && a->w_down_packed;
    const tile_choice c = tiles_for(plan, layer, rank, a, packed);
    if (rows_gateup) *rows_gateup = 32 * std::abs(c.frags[0]);
    if (rows_down) *rows_down = 32 * std::abs(c.frags[1]);
    if (riders_gateup) *riders_gateup = c.riders[0] ? 1 : 0;
    if (riders_down) *riders_down = c.riders[1] ? 1 : 0;
    return CRAFT_OK;
}

craft_status craft_moe_rank_forward_result(const void *workspace, int64_t *rows, int32_t *overflow) {
    if (!workspace) return CRAFT_EINVAL;
    int32_t ctrl[4];
    if (hipMemcpy(ctrl, workspace, sizeof(ctrl), hipMemcpyDeviceToHost) != hipSuccess) return CRAFT_EHIP;
    if (rows) *rows = ctrl[CTRL_ROWS];
    if (overflow) *overflow = ctrl[CTRL_OVERFLOW];
    return CRAFT_OK;
}

craft_status craft_probe_copy(const void *src, void *dst, int64_t bytes, void *stream) {
    if (bytes < 0 || bytes % 16) return CRAFT_EINVAL;
    if (bytes == 0) return CRAFT_OK;
    if (!src || !dst || !aligned(src, 16) || !aligned(dst, 16)) return CRAFT_EINVAL;
    return launch_probe_copy(src, dst, bytes, cached_num_cu(), as_stream(stream)) == hipSuccess ? CRAFT_OK
                                                                                                 : CRAFT_EHIP;
}

craft_status craft_probe_read(const void *src, int64_t bytes, int32_t passes, int32_t blocks, uint32_t *sink,
                              double *bytes_read, void *stream) {
    if (bytes <= 0 || bytes % (32 << 10) || passes <= 0 || blocks < 0 || blocks > (1 << 20)) return CRAFT_EINVAL;
    if (!src || !sink || !aligned(src, 16) || !aligned(sink, 4)) return CRAFT_EINVAL;
    if (blocks == 0) blocks = 8 * cached_num_cu();
    if (bytes_read) *bytes_read = (double)blocks * (double)passes * (double)bytes;
    return launch_probe_read(src, bytes, passes, blocks, sink, as_stream(stream)) == hipSuccess ? CRAFT_OK
                                                                                                 : CRAFT_EHIP;
}

craft_status craft_probe_mfma_bf16(int32_t blocks, int32_t iters, float *sink, double *flops, void *stream) {
    if (blocks < 0 || blocks > (1 << 20) || iters <= 0 || !sink || !aligned(sink, 4)) return CRAFT_EINVAL;
    if (blocks == 0) blocks = 2 * cached_num_cu();
    if (flops) *flops = (double)blocks * 4.0 * (double)iters * 4.0 * 2.0 * 32.0 * 32.0 * 16.0;
    return launch_probe_mfma(blocks, iters, sink, as_stream(stream)) == hipSuccess ? CRAFT_OK : CRAFT_EHIP;
}

craft_status craft_probe_mfma_operands(int32_t shape, int32_t data, int32_t blocks, int32_t iters, float *sink,
                                       double *flops, void *stream) {
    if (shape < 0 || shape > 1 || data < 0 || data > 2) return CRAFT_EINVAL;
    if (blocks < 0 || blocks > (1 << 20) || iters <= 0 || !sink || !aligned(sink, 4)) return CRAFT_EINVAL;
    if (blocks == 0) blocks = cached_num_cu();
    // per wave and iteration: two steps of 2 x 8 products of 32 x 32 x 16
    if (flops) *flops = (double)blocks * 4.0 * (double)iters * 32.0 * 2.0 * 32.0 * 32.0 * 16.0;
    return launch_probe_mfma_operands(shape, data, blocks, iters, sink, as_stream(stream)) == hipSuccess ? CRAFT_OK
                                                                                                        : CRAFT_EHIP;
}

craft_status craft_timing_enable(int32_t level, int32_t max_forwards) {
    if (level < 0 || level > 2 || max_forwards < 0) return CRAFT_EINVAL;
    Timing &t = g_timing;
    std::lock_guard<std::mutex> lk(t.mu);
    const size_t pairs = level == 0 ? 0 : (size_t)max_forwards * (level == 1 ? 1 : CRAFT_K_COUNT);
    while (t.ev.size() < pairs * 2) {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) return CRAFT_EHIP;
        t.ev.push_back(e);
    }
    t.kind.assign(t.ev.size() / 2, 0);
    t.used = 0;
    t.level = level;
    return CRAFT_OK;
}

craft_status craft_timing_read(double ms[CRAFT_K_COUNT], int64_t launches[CRAFT_K_COUNT]) {
    if (!ms || !launches) return CRAFT_EINVAL;
    Timing &t = g_timing;
    std::lock_guard<std::mutex> lk(t.mu);
    for (int i = 0; i < CRAFT_K_COUNT; ++i) { ms[i] = 0.0; launches[i] = 0; }
    for (size_t i = 0; i < t.used; ++i) {
        if (hipEventSynchronize(t.ev[2 * i + 1]) != hipSuccess) return CRAFT_EHIP;
        float d = 0.0f;
        if (hipEventElapsedTime(&d, t.ev[2 * i], t.ev[2 * i + 1]) != hipSuccess) return CRAFT_EHIP;
        ms[t.kind[i]] += d;
        launches[t.kind[i]] += 1;
    }
    t.used = 0;
    return CRAFT_OK;
}

}  // extern "C"
