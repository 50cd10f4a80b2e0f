// Internal layout of the plan object and of the per-rank device tables.
#pragma once

#include <array>
#include <atomic>
#include <cstdint>
#include <map>
#include <memory>
#include <mutex>
#include <utility>
#include <vector>

#include "craft.h"

struct craft_layer_plan {
    int32_t n_replicas = 0;
    std::vector<int32_t> copies;         // [E]
    std::vector<int32_t> slot_expert;    // [S]
    std::vector<int32_t> rank_slot_off;  // [D+1]
    std::vector<int64_t> rank_load;      // [D]
    std::vector<int64_t> expert_load;    // [E] profiled load summed over batches
    int64_t est_max_rank_load = 0;
    double est_balancedness = 1.0;
};

// A device buffer holding the tables of one (layer, rank), as craft_plan_tables_upload filled
// it.  Nodes are only ever added (a buffer that is filled again for another rank has its old
// node blanked), so a forward finds its buffer by walking the list without a lock.
struct craft_table_reg {
    std::atomic<const void *> dev;
    craft_table_reg *next;
    int32_t layer, rank;                  // whose list the node is in
};

// FFN tile choice made for one (T, k, H, I): for gate/up and down, the fragments per row-tile
// (negative: shared evenly) and whether cold slots ride along with busy tiles.
struct craft_tile_choice {
    int64_t T;
    int32_t k, H, I;
    int32_t frags[2];
    bool riders[2];
    craft_tile_choice *next;
};

// What the plan keeps per (layer, rank) for the forwards: written under `mu` (uploads, the
// first forward of a new shape), read lock-free.
struct craft_rank_state {
    std::mutex mu;
    std::vector<int32_t> host_tables;              // built at the first upload, never changed after
    std::atomic<craft_table_reg *> regs{nullptr};
    std::atomic<craft_tile_choice *> tiles{nullptr};
    ~craft_rank_state() {
        for (craft_table_reg *r = regs.load(); r;) { craft_table_reg *n = r->next; delete r; r = n; }
        for (craft_tile_choice *t = tiles.load(); t;) { craft_tile_choice *n = t->next; delete t; t = n; }
    }
};

struct craft_plan {
    int32_t L = 0, E = 0, D = 0, gpus_per_node = 0;
    std::vector<craft_layer_plan> layers;
    std::vector<int32_t> order;          // objective 0: layer that received each replica
    // objective 1: Alg. 1's benefit matrix and what the allocation made of it
    std::vector<int32_t> benefit_counts; // candidate replica counts 1, 2, 4, ..
    std::vector<double> benefit_base;    // [L] placement-only mean balancedness
    std::vector<double> benefit_gain;    // [K][L] mean balancedness gain at each count
    double total_gain = 0.0;             // sum of the gains of the counts chosen
    int32_t auto_R = 0;                  // replication factor picked in automatic mode
    std::unique_ptr<craft_rank_state[]> ranks;     // [L * D]
    std::mutex reg_mutex;                // uploads only: which node a device buffer belongs to
    std::map<const void *, craft_table_reg *> reg_of;
    craft_rank_state &state(int32_t layer, int32_t rank) const { return ranks[(size_t)layer * D + rank]; }
};

// Device tables of one (layer, rank): a header followed by int32 arrays, all offsets in
// int32 units from the start of the buffer.
//   copies      [E]    copies of expert e
//   efirst      [E+1]  eslots[efirst[e] + q] = slot holding copy q of expert e
//   eslots      [S]
//   slot_expert [S]
//   slot_copy   [S]    which copy of its expert the slot is
struct craft_tables_header {
    int32_t reserved;
    int32_t E, S, s_lo, s_hi;
    int32_t off_copies, off_efirst, off_eslots, off_slot_expert, off_slot_copy;
    int32_t total_words;
    int32_t pad;
};

size_t craft_tables_words(int32_t E, int32_t S);
void craft_tables_build(const craft_layer_plan &lp, int32_t E, int32_t rank, int32_t *buf);
