"""Builds one synthetic case end to end on the CPU checker side (profiling loads, plan,
evaluation batch, heaviest rank) for the GPU parity tests.  The plan comes from the
library's host planner and is asserted equal to the checker's."""
from __future__ import annotations

import numpy as np

import oracle
from oracle import plan_oracle as po
from paper_2603_28768_amd import binding, synth


class Case:
    def __init__(self, cfg: synth.LayerConfig, plan=None, layer: int = 0, pop=None, w8: bool = False):
        """Without `plan`: a one-layer plan is made from this config's profiling batches.
        With `plan` (and the layer's popularity `pop`): the evaluation batch of layer
        `layer` of a multi-layer plan made elsewhere."""
        self.cfg = cfg
        self.w8 = w8                      # expert weights stored as E4M3 codes with row scales
        self.layer_index = layer
        self.pop = synth.layer_popularity(cfg, layer) if pop is None else pop
        if plan is None:
            W = np.zeros((cfg.profile_batches, 1, cfg.E), dtype=np.int64)
            for b in range(cfg.profile_batches):
                ids, _ = oracle.route(synth.router_logits(cfg, self.pop, "profile", b), cfg.k)
                W[b, 0] = oracle.expert_load(ids[None], cfg.E, max(cfg.T, 1))[0, 0]
            self.W = W
            plan = binding.Plan(W, cfg.D, cfg.replica_slots, gpus_per_node=cfg.gpus_per_node)
            ref = po.make_plan(W.tolist(), cfg.D, None, cfg.replica_slots)
            lay = plan.layer(0)
            assert lay["slot_expert"].tolist() == ref["layers"][0]["slot_expert"]
            assert lay["rank_slot_off"].tolist() == ref["layers"][0]["rank_slot_off"]
        self.plan = plan
        self.layer = self.plan.layer(layer)
        self.slot_expert = self.layer["slot_expert"]
        self.rank_slot_off = self.layer["rank_slot_off"]
        self.logits = synth.router_logits(cfg, self.pop, "eval", layer=layer)
        self.x = synth.activations(cfg, layer=layer)
        self.ids, self.w = oracle.route(self.logits, cfg.k)
        self.dest, self.src, self.slot_cnt, self.slot_off = oracle.dispatch(
            self.ids, cfg.E, self.slot_expert)
        self.rows = po.realized_rank_rows(self.slot_cnt.tolist(), self.rank_slot_off.tolist())
        self.heaviest = po.heaviest_rank(self.rows)
        self._wcache = {}

    def weights_of(self, e: int):
        """What the checker multiplies with: the synthetic weights, or with w8 what their 8-bit
        storage decodes to (quantised by the checker itself)."""
        if e not in self._wcache:
            w = synth.expert_weights(self.cfg, e, self.layer_index)
            if self.w8:
                w = tuple(oracle.dequantize_e4m3(*oracle.quantize_e4m3(m)) for m in w)
            self._wcache[e] = w
        return self._wcache[e]

    def rank_slots(self, rank: int):
        return [int(e) for e in self.slot_expert[self.rank_slot_off[rank]:self.rank_slot_off[rank + 1]]]

    def oracle_rank(self, rank: int, tokens=None) -> dict:
        return oracle.rank_forward(self.x, self.logits, self.cfg.k, self.slot_expert,
                                   self.rank_slot_off, rank, self.weights_of, True, tokens)

    def gpu_rank(self, rank: int, max_rows: int = 0, debug: bool = True, device="cuda:0",
                 packed: bool = False, w_router=None):
        """(RankForward, x_dev, logits_dev) with this rank's weights resident; packed=True
        re-orders the weights with craft_pack_weights and runs the weight-streaming kernels."""
        import torch
        cfg = self.cfg
        wg, wu, wd, pk = [], [], [], []
        dev_cache, pack_cache = {}, {}
        for e in self.rank_slots(rank):
            if e not in dev_cache:
                raw = synth.expert_weights(cfg, e, self.layer_index)       # the library quantises itself
                dev_cache[e] = tuple(binding.to_device(m, cfg.dtype, device) for m in raw)
                if packed:
                    pack_cache[e] = (binding.pack_weights_e4m3 if self.w8 else binding.pack_weights)(*dev_cache[e])
            g, u, d = dev_cache[e]
            wg.append(g); wu.append(u); wd.append(d)
            if packed:
                pk.append(pack_cache[e])
        fwd = binding.RankForward(self.plan, self.layer_index, rank, cfg.dtype, cfg.T, cfg.H, cfg.I, cfg.k,
                                  wg, wu, wd, True, max_rows, device, want_debug_outputs=debug,
                                  packed=pk if packed else None,
                                  weight_format=binding.CRAFT_W_E4M3 if (packed and self.w8) else 0,
                                  w_router=w_router)
        x = binding.to_device(self.x, cfg.dtype, device)
        logits = torch.from_numpy(self.logits).to(device)
        return fwd, x, logits
