#!/usr/bin/env python3
"""Benchmark of the SAGE tree-verify hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input:
  a1  sage_entropy_topk   on the step's draft logits row(s)            -> confidence, renormalised top-k
  a2  sage_build_tree     from that distribution                       -> the tree the NEXT step verifies (lookahead)
  a3  sage_tree_attention once per layer, on the tree built one step ago
  a1' sage_entropy_topk   k = 1 over the per-node target logits         -> the target's greedy token per node
  a4  sage_verify_accept
All inputs are resident in HBM before the timed region; logits and query/tree inputs cycle through one input set per
step of the configuration, the KV cache through enough sets that consecutive steps do not find it in L2 / Infinity
Cache.  The timed region is a HIP graph of the requested steps, replayed until at least a few milliseconds have been
timed; every graph is first checked bit for bit against eager execution of the same steps.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 MFMA rate
MAX_NODES = 64
MIN_TIMED_MS = 5.0              # the timed region is stretched to at least this by replaying the captured steps
# HBM bytes of one sage_tree_attention call (main kernel + split merge) per workload, from the rocprofv3 FETCH_SIZE /
# WRITE_SIZE runs summarised in profiles/tree_attention_hbm_traffic_by_workload.md (scaled by the counters' readings
# for a 64 MiB copy; the summary states the commands, the tree sizes and the split counts they were taken at).
MEASURED_TRAFFIC_BYTES = {"c2": 26.88e6, "c3": 82.92e6, "c4": 265.17e6, "c5": 172.61e6}
TRAFFIC_SPLITS = {"c2": "22 KV splits per KV head (65 tiles in splits of 3)",
                  "c3": "29 KV splits per KV head (257 tiles in splits of 9); 15 + 15 for trees of more than 32 nodes",
                  "c4": "256 ranges over all sequences and KV heads (batched decomposition)",
                  "c5": "16 KV splits per column group, two column groups (513 tiles in splits of 33)"}

# Trees of the 80-layer configuration are asked to have 64 nodes every step.  With the paper's own parameters the
# rule never grows a tree that large, so that workload plants a geometric top-64 distribution (ratio 1/2) in the
# draft row and builds with a wide/deep parameter set, for which the rule saturates the 64-node cap.
C5_TREE = dict(d_min=31, d_max=31, w_min=16, w_max=16, k=64, n_max=64)
WORKLOAD_TEXT = {
    "toy": "Toy fp32, 4/1 heads d64, KV 256, vocab 1024",
    "c2": "one layer at the 72B shape (64/8 heads, d128, bf16), KV 4096, vocab 152064, adaptive tree <= 64 nodes, batch 1",
    "c3": "72B shape (64/8 heads, d128, bf16), one layer, video-length KV 16384, 256 steps of AR(1) entropy-driven trees, vocab 152064, batch 1",
    "c4": "72B shape, batch 8, ragged KV 2048..12288, ragged trees, vocab 152064",
    "c5": "80-layer attention stack at the 72B shape, KV 32768 per layer, 64-node tree, vocab 152064"}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="c3", choices=["toy", "c2", "c3", "c4", "c5"],
                    help="the workload `value` and `roofline` are measured on (default: the long-KV single-layer configuration)")
    ap.add_argument("--slots", type=int, default=None, help="number of input sets (default: the configuration's step count)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the other workloads and the closed-loop, output-projection, top-k and draft-side measurements")
    ap.add_argument("--all-schedules", action="store_true",
                    help="also time the headline workload with planning on a second stream and as launches of its own")
    ap.add_argument("--only", default=None, choices=["attention", "closed_loop", "lm_head", "entropy_topk", "draft_side"],
                    help="run one measurement alone and print its JSON (for profiling it); `attention` = graph replays of the "
                         "sage_tree_attention calls of --workload")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--eager", action="store_true", help="time the steps eagerly instead of as HIP-graph replays")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run plain 64 MiB device copies, the known-size reference for rocprofv3 FETCH_SIZE/WRITE_SIZE")
    return ap.parse_args()


class Workload:
    """Device-resident synthetic inputs of one configuration plus every output/scratch buffer of a step."""

    def __init__(self, name: str, slots: int | None = None, fused: bool = True, overlap: bool = False, carry: bool = False,
                 layers: int | None = None, keep_layer_outputs: bool = False):
        import numpy as np
        import torch
        from paper_2602_00523_amd import sage, workloads as wl
        self.torch, self.sage, self.wl, self.np = torch, sage, wl, np
        cfg = wl.CONFIGS[name]
        self.name, self.cfg = name, cfg
        dev = "cuda:0"
        self.dtype = torch.float32 if cfg["dtype"] == "f32" else torch.bfloat16
        B, Hq, Hkv, d, V = cfg["B"], cfg["Hq"], cfg["Hkv"], cfg["d"], cfg["vocab"]
        self.B, self.Hq, self.Hkv, self.d, self.V = B, Hq, Hkv, d, V
        self.layers = cfg["layers"] if layers is None else layers
        self.tree_prm = dict(C5_TREE) if name == "c5" else dict(cfg["tree"])
        self.k = self.tree_prm["k"]
        if isinstance(cfg["kv_len"], tuple):
            self.kv_lens = wl.ragged_kv_lens(wl.seed_for(name, 0, 3), B, *cfg["kv_len"])
        else:
            self.kv_lens = np.full(B, cfg["kv_len"], np.int32)
        self.max_len = int(self.kv_lens.max())
        total = int(self.kv_lens.sum())
        esz = 4 if cfg["dtype"] == "f32" else 2
        kv_bytes = 2 * total * Hkv * d * esz * self.layers
        logit_bytes = (B * MAX_NODES + B) * V * esz
        # One input set (draft row, per-node target rows, Q, tree K/V) per step of the configuration, so that the tree
        # sequence is the configuration's own (c3: all 256 steps of its AR(1) entropy process); the KV cache rotates
        # through its own, smaller number of sets: more than 512 MB in total, so that no step finds its cache on chip
        # (a multi-layer stack already walks through that much within a step).
        if slots is None:
            slots = max(2, min(cfg["steps"], int(12e9 // max(logit_bytes, 1))))
        self.slots = slots
        self.kv_slots = 1 if kv_bytes > 600e6 else max(1, min(slots, math.ceil(600e6 / max(kv_bytes, 1))))
        gen = torch.Generator(device=dev)
        gen.manual_seed(wl.seed_for(name))

        def randn(*shape):
            return torch.randn(*shape, generator=gen, device=dev, dtype=torch.float32).to(self.dtype)

        kv_start = np.zeros(B, np.int64)
        kv_start[1:] = np.cumsum(self.kv_lens.astype(np.int64))[:-1]
        self.kv_start = torch.from_numpy(kv_start).to(dev)
        self.kv_len = torch.from_numpy(self.kv_lens).to(dev)
        self.Kc = [[randn(total, Hkv, d) for _ in range(self.layers)] for _ in range(self.kv_slots)]
        self.Vc = [[randn(total, Hkv, d) for _ in range(self.layers)] for _ in range(self.kv_slots)]
        self.Q = [randn(B, MAX_NODES, Hq, d) for _ in range(self.slots)]
        self.Kt = [randn(B, MAX_NODES, Hkv, d) for _ in range(self.slots)]
        self.Vt = [randn(B, MAX_NODES, Hkv, d) for _ in range(self.slots)]

        # logits: Gaussian rows scaled toward a per-step target entropy; per-node target logits = draft row + noise
        if name == "toy":
            scales = 1.0 / wl.toy_temperatures(self.slots * B)
        else:
            scales = np.array([wl.scale_for_entropy(h) for h in wl.entropy_targets(name, self.slots * B)])
        self.draft, self.target = [], []
        rows, betas = [], []
        for s in range(self.slots):
            z = torch.randn(B, V, generator=gen, device=dev, dtype=torch.float32)
            beta = torch.tensor(scales[s * B:(s + 1) * B], device=dev, dtype=torch.float32)[:, None]
            row = z * beta
            if name == "c5":                    # planted geometric top-64 (see C5_TREE)
                row = row * 0.05 - 60.0
                pos = torch.randperm(V, generator=gen, device=dev)[:64]
                row[:, pos] = -math.log(2.0) * torch.arange(64, device=dev, dtype=torch.float32)
                beta = torch.ones_like(beta)
            rows.append(row)
            betas.append(beta)
            self.draft.append(row.to(self.dtype).contiguous())
            del z
        # The tree verified with input set s was planned one step earlier from the draft row of set s-1 and carries
        # that row's candidates as node tokens, so the target logits of set s are that row plus noise: confident
        # (low-entropy) draft rows are then accepted deep, uncertain ones shallow.
        for s in range(self.slots):
            row, beta = rows[(s - 1) % self.slots], betas[(s - 1) % self.slots]
            noise = torch.randn(B, MAX_NODES, V, generator=gen, device=dev, dtype=torch.float32)
            tgt = (row[:, None, :] + 0.5 * beta[:, None, :] * noise).reshape(B * MAX_NODES, V)
            self.target.append(tgt.to(self.dtype).contiguous())
            del noise, tgt
        del rows, betas

        f32 = lambda *s: torch.zeros(*s, device=dev, dtype=torch.float32)
        i32 = lambda *s: torch.zeros(*s, device=dev, dtype=torch.int32)
        k = self.k
        self.H, self.Hk, self.alpha = f32(B), f32(B), f32(B)
        self.idx, self.prob, self.renorm = i32(B, k), f32(B, k), f32(B, k)
        self.ws1 = torch.empty(sage.sage_entropy_topk_workspace_bytes(B, V, k), device=dev, dtype=torch.uint8)
        self.tree = [dict(n_nodes=torch.ones(B, device=dev, dtype=torch.int32), parent=i32(B, MAX_NODES) - 1,
                          depth=i32(B, MAX_NODES), rank=i32(B, MAX_NODES) - 1,
                          anc_mask=torch.ones(B, MAX_NODES, device=dev, dtype=torch.int64),
                          node_token=i32(B, MAX_NODES) - 1) for _ in range(2)]
        self.prm = sage.tree_params(**self.tree_prm)
        self.O = torch.zeros(B, MAX_NODES, Hq, d, device=dev, dtype=self.dtype)
        # tests keep every layer's output; the benchmark, like a model, lets each layer overwrite the last one's
        self.O_layers = [torch.zeros_like(self.O) for _ in range(self.layers)] if keep_layer_outputs else None
        code = sage.F32 if self.dtype == torch.float32 else sage.BF16
        self.ws3 = torch.empty(sage.sage_tree_attention_workspace_bytes(code, B, Hq, Hkv, d, self.max_len), device=dev,
                               dtype=torch.uint8)
        self.tH, self.tHk, self.talpha = f32(B * MAX_NODES), f32(B * MAX_NODES), f32(B * MAX_NODES)
        self.tgt_idx = i32(B * MAX_NODES, 1)
        self.ws1t = torch.empty(sage.sage_entropy_topk_workspace_bytes(B * MAX_NODES, V, 1), device=dev, dtype=torch.uint8)
        self.path_cap = self.tree_prm["d_max"] + 1
        self.acc_len, self.best = i32(B), i32(B)
        self.path, self.out_tok = i32(B, self.path_cap), i32(B, self.path_cap)
        self.scale = 1.0 / math.sqrt(d)
        self.cur = 0
        self.step_no = 0
        self.fused = fused
        # Sec. 3.2 lookahead: the tree planned from this step's draft row is verified in the NEXT step, so planning
        # (a1 + a2) and verification (a3, a1', a4) of a step touch disjoint data; with `overlap` they run on two streams
        # that fork at the start of a step and join at its end.
        self.overlap = overlap
        self.plan_stream = torch.cuda.Stream() if overlap else None
        # The other way to take planning off the step's chain of launches: its second half (merge + tree rule) rides in
        # the launch of the first layer's attention (sage_tree_attention_with_plan), everything on one stream.
        self.carry = carry
        assert not (carry and (overlap or not fused))
        # With carried planning, what is left of planning on the chain is the slice pass over the draft row.  It depends
        # on nothing the verification produces, so inside a run of steps (run_steps) the pass for the NEXT step shares
        # the launch of this step's target-row pass (sage_entropy_topk_slices_pair).  A run starts with the pass as a
        # launch of its own and ends with a plain target-row pass, so a captured graph is self-contained.
        self.pair = carry
        self.slices_for = -1                         # step number whose draft slices the last pair launch produced
        self.verify_first = True                     # enqueue the verification branch first (measured 2 % faster)
        self._prepare()
        torch.cuda.synchronize()

    # -- the five calls of one step, marshalled once per (input set, layer, tree buffer) ------------------------
    def _prepare(self, stream=None):
        """Marshal every call of a step once for the given stream (None = the current stream)."""
        sg = self.sage
        V = self.cfg["vocab"]
        pstream = self.plan_stream if self.overlap else stream
        if self.fused:                               # the per-row top-k pass runs inside the call that consumes it
            self.c_a1 = [sg.prepare("sage_entropy_topk_slices", self.draft[s], self.k, self.ws1, stream=pstream)
                         for s in range(self.slots)]
        else:
            self.c_a1 = [sg.prepare("sage_entropy_topk", self.draft[s], self.k, self.H, self.idx, self.prob, self.renorm,
                                    self.Hk, self.alpha, self.ws1, stream=pstream) for s in range(self.slots)]
        self.c_a2, self.c_a3, self.c_a1t, self.c_a4, self.c_a3p, self.c_pair = [], [], [], [], [], []
        for cur in range(2):
            t, nxt = self.tree[cur], self.tree[cur ^ 1]
            if self.carry:
                self.c_a3p.append([sg.prepare("sage_tree_attention_with_plan", self.Q[s], self.Kc[s % self.kv_slots][0],
                                              self.Vc[s % self.kv_slots][0], self.Kt[s], self.Vt[s],
                                              self.O if self.O_layers is None else self.O_layers[0], self.kv_start,
                                              self.kv_len, self.max_len, self.Hkv * self.d, self.d, t["anc_mask"], t["n_nodes"],
                                              self.scale, self.ws3, self.ws1, V, self.prm, self.H, self.idx, self.prob,
                                              self.renorm, self.Hk, self.alpha, nxt["n_nodes"], nxt["parent"], nxt["depth"],
                                              nxt["rank"], nxt["anc_mask"], None, nxt["node_token"], stream=stream)
                                   for s in range(self.slots)])
            if self.fused:
                self.c_a2.append(sg.prepare("sage_build_tree_from_slices", self.ws1, V, self.prm, self.H, self.idx, self.prob,
                                            self.renorm, self.Hk, self.alpha, nxt["n_nodes"], nxt["parent"], nxt["depth"],
                                            nxt["rank"], nxt["anc_mask"], None, nxt["node_token"], stream=pstream))
            else:
                self.c_a2.append(sg.prepare("sage_build_tree", self.renorm, self.alpha, self.prm, nxt["n_nodes"],
                                            nxt["parent"], nxt["depth"], nxt["rank"], nxt["anc_mask"], None, self.idx,
                                            nxt["node_token"], stream=pstream))
            self.c_a3.append([[sg.prepare("sage_tree_attention", self.Q[s], self.Kc[s % self.kv_slots][layer],
                                          self.Vc[s % self.kv_slots][layer], self.Kt[s], self.Vt[s],
                                          self.O if self.O_layers is None else self.O_layers[layer], self.kv_start,
                                          self.kv_len, self.max_len, self.Hkv * self.d, self.d, t["anc_mask"], t["n_nodes"],
                                          self.scale, self.ws3, stream=stream) for layer in range(self.layers)]
                              for s in range(self.slots)])
            if self.fused:
                self.c_a1t.append([sg.prepare("sage_entropy_topk_slices", self.target[s], 1, self.ws1t, t["n_nodes"], MAX_NODES,
                                              stream=stream) for s in range(self.slots)])
                self.c_a4.append(sg.prepare("sage_verify_accept_from_slices", self.ws1t, V, t["node_token"], t["parent"],
                                            t["depth"], t["anc_mask"], t["n_nodes"], self.path_cap, self.tH, self.tgt_idx,
                                            self.acc_len, self.best, self.path, self.out_tok, stream=stream))
            else:
                self.c_a1t.append([sg.prepare("sage_entropy_topk", self.target[s], 1, self.tH, self.tgt_idx, None, None,
                                              self.tHk, self.talpha, self.ws1t, t["n_nodes"], MAX_NODES, stream=stream)
                                   for s in range(self.slots)])
                self.c_a4.append(sg.prepare("sage_verify_accept", t["node_token"], self.tgt_idx, t["parent"], t["depth"],
                                            t["anc_mask"], t["n_nodes"], self.path_cap, self.acc_len, self.best, self.path,
                                            self.out_tok, stream=stream))
            if self.carry:
                self.c_pair.append([sg.prepare("sage_entropy_topk_slices_pair", self.target[s], t["n_nodes"], MAX_NODES, self.ws1t,
                                               self.draft[(s + 1) % self.slots], self.k, self.ws1, stream=stream)
                                    for s in range(self.slots)])

    def draft_confidence(self, s):
        self.c_a1[s]()

    def plan_next_tree(self):
        self.c_a2[self.cur]()

    def attention(self, s, layer):
        self.c_a3[self.cur][s][layer]()

    def run_steps(self, n: int):
        """n consecutive steps; inside the run the draft row's slice pass of a step rides in the previous step's
        target-row launch (carried planning only)."""
        self.slices_for = -1
        for i in range(n):
            self.step(last=i == n - 1)

    def step(self, last: bool = True):
        s = self.step_no % self.slots
        cur = self.cur
        if self.overlap:                             # fork: the plan branch starts where the main stream stands
            main = self.torch.cuda.current_stream()
            self.plan_stream.wait_stream(main)
        if self.carry:
            if not (self.pair and self.slices_for == self.step_no):
                self.c_a1[s]()                       # (otherwise the previous step's pair launch has left the slices)
            self.c_a3p[cur][s]()                     # first layer's attention with the planning inside its launch
            for call in self.c_a3[cur][s][1:]:
                call()
            if self.pair and not last:               # target rows of this step + draft row of the next in one launch
                self.c_pair[cur][s]()
                self.slices_for = self.step_no + 1
            else:
                self.c_a1t[cur][s]()
            self.c_a4[cur]()
            self.cur ^= 1
            self.step_no += 1
            return
        if not (self.overlap and self.verify_first):
            self.c_a1[s]()
            self.c_a2[cur]()
        for call in self.c_a3[cur][s]:
            call()
        self.c_a1t[cur][s]()
        self.c_a4[cur]()
        if self.overlap and self.verify_first:       # the plan branch is enqueued after the verification branch
            self.c_a1[s]()
            self.c_a2[cur]()
        if self.overlap:                             # join: the next step verifies the tree planned in this one
            main.wait_stream(self.plan_stream)
        self.cur ^= 1
        self.step_no += 1

    def attention_algorithmic_bytes(self, n_nodes_per_seq) -> float:
        """K and V of the cache once, the tree's K/V once, Q in and O out (per layer)."""
        esz = 4 if self.dtype == self.torch.float32 else 2
        kv = 2 * esz * float(self.kv_lens.sum()) * self.Hkv * self.d
        tree = float(sum(n_nodes_per_seq)) * (2 * esz * self.Hkv * self.d + 2 * esz * self.Hq * self.d)
        return kv + tree

    def attention_flops(self, n_nodes_per_seq) -> float:
        return float(sum(4.0 * n * self.Hq * self.d * (int(L) + n) for n, L in zip(n_nodes_per_seq, self.kv_lens)))


def snapshot(w: Workload):
    """What a step leaves behind, with everything the calls do not write blanked out: output rows of nodes past the
    verified tree's size and entries of the planned tree past its size keep whatever an earlier step left there,
    which depends on the steps before and is no part of the state."""
    torch = w.torch
    planned, verified = w.tree[w.cur], w.tree[w.cur ^ 1]      # planned by the last step / verified by it
    node = torch.arange(MAX_NODES, device=w.O.device)[None, :]
    live_v = node < verified["n_nodes"][:, None]
    live_p = node < planned["n_nodes"][:, None]
    outs = w.O_layers if w.O_layers is not None else [w.O]
    state = [torch.where(live_v[:, :, None, None], o, torch.zeros_like(o)) for o in outs]
    state.append(torch.where(live_v.reshape(-1, 1), w.tgt_idx, torch.full_like(w.tgt_idx, -1)))
    state += [x.clone() for x in (w.acc_len, w.best, w.path, w.out_tok, w.alpha, planned["n_nodes"])]
    state += [torch.where(live_p, planned[k], torch.zeros_like(planned[k])) for k in ("parent", "anc_mask", "node_token")]
    return state


def capture_steps(w: Workload, length: int):
    """Record the next `length` steps (an even number: the two tree buffers swap roles every step) as a HIP graph and
    check its replays against eager execution.

    The graph bakes in which input sets and tree buffers its steps use, so every replay runs the same `length` steps
    again, each starting from the tree the previous pass planned last; an eager pass over the same steps does exactly
    the same, and three replays, with eager passes in between, must each land in the eager pass's state bit for bit.
    Returns the graph, or None when capture is unavailable or a replay disagrees.
    """
    torch = w.torch
    assert length % 2 == 0
    start = (w.step_no, w.cur)

    def eager_pass():
        w.step_no, w.cur = start
        w.run_steps(length)

    torch.cuda.synchronize()
    try:
        side = torch.cuda.Stream()
        w._prepare(side)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            eager_pass()                                  # (recorded, not executed)
        w._prepare(None)
        torch.cuda.synchronize()
        eager_pass()
        for _ in range(3):
            eager_pass()
            torch.cuda.synchronize()
            want = snapshot(w)
            graph.replay()
            torch.cuda.synchronize()
            got = snapshot(w)
            if not all(torch.equal(a, b) for a, b in zip(want, got)):
                print("bench.py: graph replay differs from eager execution; timing eagerly", file=sys.stderr)
                return None
        return graph
    except Exception as ex:  # capture unsupported on this stack: time eagerly
        print(f"bench.py: graph capture unavailable ({type(ex).__name__}); timing eagerly", file=sys.stderr)
        w._prepare(None)
        w.step_no, w.cur = start
        return None


def capture_cycle(w: Workload):
    """capture_steps over one whole cycle of the input sets, from a cycle boundary.  Returns (graph, steps per replay)
    or (None, 0)."""
    cycle = w.slots if w.slots % 2 == 0 else 2 * w.slots
    while w.step_no % cycle:
        w.step()
    graph = capture_steps(w, cycle)
    return (graph, cycle) if graph is not None else (None, 0)


def time_steps(w: Workload, steps: int, warmup: int, use_graph: bool = True, min_ms: float = MIN_TIMED_MS):
    """The timed region.  `steps` consecutive steps are captured as one HIP graph (2 * steps when steps is odd, whole
    input-set cycles when steps exceeds a cycle) and the graph is replayed as often as it takes to time at least
    `steps` steps and at least `min_ms` milliseconds.  Returns a dict with the wall time, the number of steps actually
    timed and how they were launched; nothing is labelled a replay that was not one."""
    torch = w.torch
    for _ in range(warmup):
        w.step()
    if w.step_no % 2:
        w.step()
    torch.cuda.synchronize()
    cycle = w.slots if w.slots % 2 == 0 else 2 * w.slots
    if steps >= cycle:
        while w.step_no % cycle:
            w.step()
        length = cycle
    else:
        length = steps if steps % 2 == 0 else 2 * steps
    graph = capture_steps(w, length) if use_graph else None
    torch.cuda.synchronize()
    if graph is None:
        n = max(steps, 1)
        t0 = time.perf_counter()
        w.run_steps(n)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        return dict(wall_s=wall, timed_steps=n, replays=0, steps_per_replay=0, eager_steps=n, launch_mode="eager launches")
    t0 = time.perf_counter()                                    # one untimed-looking probe that is timed on its own
    graph.replay()
    torch.cuda.synchronize()
    probe = max(time.perf_counter() - t0, 1e-6)
    replays = max(math.ceil(steps / length), math.ceil(min_ms * 1e-3 / probe))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(replays):
        graph.replay()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return dict(wall_s=wall, timed_steps=replays * length, replays=replays, steps_per_replay=length, eager_steps=0,
                launch_mode=f"HIP graph replay: {replays} replays of a graph of {length} consecutive steps")


def planned_trees(w: Workload):
    """The tree every input set is verified with in the step sequence (the one planned from the previous set), as
    (mask, count, host sizes) per input set; planning is replayed untimed."""
    torch = w.torch
    masks, counts, sizes = [], [], []
    for s in range(w.slots):
        w.draft_confidence((s - 1) % w.slots)
        w.plan_next_tree()
        torch.cuda.synchronize()
        t = w.tree[w.cur ^ 1]
        masks.append(t["anc_mask"].clone())
        counts.append(t["n_nodes"].clone())
        sizes.append(t["n_nodes"].cpu().numpy().copy())
    return masks, counts, sizes


def time_attention_graph(w: Workload, min_ms: float = 20.0, max_sets: int = 64, eager: bool = False):
    """The sage_tree_attention calls of the step sequence alone, as a HIP graph: input sets in order (at most
    `max_sets` of them), each with the tree that the sequence verifies on it and with the K/V set its step uses,
    every layer; replayed between two HIP events on the capture stream until `min_ms` have been timed.  This is how
    the launches run inside the timed region (graph replay, no host gaps, rotating K/V), and what the per-kernel
    durations of a rocprofv3 trace add up to.  Returns (us per call, tree sizes of the calls)."""
    torch, sg = w.torch, w.sage
    masks, counts, sizes = planned_trees(w)
    sets = list(range(min(w.slots, max_sets)))
    side = torch.cuda.Stream()
    calls = [sg.prepare("sage_tree_attention", w.Q[s], w.Kc[s % w.kv_slots][layer], w.Vc[s % w.kv_slots][layer], w.Kt[s],
                        w.Vt[s], w.O, w.kv_start, w.kv_len, w.max_len, w.Hkv * w.d, w.d, masks[s], counts[s], w.scale,
                        w.ws3, stream=side) for s in sets for layer in range(w.layers)]
    if eager:                                                  # (counter collection wants plain dispatches)
        with torch.cuda.stream(side):
            for c in calls:
                c()
            side.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(side)
            for _ in range(3):
                for c in calls:
                    c()
            e1.record(side)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / (3 * len(calls)), [sizes[s] for s in sets]
    try:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for c in calls:
                c()
    except Exception:
        return None, sizes
    with torch.cuda.stream(side):
        graph.replay()
        side.synchronize()
        t0 = time.perf_counter()
        graph.replay()
        side.synchronize()
        reps = max(2, math.ceil(min_ms * 1e-3 / max(time.perf_counter() - t0, 1e-6)))
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(side)
        for _ in range(reps):
            graph.replay()
        e1.record(side)
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / (reps * len(calls)), [sizes[s] for s in sets]


def attention_roofline(w: Workload, name: str, eager: bool = False):
    """Roofline entry of the sage_tree_attention call at workload `name` (measured live, see time_attention_graph)."""
    us, sized = time_attention_graph(w, eager=eager)
    if us is None:
        return None
    per_bytes = sum(w.attention_algorithmic_bytes(n) for n in sized) / len(sized)
    per_flops = sum(w.attention_flops(n) for n in sized) / len(sized)
    gbps = per_bytes / (us * 1e-6) / 1e9
    tflops = per_flops / (us * 1e-6) / 1e12
    nodes = [int(x) for n in sized for x in n]
    hist = {}
    for x in nodes:
        key = f"{(x - 1) // 8 * 8 + 1}-{(x - 1) // 8 * 8 + 8}"
        hist[key] = hist.get(key, 0) + 1
    # a tree of N nodes has arithmetic intensity N * G flop per byte: past about 310 flop/B (39 nodes at G = 8) the
    # matrix rate, not the HBM rate, is the binding roof
    mfma_bound = per_flops / per_bytes > MFMA_BF16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBPS * 1e9)
    out = {"workload": name, "kernel": "sage_tree_attention (bf16 MFMA kernel + split merge, per layer call)",
           "bound": "mfma" if mfma_bound else "hbm",
           "achieved": tflops if mfma_bound else gbps, "peak": MFMA_BF16_PEAK_TFLOPS if mfma_bound else HBM_PEAK_GBPS,
           "unit": "TFLOP/s" if mfma_bound else "GB/s",
           "frac": (tflops / MFMA_BF16_PEAK_TFLOPS) if mfma_bound else gbps / HBM_PEAK_GBPS,
           "traffic": MEASURED_TRAFFIC_BYTES.get(name),
           "traffic_source": (f"rocprofv3 FETCH_SIZE + WRITE_SIZE per call, profiles/tree_attention_hbm_traffic_by_workload.md, "
                              f"taken at {TRAFFIC_SPLITS[name]}") if name in TRAFFIC_SPLITS else None,
           "avg_launch_us": us,
           "algorithmic_bytes_per_launch": per_bytes, "hbm_GBps": gbps, "hbm_frac": gbps / HBM_PEAK_GBPS,
           "mfma_TFLOPs": tflops, "mfma_frac": tflops / MFMA_BF16_PEAK_TFLOPS,
           "mean_tree_nodes": sum(nodes) / len(nodes), "tree_size_histogram": dict(sorted(hist.items(), key=lambda kv: int(kv[0].split("-")[0]))),
           "calls_timed_per_replay": len(sized) * w.layers,
           "timing": ("HIP events around graph replays of the step sequence's sage_tree_attention calls alone (each input "
                      "set with the tree the sequence verifies on it, K/V sets rotating as in the steps), per call")}
    if w.dtype == w.torch.float32:
        out.update(kernel="sage_tree_attention (fp32 FMA kernel)", note="launch-latency scale: 131 KB per call")
    return out


def cpu_baseline(w: Workload, budget_s: float):
    """The oracle, untouched, timed on the host cores over whole steps of the same workload (bounded sample)."""
    import numpy as np
    import oracle
    torch = w.torch

    def host(t):
        if t.dtype == torch.bfloat16:
            return t.view(torch.int16).cpu().numpy().view(np.uint16)
        return t.cpu().numpy()

    layers_timed = 1
    prm = w.tree_prm
    n_steps, spent, att_spent = 0, 0.0, 0.0
    tree = oracle.build_tree(np.full((w.B, w.k), 1.0 / w.k, np.float32), np.full(w.B, 0.5, np.float32), prm)
    while spent < budget_s and n_steps < 8 * w.slots:        # about budget_s seconds of oracle work, cycling the input sets
        s = n_steps % w.slots
        draft, target = host(w.draft[s]), host(w.target[s])
        Q, Kt, Vt = host(w.Q[s]), host(w.Kt[s]), host(w.Vt[s])
        Kc, Vc = host(w.Kc[s % w.kv_slots][0]), host(w.Vc[s % w.kv_slots][0])
        t0 = time.perf_counter()
        o1 = oracle.entropy_topk(draft, w.k)
        nxt = oracle.build_tree(o1["topk_renorm"].astype(np.float32), o1["alpha"].astype(np.float32), prm, o1["topk_idx"])
        ta = time.perf_counter()
        for _ in range(layers_timed):
            oracle.tree_attention(Q, Kc, Vc, Kt, Vt, w.kv_start.cpu().numpy(), w.kv_lens, w.Hkv * w.d, w.d,
                                  tree["anc_mask"], tree["n_nodes"], w.Hq, w.Hkv, w.d)
        tb = time.perf_counter()
        o1t = oracle.entropy_topk(target, 1, tree["n_nodes"], MAX_NODES)
        tok = np.where(tree["node_token"] < -1, 0, tree["node_token"])
        oracle.verify_accept(tok, o1t["topk_idx"][:, 0].reshape(w.B, MAX_NODES), tree["parent"], tree["depth"],
                             tree["n_nodes"], prm["d_max"] + 1)
        t1 = time.perf_counter()
        att_spent += tb - ta
        spent += (t1 - t0) + (tb - ta) * (w.layers - layers_timed)     # scale the attention leg to all layers
        tree = nxt
        n_steps += 1
    sample = f"{n_steps} whole steps of workload {w.name} (same device inputs copied to the host)"
    if w.layers > layers_timed:
        sample += f"; attention timed on {layers_timed} of {w.layers} layers per step and scaled"
    return dict(value=n_steps / spent, unit="steps/s", cores=oracle.num_threads(), kind="oracle", sample=sample)


def closed_loop(name="c2", steps=512, carry=True):
    """The step with its loop closed on the device: after acceptance the path's K/V rows are committed to the
    cache, the sequence length advances and the acceptance history adapts the maximum depth that the next tree may
    reach (Alg. 1 Phase 3; Sec. 3.3 adaptive history tracking).  One input-set cycle is captured as a HIP graph whose
    replays carry the state (cache, lengths, history, trees) forward; the final state of `steps` replayed steps is
    checked against the same number of eager steps from the same start.  The top-k calls are the fused ones.  With `carry`
    (bf16 workloads) the planning rides in the attention launch and everything runs on one stream; without it, planning
    runs on a second stream beside the verification."""
    import torch
    w = Workload(name, 32)
    carry = carry and w.dtype == torch.bfloat16
    sg, dev = w.sage, "cuda:0"
    B, Hkv, d = w.B, w.Hkv, w.d
    cycle = w.slots if w.slots % 2 == 0 else 2 * w.slots
    steps = max(cycle, steps // cycle * cycle)
    cap = w.max_len + steps * w.path_cap                      # positions per sequence, enough for every step
    Kc = torch.zeros(B * cap, Hkv, d, device=dev, dtype=w.dtype)
    Vc = torch.zeros_like(Kc)
    kv0 = w.kv_start.cpu().numpy()
    for b in range(B):
        L = int(w.kv_lens[b])
        Kc[b * cap:b * cap + L] = w.Kc[0][0][kv0[b]:kv0[b] + L]
        Vc[b * cap:b * cap + L] = w.Vc[0][0][kv0[b]:kv0[b] + L]
    kv_start = torch.arange(B, device=dev, dtype=torch.int64) * cap
    kv_len0 = w.kv_len.clone()
    kv_len = kv_len0.clone()
    window, lo, hi = 10, 2.0, 3.0                             # Sec. 5 "Implementation details"
    hist = torch.zeros(B, window, device=dev, dtype=torch.int32)
    count = torch.zeros(B, device=dev, dtype=torch.int32)
    # two depth-limit arrays: a step's plan and its closing call both read [cur]; the closing call writes [cur ^ 1], so the
    # plan branch, which runs beside it on another stream, never sees a limit change under it
    d_max = [torch.full((B,), w.tree_prm["d_max"], device=dev, dtype=torch.int32) for _ in range(2)]
    code = sg.F32 if w.dtype == torch.float32 else sg.BF16
    ws3 = torch.empty(sg.sage_tree_attention_workspace_bytes(code, B, w.Hq, Hkv, d, cap), device=dev, dtype=torch.uint8)
    tree0 = [{k: v.clone() for k, v in t.items()} for t in w.tree]
    acc_sum = torch.zeros(B, device=dev, dtype=torch.int32)

    plan_stream = torch.cuda.Stream()                         # planning runs beside verification (see Workload)

    def prep(stream):
        V = w.cfg["vocab"]
        c = dict(a1=[sg.prepare("sage_entropy_topk_slices", w.draft[s], w.k, w.ws1, stream=stream if carry else plan_stream)
                     for s in range(w.slots)], a2=[], a3=[], a1t=[], a4=[], commit=[], a3p=[], pair=[])
        for cur in range(2):
            t, nxt = w.tree[cur], w.tree[cur ^ 1]
            if carry:
                c["a3p"].append([sg.prepare("sage_tree_attention_with_plan", w.Q[s], Kc, Vc, w.Kt[s], w.Vt[s], w.O, kv_start,
                                            kv_len, cap, Hkv * d, d, t["anc_mask"], t["n_nodes"], w.scale, ws3, w.ws1, V, w.prm,
                                            w.H, w.idx, w.prob, w.renorm, w.Hk, w.alpha, nxt["n_nodes"], nxt["parent"],
                                            nxt["depth"], nxt["rank"], nxt["anc_mask"], None, nxt["node_token"], stream=stream,
                                            d_max_seq=d_max[cur]) for s in range(w.slots)])
            c["a2"].append(sg.prepare("sage_build_tree_from_slices", w.ws1, V, w.prm, w.H, w.idx, w.prob, w.renorm, w.Hk, w.alpha,
                                      nxt["n_nodes"], nxt["parent"], nxt["depth"], nxt["rank"], nxt["anc_mask"], None,
                                      nxt["node_token"], stream=plan_stream, d_max_seq=d_max[cur]))
            c["a3"].append([sg.prepare("sage_tree_attention", w.Q[s], Kc, Vc, w.Kt[s], w.Vt[s], w.O, kv_start, kv_len, cap,
                                       Hkv * d, d, t["anc_mask"], t["n_nodes"], w.scale, ws3, stream=stream)
                            for s in range(w.slots)])
            c["a1t"].append([sg.prepare("sage_entropy_topk_slices", w.target[s], 1, w.ws1t, t["n_nodes"], MAX_NODES,
                                        stream=stream) for s in range(w.slots)])
            if carry:                                         # ... or with the next step's draft row in the same launch
                c["pair"].append([sg.prepare("sage_entropy_topk_slices_pair", w.target[s], t["n_nodes"], MAX_NODES, w.ws1t,
                                             w.draft[(s + 1) % w.slots], w.k, w.ws1, stream=stream) for s in range(w.slots)])
            # acceptance, commit, advance and history in one launch
            c["a4"].append([sg.prepare("sage_verify_accept_close_from_slices", w.ws1t, V, t["node_token"], t["parent"], t["depth"],
                                       t["anc_mask"], t["n_nodes"], w.path_cap, w.tH, w.tgt_idx, w.acc_len, w.best, w.path,
                                       w.out_tok, w.Kt[s], w.Vt[s], Kc, Vc, kv_start, kv_len, cap, Hkv * d, d, hist, count,
                                       d_max[cur], d_max[cur ^ 1], lo, hi, w.tree_prm["d_min"], w.tree_prm["d_max"],
                                       stream=stream) for s in range(w.slots)])
        return c

    state = dict(cur=0, step=0, slices_for=-1)

    def step(c, last=True):
        s, cur = state["step"] % w.slots, state["cur"]
        if carry:                                             # one stream: the plan (depth limit of the previous step) rides
            if state["slices_for"] != state["step"]:         # in the attention launch, and inside a run of steps the draft
                c["a1"][s]()                                  # row's slice pass rides in the previous step's target-row launch
            c["a3p"][cur][s]()
            if last:
                c["a1t"][cur][s]()
            else:
                c["pair"][cur][s]()
                state["slices_for"] = state["step"] + 1
            c["a4"][cur][s]()
            acc_sum.add_(w.acc_len)
            state["cur"] ^= 1
            state["step"] += 1
            return
        main = torch.cuda.current_stream()
        plan_stream.wait_stream(main)                         # fork: the plan uses the depth limit of the previous step
        c["a3"][cur][s](); c["a1t"][cur][s](); c["a4"][cur][s]()
        acc_sum.add_(w.acc_len)
        c["a1"][s](); c["a2"][cur]()                          # plan branch, enqueued after the verification branch
        main.wait_stream(plan_stream)                         # join: the next step verifies the tree planned here
        state["cur"] ^= 1
        state["step"] += 1

    def reset():
        kv_len.copy_(kv_len0); hist.zero_(); count.zero_(); acc_sum.zero_()
        for dm in d_max:
            dm.fill_(w.tree_prm["d_max"])
        for t, t0 in zip(w.tree, tree0):
            for k in t:
                t[k].copy_(t0[k])
        state.update(cur=0, step=0, slices_for=-1)

    def snapshot_state():
        grown = int((kv_len - kv_len0).max().item())
        rows = torch.cat([Kc[b * cap + int(w.kv_lens[b]):b * cap + int(w.kv_lens[b]) + grown] for b in range(B)])
        return [x.clone() for x in (kv_len, hist, count, d_max[state["cur"]], acc_sum, w.acc_len, w.O, rows)]

    eager = prep(None)
    reset()
    for _ in range(steps):
        step(eager)
    torch.cuda.synchronize()
    want = snapshot_state()
    reset()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graphed = prep(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        for i in range(cycle):
            step(graphed, last=i == cycle - 1)
    reset()                                                    # capture does not execute, but keep the start exact
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps // cycle):
        graph.replay()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    got = snapshot_state()
    verified = all(torch.equal(a, b) for a, b in zip(want, got))
    out = dict(workload=name, steps=steps, steps_per_s=steps / wall, ms_per_step=wall * 1e3 / steps,
               calls_per_step=("tree_attention_with_plan (per-sequence depth), entropy_topk_slices_pair (target rows + the next "
                               "step's draft row), verify_accept_close_from_slices (acceptance, commit, advance, history); one "
                               "stream; the first step of a graph runs entropy_topk_slices on its draft row itself") if carry else
                              ("entropy_topk_slices, build_tree_from_slices (per-sequence depth), tree_attention, "
                               "entropy_topk_slices (k=1), verify_accept_close_from_slices (acceptance, commit, advance, "
                               "history); the first two on a second stream beside the rest"),
               kv_len_start=[int(x) for x in w.kv_lens], kv_len_end=[int(x) for x in kv_len.cpu().numpy()],
               mean_accept_len=float(acc_sum.sum().item()) / (steps * B),
               d_max_end=[int(x) for x in d_max[state["cur"]].cpu().numpy()],
               replay_equals_eager=bool(verified))
    del w
    torch.cuda.empty_cache()
    return out


def lm_head_projection(dim=8192, vocab=152064, launches=12):
    """The target's greedy token and softmax statistics taken straight from the output projection at the 72B shape
    (sage_lm_head_topk): the [vocab, dim] weight matrix (2.5 GB) is streamed once, the rows x vocab logits never exist
    in memory.  Weights ~ N(0, 9/dim), hidden rows ~ N(0,1): logits ~ N(0, 9).  Cases: the 64 node rows of one tree,
    the 512 of a batch of eight with every row live (the contraction then bounds the call, not the weight stream),
    and the same batch with tree sizes like c4's (about 160 live rows, packed into three blocks)."""
    import torch
    from paper_2602_00523_amd import sage
    dev = "cuda:0"
    g = torch.Generator(device=dev)
    g.manual_seed(523007)
    W = (torch.randn(vocab, dim, generator=g, device=dev, dtype=torch.float32) * (3.0 / math.sqrt(dim))).to(torch.bfloat16)
    Wf = W.float()
    out = []
    for rows, n_valid in ((64, None), (512, None), (512, [12, 25, 9, 40, 16, 8, 30, 20])):
        H = torch.randn(rows, dim, generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
        ent = torch.zeros(rows, device=dev)
        idx = torch.zeros(rows, 1, device=dev, dtype=torch.int32)
        ws = torch.empty(sage.sage_lm_head_topk_workspace_bytes(rows, vocab, 1), device=dev, dtype=torch.uint8)
        nv = None if n_valid is None else torch.tensor(n_valid, device=dev, dtype=torch.int32)
        call = sage.prepare("sage_lm_head_topk", H, W, 1, ent, idx, None, None, None, None, ws, nv, 64)
        for _ in range(3):
            call()
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2 * launches)]
        for i in range(launches):
            ev[2 * i].record()
            call()
            ev[2 * i + 1].record()
        torch.cuda.synchronize()
        t = [ev[2 * i].elapsed_time(ev[2 * i + 1]) for i in range(launches)]
        avg_s = sum(t) / len(t) * 1e-3
        live = rows if n_valid is None else sum(n_valid)
        alive = torch.ones(rows, dtype=torch.bool, device=dev) if n_valid is None else \
            (torch.arange(rows, device=dev) % 64) < nv.repeat_interleave(64)
        byts = 2.0 * vocab * dim + 2.0 * live * dim            # the weights once, whatever the number of rows
        flops = 2.0 * live * dim * vocab
        ref = (H.float() @ Wf.T).argmax(1)
        out.append(dict(rows=rows, live_rows=live, dim=dim, vocab=vocab, avg_us=avg_s * 1e6, min_us=min(t) * 1e3,
                        algorithmic_bytes=byts, hbm_GBps=byts / avg_s / 1e9, hbm_frac=byts / avg_s / 1e9 / HBM_PEAK_GBPS,
                        mfma_TFLOPs=flops / avg_s / 1e12, mfma_frac=flops / avg_s / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                        bound="mfma" if flops / byts > MFMA_BF16_PEAK_TFLOPS * 1e3 / HBM_PEAK_GBPS else "hbm",
                        argmax_agrees_with_fp32_matmul=float((ref == idx[:, 0].long())[alive].float().mean().item())))
        del H
    del W, Wf
    torch.cuda.empty_cache()
    # The draft side (Sec. 3.1): a 7B-shape projection (hidden 3584) with candidate lists of k = 10, for the one row of a
    # step's root and for the 16 rows of a wide tree level.
    ddim, k = 3584, 10
    Wd = (torch.randn(vocab, ddim, generator=g, device=dev, dtype=torch.float32) * (3.0 / math.sqrt(ddim))).to(torch.bfloat16)
    for rows in (1, 16):
        H = torch.randn(rows, ddim, generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
        f = lambda *sh: torch.zeros(*sh, device=dev)
        ent, hk, al, pr, rn = f(rows), f(rows), f(rows), f(rows, k), f(rows, k)
        idx = torch.zeros(rows, k, device=dev, dtype=torch.int32)
        ws = torch.empty(sage.sage_lm_head_topk_workspace_bytes(rows, vocab, k), device=dev, dtype=torch.uint8)
        call = sage.prepare("sage_lm_head_topk", H, Wd, k, ent, idx, pr, rn, hk, al, ws)
        for _ in range(3):
            call()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(launches):
            call()
        e1.record()
        torch.cuda.synchronize()
        avg_s = e0.elapsed_time(e1) * 1e-3 / launches
        byts = 2.0 * vocab * ddim + 2.0 * rows * ddim
        ref = torch.topk(H.float() @ Wd.float().T, k, dim=1).indices
        out.append(dict(rows=rows, live_rows=rows, dim=ddim, vocab=vocab, k=k, avg_us=avg_s * 1e6, algorithmic_bytes=byts,
                        hbm_GBps=byts / avg_s / 1e9, hbm_frac=byts / avg_s / 1e9 / HBM_PEAK_GBPS, bound="hbm",
                        topk_agrees_with_fp32_matmul=float((ref == idx.long()).float().mean().item())))
        del H
    del Wd
    torch.cuda.empty_cache()
    return out


def entropy_topk_streams(vocab=152064):
    """sage_entropy_topk alone: the target rows of one tree (64 x vocab, k = 1), a batch of them (512 rows) and the
    draft row (k = 10), as HIP-graph replays over rotating inputs (> 512 MB for the k = 1 cases)."""
    import torch
    from paper_2602_00523_amd import sage
    dev = "cuda:0"
    g = torch.Generator(device=dev)
    g.manual_seed(523011)
    out = []
    for rows, k, nbuf in ((64, 1, 32), (512, 1, 4), (1, 10, 64)):
        X = [(torch.randn(rows, vocab, generator=g, device=dev, dtype=torch.float32) * 2.0).to(torch.bfloat16) for _ in range(nbuf)]
        f = lambda *s: torch.zeros(*s, device=dev)
        H, pr, rn, hk, al = f(rows), f(rows, k), f(rows, k), f(rows), f(rows)
        idx = torch.zeros(rows, k, device=dev, dtype=torch.int32)
        ws = torch.empty(sage.sage_entropy_topk_workspace_bytes(rows, vocab, k), device=dev, dtype=torch.uint8)
        side = torch.cuda.Stream()
        calls = [sage.prepare("sage_entropy_topk", x, k, H, idx, pr, rn, hk, al, ws, stream=side) for x in X]
        with torch.cuda.stream(side):
            for c in calls:
                c()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for c in calls:
                c()
        graph.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 10
        e0.record()
        for _ in range(reps):
            graph.replay()
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / (reps * nbuf)
        byts = 2.0 * rows * vocab
        out.append(dict(rows=rows, k=k, vocab=vocab, us_per_call=us, algorithmic_bytes=byts, hbm_GBps=byts / us / 1e3,
                        hbm_frac=byts / us / 1e3 / HBM_PEAK_GBPS))
        del X
        torch.cuda.empty_cache()
    return out


def draft_side_attention(launches=40):
    """The same attention call at a draft-model shape: 28 query / 4 KV heads (group size 7), head_dim 128, and a cache
    whose visual positions were pruned to 10-20 % (Sec. 5 "Implementation details": 90 % pruning for video, 80 % for
    image), i.e. short caches: 3072 image + 1024 text -> 614 + 1024; 15360 video + 1024 text -> 1536 + 1024.  Trees of
    12 and 25 nodes with random topology.  HIP events around each launch, rotating K/V buffers."""
    import torch
    import numpy as np
    from paper_2602_00523_amd import sage
    dev = "cuda:0"
    Hq, Hkv, d = 28, 4, 128
    g = torch.Generator(device=dev)
    g.manual_seed(523013)
    rn = lambda *s: torch.randn(*s, generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    rng = np.random.default_rng(13)
    out = []
    for L, n in ((1638, 12), (2560, 12), (2560, 25)):
        nbuf = 16
        Kc = [rn(L, Hkv, d) for _ in range(nbuf)]
        Vc = [rn(L, Hkv, d) for _ in range(nbuf)]
        Q, Kt, Vt = rn(1, MAX_NODES, Hq, d), rn(1, MAX_NODES, Hkv, d), rn(1, MAX_NODES, Hkv, d)
        O = torch.zeros_like(Q)
        mask = np.zeros((1, MAX_NODES), np.uint64)
        par = [-1] + [int(rng.integers(0, v)) for v in range(1, n)]
        for v in range(n):
            u, bits = v, 0
            while u >= 0:
                bits |= 1 << u
                u = par[u]
            mask[0, v] = bits
        maskd = torch.from_numpy(mask.view(np.int64)).to(dev)
        nn = torch.full((1,), n, device=dev, dtype=torch.int32)
        kv_start = torch.zeros(1, device=dev, dtype=torch.int64)
        kv_len = torch.full((1,), L, device=dev, dtype=torch.int32)
        ws = torch.empty(sage.sage_tree_attention_workspace_bytes(sage.BF16, 1, Hq, Hkv, d, L), device=dev, dtype=torch.uint8)
        calls = [sage.prepare("sage_tree_attention", Q, Kc[i], Vc[i], Kt, Vt, O, kv_start, kv_len, L, Hkv * d, d, maskd, nn,
                              1.0 / math.sqrt(d), ws) for i in range(nbuf)]
        for c in calls:
            c()
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2 * launches)]
        for i in range(launches):
            ev[2 * i].record()
            calls[i % nbuf]()
            ev[2 * i + 1].record()
        torch.cuda.synchronize()
        t = [ev[2 * i].elapsed_time(ev[2 * i + 1]) for i in range(launches)]
        avg_ms = sum(t) / len(t)
        byts = 2.0 * 2 * L * Hkv * d + n * (2.0 * 2 * Hkv * d + 2.0 * 2 * Hq * d)
        out.append(dict(heads=f"{Hq}/{Hkv}", kv_len=L, nodes=n, avg_us=avg_ms * 1e3, min_us=min(t) * 1e3,
                        algorithmic_bytes=byts, hbm_GBps=byts / (avg_ms * 1e-3) / 1e9))

    # Level-by-level growth (Alg. 1 Phase 1: the draft model extends the tree by one level per forward pass): the same
    # call once per level on the level-ordered tree; call l sees the nodes of levels 0..l as keys and computes the rows
    # of level l only (first_node).  One drafting pass = all levels; the passes over the rotating K/V buffers are one
    # HIP graph, as a drafting loop would replay them.
    L, n = 2560, 25
    par = [-1] + [int(rng.integers(max(0, v - 6), v)) for v in range(1, n)]
    dep = [0] * n
    for v in range(1, n):
        dep[v] = dep[par[v]] + 1
    order = sorted(range(n), key=lambda v: (dep[v], v))          # level order: parents stay ahead of their children
    new_of_old = {o: i for i, o in enumerate(order)}
    par_l = [-1 if par[o] < 0 else new_of_old[par[o]] for o in order]
    dep_l = [dep[o] for o in order]
    mask = np.zeros((1, MAX_NODES), np.uint64)
    for v in range(n):
        u, bits = v, 0
        while u >= 0:
            bits |= 1 << u
            u = par_l[u]
        mask[0, v] = bits
    maskd = torch.from_numpy(mask.view(np.int64)).to(dev)
    counts = [sum(1 for x in dep_l if x <= lvl) for lvl in range(max(dep_l) + 1)]
    nns = [torch.full((1,), c, device=dev, dtype=torch.int32) for c in counts]
    firsts = [torch.full((1,), c, device=dev, dtype=torch.int32) for c in [0] + counts[:-1]]
    nbuf = 16
    Kc = [rn(L, Hkv, d) for _ in range(nbuf)]
    Vc = [rn(L, Hkv, d) for _ in range(nbuf)]
    Q, Kt, Vt = rn(1, MAX_NODES, Hq, d), rn(1, MAX_NODES, Hkv, d), rn(1, MAX_NODES, Hkv, d)
    kv_start = torch.zeros(1, device=dev, dtype=torch.int64)
    kv_len = torch.full((1,), L, device=dev, dtype=torch.int32)
    ws = torch.empty(sage.sage_tree_attention_workspace_bytes(sage.BF16, 1, Hq, Hkv, d, L), device=dev, dtype=torch.uint8)
    side = torch.cuda.Stream()
    for rows_only in (False, True):
        O = torch.zeros_like(Q)
        passes = [[sage.prepare("sage_tree_attention", Q, Kc[i], Vc[i], Kt, Vt, O, kv_start, kv_len, L, Hkv * d, d, maskd, nn,
                                1.0 / math.sqrt(d), ws, stream=side, first_node=fn if rows_only else None)
                   for nn, fn in zip(nns, firsts)] for i in range(nbuf)]
        with torch.cuda.stream(side):
            for calls in passes:
                for c in calls:
                    c()
        torch.cuda.synchronize()
        eager = O.clone()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for calls in passes:
                for c in calls:
                    c()
        O.zero_()
        graph.replay()
        torch.cuda.synchronize()
        same = bool(torch.equal(O.view(torch.int16), eager.view(torch.int16)))
        reps = 20
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        with torch.cuda.stream(side):
            e0.record(side)
            for _ in range(reps):
                graph.replay()
            e1.record(side)
        torch.cuda.synchronize()
        us_pass = e0.elapsed_time(e1) * 1e3 / (reps * nbuf)
        out.append(dict(heads=f"{Hq}/{Hkv}", kv_len=L, growth="level by level",
                        rows_computed="the new level only (first_node)" if rows_only else "every node so far",
                        nodes_after_each_level=counts, calls_per_pass=len(counts), launch_mode="HIP graph replay",
                        replay_equals_eager=same, avg_us_per_pass=us_pass, avg_us_per_call=us_pass / len(counts)))
        del graph, passes
    return out


def run_workload(name, steps, warmup, slots=None, eager=False, all_schedules=False, verify=True):
    """Whole steps of one workload in its timed configuration plus the roofline of its attention call.  Returns
    (entry for the JSON line, the Workload object, still alive for the CPU baseline)."""
    import torch
    bf16 = name != "toy"
    # the reference state: the same number of steps modulo a cycle through the five separate calls, eagerly
    w = Workload(name, slots, fused=True, carry=bf16, overlap=not bf16)
    timing = time_steps(w, steps, warmup, not eager)
    torch.cuda.synchronize()
    ms = timing["wall_s"] * 1e3 / timing["timed_steps"]
    entry = {"workload": name, "description": WORKLOAD_TEXT[name], "ms_per_step": ms, "steps_per_s": 1e3 / ms,
             "launch_mode": timing["launch_mode"], "timed_steps": timing["timed_steps"], "replays": timing["replays"],
             "steps_per_replay": timing["steps_per_replay"], "eager_steps": timing["eager_steps"],
             "timed_region_ms": timing["wall_s"] * 1e3, "layers": w.layers, "batch": w.B, "input_sets": w.slots,
             "kv_sets": w.kv_slots, "kv_len": [int(x) for x in w.kv_lens], "tree_params": w.tree_prm,
             "schedule": ("one stream, three launches per step: sage_tree_attention_with_plan (first layer; sage_tree_attention for "
                          "the others), sage_entropy_topk_slices_pair, sage_verify_accept_from_slices.  The merge + tree rule of "
                          "the planning ride in the attention launch (the tree planned in a step is verified in the next one, "
                          "Sec. 3.2 lookahead) and the slice pass over the NEXT step's draft row shares the launch of this step's "
                          "target-row pass; the first step of a graph runs sage_entropy_topk_slices on its draft row itself") if bf16 else
                         ("two streams forked and joined every step: planning (sage_entropy_topk_slices, "
                          "sage_build_tree_from_slices) beside verification (sage_tree_attention, sage_entropy_topk_slices, "
                          "sage_verify_accept_from_slices)")}
    if verify:
        # the same step sequence through the five separate calls, eagerly, must end in the same state (bit for bit)
        ref = Workload(name, slots, fused=False)
        cycle = ref.slots if ref.slots % 2 == 0 else 2 * ref.slots
        for _ in range(cycle + w.step_no % cycle):
            ref.step()
        torch.cuda.synchronize()
        same = (ref.step_no - w.step_no) % cycle == 0 and all(torch.equal(a, b) for a, b in zip(snapshot(ref), snapshot(w)))
        entry["state_equals_separate_calls"] = bool(same)
        if not same:
            print(f"bench.py: {name}: the timed schedule and the five separate calls ended in different states", file=sys.stderr)
            sys.exit(4)
        if all_schedules:
            t = time_steps(ref, steps, warmup, not eager)
            entry["separate_calls_ms_per_step"] = t["wall_s"] * 1e3 / t["timed_steps"]
        del ref
        torch.cuda.empty_cache()
    if all_schedules:
        for key, kw in (("one_stream_ms_per_step", dict(fused=True)), ("two_streams_ms_per_step", dict(fused=True, overlap=True))):
            alt = Workload(name, slots, **kw)
            t = time_steps(alt, steps, warmup, not eager)
            entry[key] = t["wall_s"] * 1e3 / t["timed_steps"]
            del alt
            torch.cuda.empty_cache()
    w.carry, w.overlap = False, False                    # the measurement passes below run on one stream
    w._prepare(None)
    entry["roofline"] = attention_roofline(w, name)
    return entry, w


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    from paper_2602_00523_amd import sage
    sage.lib()                                          # fail loudly if the HIP library is not built

    def calibrate_copy():
        src = torch.empty(64 << 20, device="cuda:0", dtype=torch.uint8).random_()
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()

    if args.only:
        if args.calibrate_copy:
            calibrate_copy()
        if args.only == "attention":
            w = Workload(args.workload, args.slots)
            extra = attention_roofline(w, args.workload, eager=args.eager)
        else:
            extra = {"closed_loop": lambda: closed_loop("c2"), "lm_head": lm_head_projection,
                     "entropy_topk": entropy_topk_streams, "draft_side": draft_side_attention}[args.only]()
        print(json.dumps({args.only: extra}))
        return
    defaults = {"toy": (2000, 50), "c2": (2000, 100), "c3": (1024, 64), "c4": (320, 16), "c5": (24, 4)}
    steps = args.steps if args.steps is not None else defaults[args.workload][0]
    warmup = args.warmup if args.warmup is not None else defaults[args.workload][1]

    head, w = run_workload(args.workload, steps, warmup, args.slots, args.eager, args.all_schedules)
    roof = dict(head["roofline"])
    result = {
        "metric": "tree-verify steps/sec + attention HBM GB/s (% of peak), 72B shape, 1 MI355X",
        "value": head["steps_per_s"], "unit": "steps/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.cfg["dtype"], "data": "synthetic",
        "config": {"workload": f"{args.workload}: {WORKLOAD_TEXT[args.workload]}",
                   **{k: head[k] for k in ("layers", "batch", "input_sets", "kv_sets", "kv_len", "tree_params", "launch_mode",
                                           "timed_steps", "replays", "steps_per_replay", "eager_steps", "timed_region_ms",
                                           "schedule", "state_equals_separate_calls")
                      if k in head},
                   **{k: head[k] for k in ("separate_calls_ms_per_step", "one_stream_ms_per_step", "two_streams_ms_per_step")
                      if k in head},
                   "mean_tree_nodes": roof["mean_tree_nodes"]},
        "roofline": roof,
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, args.cpu_seconds)
    if args.calibrate_copy:
        calibrate_copy()
    del w
    torch.cuda.empty_cache()
    if not args.no_extras:
        # every configuration, whole steps and the attention call's roofline, from this same run
        by_workload = []
        for name in ("toy", "c2", "c3", "c4", "c5"):
            if name == args.workload:
                by_workload.append({k: v for k, v in head.items()})
                continue
            k_steps, k_warm = defaults[name]
            entry, wk = run_workload(name, min(k_steps, 512), min(k_warm, 32))
            del wk
            torch.cuda.empty_cache()
            by_workload.append(entry)
        result["by_workload"] = by_workload
        result["closed_loop"] = closed_loop("c2")
        result["lm_head_projection"] = lm_head_projection()
        result["entropy_topk_streams"] = entropy_topk_streams()
        result["draft_side_attention"] = draft_side_attention()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
