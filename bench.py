#!/usr/bin/env python3
"""Benchmark of the measurement-and-recovery decode step on one MI355X.

A step is one pass of the whole path over one batch: for each of the 32 layers of
a 7B-shaped decoder, sketch the head-usage and channel-usage vectors, recover the
head and channel-block supports, run head-pruned attention over the KV cache and
the block-sparse SwiGLU FFN on the recovered supports.  All inputs are synthetic
and seeded, resident in HBM before the timed region.

Prints one JSON line (see --help for the knobs).
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np
import torch

HBM_PEAK_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=100,
                    help="untimed steps before the timed ones.  The first 60-80 steps after the set-up run 2-3 %% slower "
                         "(the device comes out of an idle gap during graph capture), then the step time is flat for "
                         "seconds; only the last 3 warm-up steps have inputs of their own, the ones before them cycle "
                         "through the steps' graphs.  With a smaller value the set-up makes up the difference to 100 "
                         "replays (settle_steps in the output)")
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--batch", type=int, default=16)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="skip the single-layer side measurements")
    ap.add_argument("--counter-pass", action="store_true",
                    help="for rocprofv3 --pmc runs: one 1 GiB device copy (calibration), then every call once per "
                         "layer on one stream, no graphs, no timing")
    ap.add_argument("--prefill-pass", action="store_true",
                    help="run only the shared-support FFN at the two prompt shapes (configs 4 and 5) and print their "
                         "timings; the command the prefill profiles under profiles/ are taken from")
    ap.add_argument("--solver", choices=["omp", "iht"], default="omp",
                    help="recovery of the FFN block supports: block-OMP (default) or block iterative hard thresholding")
    ap.add_argument("--iht-iters", type=int, default=12)
    ap.add_argument("--recovery", choices=["next-step", "same-step"], default="next-step",
                    help="next-step: the sketches of step t give the supports step t+1 executes, and the recoveries of "
                         "all layers are solved in batched launches; same-step: every layer's support is recovered "
                         "just ahead of that layer's execution in the same step")
    ap.add_argument("--recovery-stream", choices=["second", "same"], default="same",
                    help="next-step mode: measurement and recovery on the execution stream between the groups' layers "
                         "(default: adds the kernels' own 0.18 ms to the step), or on a second stream beside execution "
                         "(the workgroups of the recovery hold compute units the FFN kernels need: measured slower, "
                         "the default run times both in alternation and reports them as stream_arrangements)")
    ap.add_argument("--groups", type=int, default=None,
                    help="next-step mode: number of layer groups per step (each is sketched and recovered with one launch per kind)")
    ap.add_argument("--no-verify", action="store_true",
                    help="skip the comparison of the last step's supports and outputs with the CPU oracle (after the timed region)")
    ap.add_argument("--no-graph", action="store_true", help="launch every kernel from the host instead of replaying HIP graphs")
    return ap.parse_args()


class DecodeState:
    """Weights, caches, dictionaries and per-step planted inputs of the decode workload."""

    def __init__(self, ctx, wl, binding, layers, B, nsteps, seed=3000):
        dev = "cuda:0"
        c, hs = wl.CFG2, wl.CFG3_HEADS
        self.c, self.hs, self.B, self.layers = c, hs, B, layers
        gen = torch.Generator(device=dev).manual_seed(seed)
        bf = torch.bfloat16

        def randn(shape, std=1.0, dtype=bf):
            t = torch.randn(shape, generator=gen, device=dev, dtype=torch.float32 if dtype != bf else bf)
            return t.mul_(std) if std != 1.0 else t

        self.Wg = [randn((c.G, c.b, c.d), c.wstd) for _ in range(layers)]
        self.Wu = [randn((c.G, c.b, c.d), c.wstd) for _ in range(layers)]
        self.Wd = [randn((c.G, c.d, c.b), c.wstd) for _ in range(layers)]
        self.K = [randn((B, hs.H, hs.L, hs.dh)) for _ in range(layers)]
        self.V = [randn((B, hs.H, hs.L, hs.dh)) for _ in range(layers)]
        # dictionaries: one unit-norm profile per channel block and layer
        self.pi = torch.randn((layers, c.G, c.b), generator=gen, device=dev)
        self.psi = [(self.pi[l] / self.pi[l].norm(dim=1, keepdim=True)).reshape(c.G, c.b, 1).contiguous()
                    for l in range(layers)]
        self.ffn_op = [binding.make_op(c.ens, seed, 2 * l, c.m, c.n) for l in range(layers)]
        self.head_op = [binding.make_op(hs.ens, seed, 2 * l + 1, hs.m, hs.H) for l in range(layers)]
        self.ffn_dict = [binding.make_dict(self.psi[l], c.G, c.b, 1) for l in range(layers)]
        self.head_dict = binding.make_dict(None, hs.H, 1, 1)
        for l in range(layers):
            ctx.cs_plan(self.ffn_op[l], self.ffn_dict[l], self.psi[l])
            ctx.cs_plan(self.head_op[l], self.head_dict)
        # per-step planted inputs (fresh every step)
        self.z, self.u, self.x, self.q, self.S_true, self.H_true = [], [], [], [], [], []
        for _ in range(nsteps):
            zs, us, st_, ht_ = [], [], [], []
            for l in range(layers):
                # k active blocks per token with Laplace magnitudes, plus dense background
                perm = torch.rand((B, c.G), generator=gen, device=dev).argsort(dim=1)[:, :c.k]
                amp = torch.zeros((B, c.G), device=dev)
                e = -torch.log(torch.rand((B, c.k), generator=gen, device=dev).clamp_min(1e-12))
                sgn = torch.where(torch.rand((B, c.k), generator=gen, device=dev) < 0.5, -1.0, 1.0)
                amp.scatter_(1, perm, e * sgn)
                z = (amp[:, :, None] * self.pi[l][None]).reshape(B, c.n)
                z += c.bg * torch.randn((B, c.n), generator=gen, device=dev)
                zs.append(z.contiguous())
                st_.append(perm)
                hperm = torch.rand((B, hs.H), generator=gen, device=dev).argsort(dim=1)[:, :hs.kh]
                u = hs.bg * torch.randn((B, hs.H), generator=gen, device=dev)
                u.scatter_add_(1, hperm, torch.randn((B, hs.kh), generator=gen, device=dev))
                us.append(u.contiguous())
                ht_.append(hperm)
            # one tensor per step, [layers][B][n]: a layer's usage vectors are a row block of it, and the
            # vectors of a group of layers can be sketched with one launch
            self.z.append(torch.stack(zs))
            self.u.append(torch.stack(us))
            self.S_true.append(torch.stack(st_))        # planted units, [layers][B][k], unordered
            self.H_true.append(torch.stack(ht_))
            self.x.append(randn((layers, B, c.d)))
            self.q.append(randn((layers, B, hs.H, hs.dh)))
        # outputs and intermediates, allocated once
        self.y = torch.empty((B, c.m), device=dev)
        self.yh = torch.empty((B, hs.m), device=dev)
        self.S = [torch.empty((B, c.k), dtype=torch.int32, device=dev) for _ in range(2)]
        self.heads = [torch.empty((B, hs.kh), dtype=torch.int32, device=dev) for _ in range(2)]
        self.resid = torch.empty((B,), device=dev)
        self.margin = torch.empty((B,), device=dev)
        self.marginh = torch.empty((B,), device=dev)
        # per-layer buffers of the pipelined step
        self.y_l = [torch.empty((B, c.m), device=dev) for _ in range(layers)]
        self.yh_l = [torch.empty((B, hs.m), device=dev) for _ in range(layers)]
        self.S_l = [torch.empty((B, c.k), dtype=torch.int32, device=dev) for _ in range(layers)]
        self.heads_l = [torch.empty((B, hs.kh), dtype=torch.int32, device=dev) for _ in range(layers)]
        self.margin_l = [torch.empty((B,), device=dev) for _ in range(layers)]
        self.marginh_l = [torch.empty((B,), device=dev) for _ in range(layers)]
        self.o = torch.empty((B, hs.H, hs.dh), device=dev, dtype=bf)
        self.out = torch.empty((B, c.d), device=dev, dtype=bf)
        # next-step mode: sketches of all layers of a step, and two generations of supports
        self.Y_all = torch.empty((layers, B, c.m), device=dev)
        self.Yh_all = torch.empty((layers, B, hs.m), device=dev)
        self.S_gen = [torch.zeros((layers, B, c.k), dtype=torch.int32, device=dev) for _ in range(2)]
        self.H_gen = [torch.zeros((layers, B, hs.kh), dtype=torch.int32, device=dev) for _ in range(2)]
        self.margin_all = torch.empty((layers, B), device=dev)
        self.marginh_all = torch.empty((layers, B), device=dev)
        self.groups = self.make_groups(binding, NEXT_GROUPS)

    def make_groups(self, binding, ngroups):
        """Layer groups of the batched measurement and recovery (ctypes arrays of operators and dictionaries per group)."""
        layers = self.layers
        groups = []
        ngroups = min(max(1, ngroups), layers)
        per = (layers + ngroups - 1) // ngroups
        for g0 in range(0, layers, per):
            ls = list(range(g0, min(layers, g0 + per)))
            groups.append({
                "layers": ls,
                "ffn_ops": (binding.CsOp * len(ls))(*[self.ffn_op[l] for l in ls]),
                "ffn_dicts": (binding.CsDict * len(ls))(*[self.ffn_dict[l] for l in ls]),
                "head_ops": (binding.CsOp * len(ls))(*[self.head_op[l] for l in ls]),
                "head_dicts": (binding.CsDict * len(ls))(*[self.head_dict for _ in ls]),
            })
        return groups


SOLVER = {"name": "omp", "iters": 12}
SETTLE_STEPS = 100  # untimed replays before the timed region, at least (set-up steps make up for a smaller --warmup)
NEXT_GROUPS = 1     # layer groups per step: each is sketched and recovered with one launch per kind


def recover_ffn(cx, st, l, y, S, margin):
    """FFN block-support recovery with the selected solver (support + confidence margin only)."""
    c = st.c
    if SOLVER["name"] == "iht":
        return cx.cs_recover_support_iht(st.ffn_op[l], st.ffn_dict[l], c.k, SOLVER["iters"], y, S, None, None, margin,
                                         want_coef=False, want_resid=False)
    return cx.cs_recover_support(st.ffn_op[l], st.ffn_dict[l], c.k, y, S, None, None, margin,
                                 want_coef=False, want_resid=False)


def decode_step(ctx, st, i, ev=None):
    """One decode step over all layers, every call in order on one stream.
    ev: optional dict of event lists for per-call timing."""
    c, hs = st.c, st.hs
    for l in range(st.layers):
        def timed(name, fn):
            if ev is None:
                return fn()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            fn()
            b.record()
            ev[name].append((a, b))
        timed("sketch", lambda: ctx.cs_sketch(st.head_op[l], st.u[i][l], st.yh))
        timed("recover", lambda: ctx.cs_recover_support(st.head_op[l], st.head_dict, hs.kh, st.yh, st.heads[0],
                                                        None, None, st.marginh, want_coef=False, want_resid=False))
        timed("attn", lambda: ctx.cs_head_attn(st.q[i][l], st.K[l], st.V[l], st.heads[0], st.o))
        timed("sketch", lambda: ctx.cs_sketch(st.ffn_op[l], st.z[i][l], st.y))
        timed("recover", lambda: recover_ffn(ctx, st, l, st.y, st.S[0], st.margin))
        timed("ffn", lambda: ctx.cs_block_ffn(st.Wg[l], st.Wu[l], st.Wd[l], st.x[i][l], st.S[0], False, st.out))


PIPE_CHUNK = 1      # layers per synchronisation point between the two streams
PIPE_AHEAD = 4      # chunks the recovery stream may run ahead of execution


def decode_step_pipelined(ctx, rctx, st, i, s_exec, s_rec, chunk=None, ahead=None):
    """The same step with measurement and recovery on a second stream, running ahead of execution
    (the recovered support is consumed by a later piece of reduced computation, paper Sec. 5).
    Every layer has its own support buffers.  The streams meet once per chunk of layers: execution
    of a chunk waits for the event that marks the chunk's supports ready, and recovery of chunk c
    waits until execution has finished chunk c - ahead, which keeps the two streams interleaved
    when the step is replayed as a graph without a cross-stream edge at every layer."""
    c, hs = st.c, st.hs
    chunk = PIPE_CHUNK if chunk is None else chunk
    ahead = PIPE_AHEAD if ahead is None else ahead
    s_rec.wait_stream(s_exec)
    nchunks = (st.layers + chunk - 1) // chunk
    done = [None] * nchunks
    for ci in range(nchunks):
        layers = range(ci * chunk, min(st.layers, (ci + 1) * chunk))
        with torch.cuda.stream(s_rec):
            if ci >= ahead:
                s_rec.wait_event(done[ci - ahead])
            for l in layers:
                rctx.cs_sketch(st.head_op[l], st.u[i][l], st.yh_l[l])
                rctx.cs_recover_support(st.head_op[l], st.head_dict, hs.kh, st.yh_l[l], st.heads_l[l],
                                        None, None, st.marginh_l[l], want_coef=False, want_resid=False)
                rctx.cs_sketch(st.ffn_op[l], st.z[i][l], st.y_l[l])
                recover_ffn(rctx, st, l, st.y_l[l], st.S_l[l], st.margin_l[l])
            ready = torch.cuda.Event()
            ready.record(s_rec)
        with torch.cuda.stream(s_exec):
            s_exec.wait_event(ready)
            for l in layers:
                ctx.cs_head_attn(st.q[i][l], st.K[l], st.V[l], st.heads_l[l], st.o)
                ctx.cs_block_ffn(st.Wg[l], st.Wu[l], st.Wd[l], st.x[i][l], st.S_l[l], False, st.out)
            done[ci] = torch.cuda.Event()
            done[ci].record(s_exec)
    s_exec.wait_stream(s_rec)


def sketch_group(cx, st, grp, i):
    """The sketches of one group of layers at step i, one launch per kind."""
    l0, l1 = grp["layers"][0], grp["layers"][-1] + 1
    cx.cs_sketch_multi(grp["head_ops"], st.u[i][l0:l1], st.Yh_all[l0:l1])
    cx.cs_sketch_multi(grp["ffn_ops"], st.z[i][l0:l1], st.Y_all[l0:l1])


def recover_group(cx, st, grp, gen):
    """Batched recovery of one group of layers into support generation `gen`."""
    c, hs = st.c, st.hs
    l0, l1 = grp["layers"][0], grp["layers"][-1] + 1
    cx.cs_recover_support_multi(grp["head_ops"], grp["head_dicts"], hs.kh, st.Yh_all[l0:l1], st.H_gen[gen][l0:l1],
                                None, None, st.marginh_all[l0:l1], want_coef=False, want_resid=False)
    cx.cs_recover_support_multi(grp["ffn_ops"], grp["ffn_dicts"], c.k, st.Y_all[l0:l1], st.S_gen[gen][l0:l1],
                                None, None, st.margin_all[l0:l1], want_coef=False, want_resid=False)


NEXT_INLINE = False   # True: measurement and recovery run on the execution stream, between the groups' layers


def support_source(st, l, i):
    """Where layer l's supports stand once step i has run: (generation, step whose usage they were recovered from)."""
    if not NEXT_INLINE and l in st.groups[-1]["layers"]:
        return i % 2, max(i - 1, 0)
    return (i + 1) % 2, i


def decode_step_next(ctx, rctx, st, i, s_exec, s_rec):
    """One decode step in which the sketches of a step give the supports of the next one (paper Sec. 5: the
    reduced computation for the next step uses the units recovered now).  Execution of layer l at step i
    reads generation i % 2.  A layer's usage vector exists once the layer has run, so the second stream
    measures a group of layers only after the execution stream has issued the group's last layer (one
    event per group), then recovers the group with one launch per kind into generation (i + 1) % 2.  The
    last group of a step would leave that work exposed at the end of the step; it is carried over instead:
    step i begins, on the second stream, with the last group's sketches of step i - 1 and their recovery
    into generation i % 2, and the execution stream waits for that once, just before the group's first
    layer.  The streams join at the end of the step."""
    cur, nxt = i % 2, (i + 1) % 2
    prev = max(i - 1, 0)
    last = st.groups[-1]
    s_rec.wait_stream(s_exec)
    with torch.cuda.stream(s_rec):
        sketch_group(rctx, st, last, prev)
        recover_group(rctx, st, last, cur)
        carried = torch.cuda.Event()
        carried.record(s_rec)
    for grp in st.groups:
        with torch.cuda.stream(s_exec):
            if grp is last:
                s_exec.wait_event(carried)
            for l in grp["layers"]:
                ctx.cs_head_attn(st.q[i][l], st.K[l], st.V[l], st.H_gen[cur][l], st.o)
                ctx.cs_block_ffn(st.Wg[l], st.Wu[l], st.Wd[l], st.x[i][l], st.S_gen[cur][l], False, st.out)
            if grp is not last:
                issued = torch.cuda.Event()
                issued.record(s_exec)
        if grp is not last:
            with torch.cuda.stream(s_rec):
                s_rec.wait_event(issued)
                sketch_group(rctx, st, grp, i)
                recover_group(rctx, st, grp, nxt)
    s_exec.wait_stream(s_rec)


def decode_step_next_inline(ctx, rctx, st, i, s_exec, s_rec):
    """The same data flow on one stream: after a group's layers have run, the group is sketched and recovered
    (one launch per kind) into the generation the next step reads.  No second stream, no events: the
    measurement and recovery launches add their own duration to the step and disturb nothing else."""
    cur, nxt = i % 2, (i + 1) % 2
    with torch.cuda.stream(s_exec):
        for grp in st.groups:
            for l in grp["layers"]:
                ctx.cs_head_attn(st.q[i][l], st.K[l], st.V[l], st.H_gen[cur][l], st.o)
                ctx.cs_block_ffn(st.Wg[l], st.Wu[l], st.Wd[l], st.x[i][l], st.S_gen[cur][l], False, st.out)
            sketch_group(ctx, st, grp, i)
            recover_group(ctx, st, grp, nxt)


def prime_supports(ctx, st):
    """Generation 0 of the supports, from the sketches of step 0 (before the timed region)."""
    for grp in st.groups:
        sketch_group(ctx, st, grp, 0)
        recover_group(ctx, st, grp, 0)



def call_loops(ctx, st, stream):
    """ms per call of each call type, measured with HIP events around loops that launch that
    call for every layer in turn (two passes after one warm pass).  Returns (per, mean union size)."""
    c, hs = st.c, st.hs
    nl = st.layers
    # supports of every layer from one recovery pass on step 0
    S_all, H_all = [], []
    for l in range(nl):
        ctx.cs_sketch(st.ffn_op[l], st.z[0][l], st.y)
        S_all.append(recover_ffn(ctx, st, l, st.y, None, st.margin)[0])
        ctx.cs_sketch(st.head_op[l], st.u[0][l], st.yh)
        H_all.append(ctx.cs_recover_support(st.head_op[l], st.head_dict, hs.kh, st.yh, None, None, None, st.marginh,
                                            want_coef=False, want_resid=False)[0])
    torch.cuda.synchronize()
    union_mean = float(np.mean([union_blocks(S, c.G) for S in S_all]))
    loops = {
        "attn": lambda i: ctx.cs_head_attn(st.q[0][i % nl], st.K[i % nl], st.V[i % nl], H_all[i % nl], st.o),
        "ffn": lambda i: ctx.cs_block_ffn(st.Wg[i % nl], st.Wu[i % nl], st.Wd[i % nl], st.x[0][i % nl], S_all[i % nl],
                                          False, st.out),
        "recover_ffn": lambda i: recover_ffn(ctx, st, i % nl, st.y, st.S[0], st.margin),
        "recover_heads": lambda i: ctx.cs_recover_support(st.head_op[i % nl], st.head_dict, hs.kh, st.yh, st.heads[0],
                                                          None, None, st.marginh, want_coef=False, want_resid=False),
        "sketch_ffn": lambda i: ctx.cs_sketch(st.ffn_op[i % nl], st.z[0][i % nl], st.y),
        "sketch_heads": lambda i: ctx.cs_sketch(st.head_op[i % nl], st.u[0][i % nl], st.yh),
    }
    raw = {}
    for name, fn in loops.items():
        time_loop(fn, nl, stream)
        raw[name] = time_loop(fn, 2 * nl, stream)
    # batched recovery of a whole step (all groups, both kinds), as the next-step mode launches it
    fn = lambda i: [recover_group(ctx, st, grp, 1) for grp in st.groups]
    time_loop(fn, 2, stream)
    raw["recover_step_batched"] = time_loop(fn, 8, stream)
    fn = lambda i: [sketch_group(ctx, st, grp, 0) for grp in st.groups]
    time_loop(fn, 2, stream)
    raw["sketch_step_batched"] = time_loop(fn, 8, stream)
    per = {"attn": raw["attn"], "ffn": raw["ffn"], "recover_step_batched": raw["recover_step_batched"],
           "sketch_step_batched": raw["sketch_step_batched"],
           "recover": 0.5 * (raw["recover_ffn"] + raw["recover_heads"]),
           "sketch": 0.5 * (raw["sketch_ffn"] + raw["sketch_heads"])}
    per.update({k: raw[k] for k in ("recover_ffn", "recover_heads", "sketch_ffn", "sketch_heads")})
    return per, union_mean


def recorded_traffic(call):
    """HBM bytes per launch of `call` from the committed rocprofv3 --pmc summary, or None when the
    kernel sources have changed since the counters were taken."""
    import hashlib
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if not os.path.exists(path):
        return None
    rec = json.load(open(path)).get("calls", {}).get(call)
    if rec is None:
        return None
    for fname, digest in rec["sources"].items():
        src = os.path.join(ROOT, "paper_2604_14156_amd", "csrc", fname)
        if not os.path.exists(src) or hashlib.sha256(open(src, "rb").read()).hexdigest() != digest:
            return None
    return rec["hbm_bytes_per_call"]


def union_blocks(S, G):
    return int(torch.unique(S).numel())


def verify_last_step(ctx, st, wl, i_last, n_layers_sup=4, n_layers_out=2):
    """After the timed region: what the last step left on the device against the CPU oracle.
    Supports: for `n_layers_sup` layers spread over the stack and all tokens, the oracle sketches the same
    usage vectors and recovers from its own sketches; a support counts as exact when it is the oracle's set,
    as valid when it is exact or, below the oracle's selection margin of 1e-3, a greedy path within a
    relative slack of 1e-3 (the oracle reproduces it when told to prefer its units).  Outputs: for
    `n_layers_out` layers the attention and FFN calls of the step are issued again with the step's supports
    and every (sequence, kept head) and token is compared with the oracle (relative L2 and largest element
    error over the row's root mean square).  Also, over all layers and tokens: the overlap of the recovered
    with the planted supports (F1; both sets have k units, so F1 = overlap / k) and the share of problems
    whose reported margin clears 1e-3."""
    import oracle
    c, hs = st.c, st.hs
    nl, B = st.layers, st.B
    host = lambda t: t.detach().float().cpu().numpy().astype(np.float64) if t.is_floating_point() else t.cpu().numpy()
    pick = sorted(set(int(round(v)) for v in np.linspace(0, nl - 1, min(n_layers_sup, nl))))
    res = {"layers_checked": pick, "supports_checked": 0, "supports_exact": 0, "supports_valid": 0,
           "heads_checked": 0, "heads_exact": 0, "heads_valid": 0, "sketch_max_rel_err": 0.0}
    seed = st.ffn_op[0].seed
    for l in pick:
        gen, src = support_source(st, l, i_last)
        psi = host(st.psi[l]).reshape(c.G, c.b, 1)
        M = oracle.effective_matrix(c.ens, seed, st.ffn_op[l].stream_id, c.m, c.n, c.G, c.b, 1, psi)
        Y = oracle.sketch(c.ens, seed, st.ffn_op[l].stream_id, c.m, host(st.z[src][l]))
        got_y, got_S = host(st.Y_all[l]), host(st.S_gen[gen][l])
        Mh = oracle.effective_matrix(hs.ens, seed, st.head_op[l].stream_id, hs.m, hs.H, hs.H, 1, 1, None)
        Yh = oracle.sketch(hs.ens, seed, st.head_op[l].stream_id, hs.m, host(st.u[src][l]))
        got_H = host(st.H_gen[gen][l])
        for t in range(B):
            res["sketch_max_rel_err"] = max(res["sketch_max_rel_err"],
                                            float(np.linalg.norm(got_y[t] - Y[t]) / np.linalg.norm(Y[t])))
            for key, Mx, y, G, k, norm, got in (("supports", M, Y[t], c.G, c.k, True, got_S[t]),
                                                 ("heads", Mh, Yh[t], hs.H, hs.kh, False, got_H[t])):
                rec = oracle.block_omp(Mx, y, G, 1, k, norm)
                res[key + "_checked"] += 1
                if list(got) == list(rec["support"]):
                    res[key + "_exact"] += 1
                    res[key + "_valid"] += 1
                elif rec["margin"] <= 1e-3:
                    rep = oracle.block_omp(Mx, y, G, 1, k, norm, prefer=got, slack=1e-3)
                    res[key + "_valid"] += int(list(rep["support"]) == list(got))
    # planted-support overlap and margin pass rate over the whole step
    f1_ffn, f1_heads, mp, mph = [], [], [], []
    for l in range(nl):
        gen, src = support_source(st, l, i_last)
        S, Sp = st.S_gen[gen][l].long(), st.S_true[src][l]
        f1_ffn.append(float((S[:, :, None] == Sp[:, None, :]).any(dim=2).float().mean()))
        Hh, Hp = st.H_gen[gen][l].long(), st.H_true[src][l]
        f1_heads.append(float((Hh[:, :, None] == Hp[:, None, :]).any(dim=2).float().mean()))
    res["planted_f1_ffn"] = float(np.mean(f1_ffn))
    res["planted_f1_heads"] = float(np.mean(f1_heads))
    res["margin_pass_rate_ffn"] = float((st.margin_all > 1e-3).float().mean())
    res["margin_pass_rate_heads"] = float((st.marginh_all > 1e-3).float().mean())
    res["problems_in_pass_rate"] = int(st.margin_all.numel())
    # outputs of the step's execution calls
    worst = {"attn_rel_l2": 0.0, "attn_elt_over_rms": 0.0, "ffn_rel_l2": 0.0, "ffn_elt_over_rms": 0.0}
    rows = 0
    for l in pick[:: max(1, len(pick) // n_layers_out)][:n_layers_out]:
        gen, _ = support_source(st, l, i_last)
        o = torch.empty_like(st.o)
        out = torch.empty_like(st.out)
        ctx.cs_head_attn(st.q[i_last][l], st.K[l], st.V[l], st.H_gen[gen][l], o)
        ctx.cs_block_ffn(st.Wg[l], st.Wu[l], st.Wd[l], st.x[i_last][l], st.S_gen[gen][l], False, out)
        torch.cuda.synchronize()
        heads = st.H_gen[gen][l].long()
        go, gout = host(o), host(out)
        for b in range(B):
            Kb, Vb = host(st.K[l][b][heads[b]]), host(st.V[l][b][heads[b]])
            qb = host(st.q[i_last][l][b][heads[b]])
            want = oracle.head_attn(qb[None], Kb[None], Vb[None], np.arange(hs.kh)[None])[0]
            for j, h in enumerate(heads[b].tolist()):
                e = go[b, h] - want[j]
                worst["attn_rel_l2"] = max(worst["attn_rel_l2"], float(np.linalg.norm(e) / np.linalg.norm(want[j])))
                worst["attn_elt_over_rms"] = max(worst["attn_elt_over_rms"], float(np.abs(e).max() / np.sqrt(np.mean(want[j] ** 2))))
                rows += 1
        hWg, hWu, hWd = host(st.Wg[l]), host(st.Wu[l]), host(st.Wd[l])
        want = oracle.block_ffn(hWg, hWu, hWd, host(st.x[i_last][l]), host(st.S_gen[gen][l]))
        del hWg, hWu, hWd
        for t in range(B):
            e = gout[t] - want[t]
            worst["ffn_rel_l2"] = max(worst["ffn_rel_l2"], float(np.linalg.norm(e) / np.linalg.norm(want[t])))
            worst["ffn_elt_over_rms"] = max(worst["ffn_elt_over_rms"], float(np.abs(e).max() / np.sqrt(np.mean(want[t] ** 2))))
            rows += 1
    res["outputs"] = dict(worst, rows_checked=rows, tolerance=2e-2,
                          within_tolerance=bool(max(worst.values()) <= 2e-2))
    return res


def cpu_baseline(wl, layers_all=12, layers_one=3, B=16, seed=3000):
    """The CPU oracle, as it stands, on a bounded sample of the same workload: whole layers of one decode
    step (sketch, block-OMP, attention over the kept heads, FFN), once with the thread pools of the
    numerical libraries as they come (`cores`), once limited to one thread."""
    import oracle
    from threadpoolctl import threadpool_info, threadpool_limits
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    c, hs = wl.CFG2, wl.CFG3_HEADS
    rng = wl.rng_for(seed)
    # inputs and plan-time products (not timed)
    pi, psi = wl.make_profiles(rng, c.G, c.b)
    Wg, Wu, Wd = wl.make_ffn_weights(rng, c.G, c.b, c.d, c.wstd, "bf16")
    M = oracle.effective_matrix(c.ens, seed, 0, c.m, c.n, c.G, c.b, 1, psi)
    Mh = oracle.effective_matrix(hs.ens, seed, 1, hs.m, hs.H, hs.H, 1, 1, None)
    # the cache is materialised for kh heads only: the oracle touches kept heads alone, so the
    # recovered head set is relabelled 0..kh-1 (same arithmetic, 12/32 of the host memory)
    q, K, V = wl.make_kv(rng, B, hs.kh, hs.L, hs.dh)
    compact = np.tile(np.arange(hs.kh), (B, 1))

    def layers(n):
        t_total = 0.0
        for _ in range(n):
            z, _ = wl.plant_usage(rng, pi, c.k, B, c.amp, c.bg)
            u, _ = wl.plant_head_usage(rng, hs, B)
            x = wl.make_tokens(rng, B, c.d, "bf16")
            t0 = time.perf_counter()
            yh = oracle.sketch(hs.ens, seed, 1, hs.m, u)
            heads = np.stack([oracle.block_omp(Mh, yh[t], hs.H, 1, hs.kh, False)["support"] for t in range(B)])
            assert heads.shape == compact.shape
            oracle.head_attn(q, K, V, compact)
            y = oracle.sketch(c.ens, seed, 0, c.m, z)
            S = np.stack([oracle.block_omp(M, y[t], c.G, 1, c.k, True)["support"] for t in range(B)])
            oracle.block_ffn(Wg, Wu, Wd, x, S)
            t_total += time.perf_counter() - t0
        return t_total

    t_all = layers(layers_all)
    with threadpool_limits(limits=1):
        t_one = layers(layers_one)
    rate = lambda t, n: B / (t / n * 32)

    # the oracle's plain C twin (loops, -O2, OpenMP over independent tokens and rows) on the same layers:
    # what the host does without an interpreter and without a tuned BLAS, on one core and on all of them
    def twin_layers(n):
        from oracle import c_twin
        t_total = 0.0
        for _ in range(n):
            z, _ = wl.plant_usage(rng, pi, c.k, B, c.amp, c.bg)
            u, _ = wl.plant_head_usage(rng, hs, B)
            x = wl.make_tokens(rng, B, c.d, "bf16")
            t0 = time.perf_counter()
            yh = c_twin.sketch(hs.ens, seed, 1, hs.m, u)
            c_twin.block_omp(Mh, yh, hs.H, hs.kh, False)
            c_twin.head_attn(q64, K64, V64, compact)
            y = c_twin.sketch(c.ens, seed, 0, c.m, z)
            S = c_twin.block_omp(M, y, c.G, c.k, True)[0]
            c_twin.block_ffn(Wg64, Wu64, Wd64, x, S)
            t_total += time.perf_counter() - t0
        return t_total

    twin = None
    try:
        from oracle import c_twin
        Wg64, Wu64, Wd64 = (np.ascontiguousarray(w, dtype=np.float64) for w in (Wg, Wu, Wd))
        q64, K64, V64 = (np.ascontiguousarray(w, dtype=np.float64) for w in (q, K, V))
        ncores = c_twin.set_threads(0)
        t_tw_all = twin_layers(32)
        c_twin.set_threads(1)
        t_tw_one = twin_layers(8)
        c_twin.set_threads(0)
        twin = {"all_cores": {"value": rate(t_tw_all, 32), "unit": "tokens/s", "cores": ncores,
                              "sample": "32 of 32 layers (%.1f s)" % t_tw_all},
                "single_thread": {"value": rate(t_tw_one, 8), "unit": "tokens/s", "cores": 1,
                                  "sample": "8 of 32 layers (%.1f s), scaled to 32 layers" % t_tw_one},
                "what": "oracle/c_twin: the same definitions as plain C loops in fp64 (gcc -O2, OpenMP over tokens and rows)"}
    except Exception as exc:                              # no compiler on the box: the NumPy figures stand alone
        twin = {"error": str(exc)[:200]}
    numpy_leg = {"value": rate(t_all, layers_all), "unit": "tokens/s", "cores": int(threads),
                 "sample": "%d of 32 layers of one decode step at batch %d (%.1f s), scaled to 32 layers"
                           % (layers_all, B, t_all),
                 "single_thread": {"value": rate(t_one, layers_one), "unit": "tokens/s", "cores": 1,
                                   "sample": "%d of 32 layers (%.1f s), scaled to 32 layers" % (layers_one, t_one)},
                 "what": "oracle/*.py: NumPy fp64, Python loops over tokens and rounds, the numerical libraries' thread pools as they come"}
    if "all_cores" in twin:
        # the headline of the baseline is the faster of the two forms of the oracle: the C twin on all cores
        return {"value": twin["all_cores"]["value"], "unit": "tokens/s", "cores": twin["all_cores"]["cores"], "kind": "oracle",
                "sample": "oracle/c_twin (plain C loops, fp64, gcc -O2, OpenMP over tokens and rows): "
                          + twin["all_cores"]["sample"] + " of one decode step at batch %d" % B,
                "single_thread": twin["single_thread"], "numpy_oracle": numpy_leg}
    out = dict(numpy_leg)
    out["kind"] = "oracle"
    out["c_twin"] = twin
    return out


def time_loop(fn, iters, stream):
    """ms per iteration between two HIP events recorded on `stream`."""
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record(stream)
    for i in range(iters):
        fn(i)
    b.record(stream)
    b.synchronize()
    return a.elapsed_time(b) / iters          # ms per iteration


MFMA_BF16_PEAK_TFLOPS = 2500.0


def prefill_measurements(ctx, wl, stream, binding_mod, iters=20):
    """Shared-support FFN (one support for all rows) at the two prompt shapes: config 4 (T = 2048 rows,
    d = 8192, 112 of 448 blocks) and config 5 (2048 kept tokens, d = 4096, 43 of 172 blocks).  The call is a
    dense contraction over the gathered blocks, 6 T |S| b d flop, priced against the bf16 matrix peak.
    `net_us` adds what selects the support in front of it on the same stream: config 4 the sketch of the
    prompt-level usage vector and its recovery; config 5 the two sketches, joint token/unit selection and
    the gather of the kept tokens' rows."""
    dev = "cuda:0"
    res = {}
    for name, c, T in (("cfg4", wl.CFG4, 2048), ("cfg5", wl.CFG2, wl.CFG5_TOK["k_tok"])):
        gen = torch.Generator(device=dev).manual_seed(4000 if name == "cfg4" else 5000)
        Wg, Wu = (torch.randn((c.G, c.b, c.d), generator=gen, device=dev).mul_(c.wstd).to(torch.bfloat16) for _ in range(2))
        Wd = torch.randn((c.G, c.d, c.b), generator=gen, device=dev).mul_(c.wstd).to(torch.bfloat16)
        x = torch.randn((T, c.d), generator=gen, device=dev).to(torch.bfloat16)
        sup = torch.rand((c.G,), generator=gen, device=dev).argsort()[:c.k].sort().values.to(torch.int32).contiguous()
        out = torch.empty_like(x)
        fn = lambda i: ctx.cs_block_ffn(Wg, Wu, Wd, x, sup, True, out)
        time_loop(fn, iters, stream)                  # also brings the clocks up: the first calls run 15 % slower
        ms = time_loop(fn, iters, stream)
        flop = 6.0 * T * c.k * c.b * c.d
        # net: selection of the support in front of the layer
        pi = torch.randn((c.G, c.b), generator=gen, device=dev)
        psi = (pi / pi.norm(dim=1, keepdim=True)).reshape(c.G, c.b, 1).contiguous()
        op = binding_mod.make_op(c.ens, 4000, 900, c.m, c.n)
        dct = binding_mod.make_dict(psi, c.G, c.b, 1)
        ctx.cs_plan(op, dct, psi)
        zbar = torch.randn((1, c.n), generator=gen, device=dev)
        ybar = torch.empty((1, c.m), device=dev)
        S_rec = torch.empty((1, c.k), dtype=torch.int32, device=dev)
        mg = torch.empty((1,), device=dev)
        if name == "cfg4":
            def net(i):
                ctx.cs_sketch(op, zbar, ybar)
                ctx.cs_recover_support(op, dct, c.k, ybar, S_rec, None, None, mg, want_coef=False, want_resid=False)
                ctx.cs_block_ffn(Wg, Wu, Wd, x, sup, True, out)
        else:
            t = wl.CFG5_TOK
            tok_op = binding_mod.make_op(t["ens"], 5000, 901, t["m_tok"], t["n_tok"])
            sal = torch.randn((1, t["n_tok"]), generator=gen, device=dev)
            y_tok = torch.empty((1, t["m_tok"]), device=dev)
            X_all = torch.randn((t["n_tok"], c.d), generator=gen, device=dev).to(torch.bfloat16)

            def net(i):
                ctx.cs_sketch(tok_op, sal, y_tok)
                ctx.cs_sketch(op, zbar, ybar)
                tokens = ctx.cs_joint_select(tok_op, y_tok[0], T, op, dct, ybar[0], c.k)[0]
                ctx.cs_gather_rows(X_all, tokens, x)
                ctx.cs_block_ffn(Wg, Wu, Wd, x, sup, True, out)
        time_loop(net, 4, stream)
        net_ms = time_loop(net, iters, stream)
        res["prefill_ffn_" + name] = {"us": ms * 1e3, "net_us": net_ms * 1e3, "rows": T, "d": c.d, "blocks": "%d/%d" % (c.k, c.G),
                                      "TFLOP": flop / 1e12, "TFLOPs": flop / (ms * 1e-3) / 1e12,
                                      "mfma_frac": flop / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS}
        ctx.cs_plan_drop(op, dct)
        del Wg, Wu, Wd, x, out
    return res


def extra_measurements(ctx, st, wl, stream, binding_mod):
    """Single-layer side figures: FFN at batch 1/8/64 on rotating layers, recovery and sketch per call."""
    c, hs = st.c, st.hs
    dev = "cuda:0"
    res = {}
    nl = st.layers
    gen = torch.Generator(device=dev).manual_seed(77)
    for B in (1, 8, 64):
        sup = [torch.rand((B, c.G), generator=gen, device=dev).argsort(dim=1)[:, :c.k].to(torch.int32).contiguous()
               for _ in range(nl)]
        x = torch.randn((B, c.d), generator=gen, device=dev).to(torch.bfloat16)
        out = torch.empty_like(x)
        fn = lambda i: ctx.cs_block_ffn(st.Wg[i % nl], st.Wu[i % nl], st.Wd[i % nl], x, sup[i % nl], False, out)
        time_loop(fn, nl, stream)
        ms = time_loop(fn, 2 * nl, stream)
        blocks = float(np.mean([union_blocks(s, c.G) for s in sup]))
        bytes_active = blocks * 3 * c.b * c.d * 2
        # net: measurement and recovery of the same tokens in front of the layer, on one stream
        zB = st.z[0][0][:1].expand(B, c.n).contiguous() if B > st.B else st.z[0][0][:B].contiguous()
        yB = torch.empty((B, c.m), device=dev)
        SB = torch.empty((B, c.k), dtype=torch.int32, device=dev)
        mB = torch.empty((B,), device=dev)

        def net(i):
            l = i % nl
            ctx.cs_sketch(st.ffn_op[l], zB, yB)
            ctx.cs_recover_support(st.ffn_op[l], st.ffn_dict[l], c.k, yB, SB, None, None, mB, want_coef=False, want_resid=False)
            ctx.cs_block_ffn(st.Wg[l], st.Wu[l], st.Wd[l], x, sup[l], False, out)
        time_loop(net, nl, stream)
        net_ms = time_loop(net, 2 * nl, stream)
        res["ffn_B%d" % B] = {"us": ms * 1e3, "active_MB": bytes_active / 1e6,
                              "GBs": bytes_active / (ms * 1e-3) / 1e9,
                              "hbm_frac": bytes_active / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                              "tokens_per_s_layer": B / (ms * 1e-3),
                              "net_us_with_sketch_and_recovery": net_ms * 1e3}
    B = st.B
    ctx.cs_sketch(st.ffn_op[0], st.z[0][0], st.y)
    ctx.cs_sketch(st.head_op[0], st.u[0][0], st.yh)
    for tag, fit in (("support_margin", False), ("with_refit", True)):
        coef = torch.empty((B, c.k), device=dev) if fit else None
        fn = lambda i: ctx.cs_recover_support(st.ffn_op[i % nl], st.ffn_dict[i % nl], c.k, st.y, st.S[0], coef,
                                              st.resid if fit else None, st.margin, want_coef=False, want_resid=False)
        time_loop(fn, nl, stream)
        res["recover_ffn_us_per_call_B%d_%s" % (B, tag)] = time_loop(fn, 2 * nl, stream) * 1e3
        coefh = torch.empty((B, hs.kh), device=dev) if fit else None
        fn = lambda i: ctx.cs_recover_support(st.head_op[i % nl], st.head_dict, hs.kh, st.yh, st.heads[0], coefh,
                                              st.resid if fit else None, st.marginh, want_coef=False, want_resid=False)
        time_loop(fn, nl, stream)
        res["recover_heads_us_per_call_B%d_%s" % (B, tag)] = time_loop(fn, 2 * nl, stream) * 1e3
    # warm-started recovery: previous supports = an earlier recovery of the same shape, drift budget `swaps`
    prev = torch.empty((B, c.k), dtype=torch.int32, device=dev)
    ctx.cs_recover_support(st.ffn_op[0], st.ffn_dict[0], c.k, st.y, prev, None, None, st.margin,
                           want_coef=False, want_resid=False)
    for swaps in (0, 2, 4, 8):
        fn = lambda i: ctx.cs_recover_support_inc(st.ffn_op[i % nl], st.ffn_dict[i % nl], c.k, st.y, prev, swaps,
                                                  support=st.S[0], margin=st.margin, want_coef=False, want_resid=False)
        time_loop(fn, nl, stream)
        res["recover_ffn_incremental_us_per_call_B%d_swaps%d" % (B, swaps)] = time_loop(fn, 2 * nl, stream) * 1e3
    # the same exchange with the state carried from call to call: every layer keeps its own previous supports
    # (updated in place by each call, as a decode loop would) and its own state
    prevs = prev.unsqueeze(0).repeat(nl, 1, 1).contiguous()
    states = [ctx.cs_inc_state(B, c.k, dev) for _ in range(nl)]
    for swaps in (0, 2, 4, 8):
        fn = lambda i: ctx.cs_recover_support_inc_carry(st.ffn_op[i % nl], st.ffn_dict[i % nl], c.k, st.y, prevs[i % nl], swaps,
                                                        states[i % nl], support=prevs[i % nl], margin=st.margin,
                                                        want_coef=False, want_resid=False)
        time_loop(fn, 2 * nl, stream)                     # first pass builds the states, second settles the supports
        res["recover_ffn_carried_us_per_call_B%d_swaps%d" % (B, swaps)] = time_loop(fn, 2 * nl, stream) * 1e3
    res["recover_ffn_carried_state_age"] = int(states[0][0, 1])
    fn = lambda i: ctx.cs_sketch(st.ffn_op[i % nl], st.z[0][i % nl], st.y)
    time_loop(fn, nl, stream)
    res["sketch_ffn_us_per_call_B%d" % B] = time_loop(fn, 2 * nl, stream) * 1e3
    # measurement cost against the budget m (the controller of Sec. 8.1 moves m between steps): dense
    # Rademacher sketch and the fast-transform Hadamard sketch, and the controller's entropy sensor
    curve = {}
    for m_t in (64, 128, 256, 512):
        yb = torch.empty((B, m_t), device=dev)
        for name, ens in (("rademacher", wl.RADEMACHER), ("hadamard", wl.SRHT)):
            op_t = binding_mod.make_op(ens, 5, 2001, m_t, c.n)
            fn = lambda i: ctx.cs_sketch(op_t, st.z[0][i % nl], yb)
            time_loop(fn, nl, stream)
            curve["%s_m%d" % (name, m_t)] = time_loop(fn, 2 * nl, stream) * 1e3
    res["sketch_us_per_call_B%d_vs_m" % B] = curve
    logits = torch.randn((B, 128256), generator=gen, device=dev)
    ent = torch.empty((B,), device=dev)
    fn = lambda i: ctx.cs_softmax_entropy(logits, ent)
    time_loop(fn, 4, stream)
    us = time_loop(fn, 32, stream) * 1e3
    res["softmax_entropy_B%d_V128256" % B] = {"us": us, "GBs": B * 128256 * 4 / (us * 1e-6) / 1e9}
    # joint prompt/model selection at the prompt shape: 8192 tokens, 2048 kept (sequential and coupled arm)
    t = wl.CFG5_TOK
    tok_op = binding_mod.make_op(t["ens"], 5, 1001, t["m_tok"], t["n_tok"])
    y_tok = torch.randn((t["m_tok"],), generator=gen, device=dev)
    Y_ch = torch.randn((t["n_tok"], c.m), generator=gen, device=dev)
    fn = lambda i: ctx.cs_joint_select(tok_op, y_tok, t["k_tok"], st.ffn_op[i % nl], st.ffn_dict[i % nl], st.y[0], c.k)
    time_loop(fn, 4, stream)
    res["joint_select_us_per_call"] = time_loop(fn, 16, stream) * 1e3
    fn = lambda i: ctx.cs_joint_select_coupled(tok_op, y_tok, t["k_tok"], st.ffn_op[i % nl], st.ffn_dict[i % nl], Y_ch, c.k)
    time_loop(fn, 4, stream)
    res["joint_select_coupled_us_per_call"] = time_loop(fn, 16, stream) * 1e3
    # what plain streaming reaches on this device, for context beside the published peak: a 1 GiB
    # device-to-device copy (bytes read + bytes written)
    src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
    dst = torch.empty_like(src)
    fn = lambda i: dst.copy_(src)
    time_loop(fn, 2, stream)
    ms = time_loop(fn, 10, stream)
    res["plain_copy_1GiB"] = {"us": ms * 1e3, "GBs_read_plus_write": 2 * (1 << 30) / (ms * 1e-3) / 1e9}
    del src, dst
    return res


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: this library has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    from paper_2604_14156_amd import binding, workloads as wl
    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU and the HIP library; there is no CPU fallback")
    SOLVER["name"], SOLVER["iters"] = args.solver, args.iht_iters
    global NEXT_GROUPS
    if args.groups is not None:
        NEXT_GROUPS = max(1, args.groups)
    else:
        # on one stream a single group has the fewest launches; beside a second stream the last group's work is
        # carried into the next step, which needs two
        NEXT_GROUPS = 1 if args.recovery_stream == "same" else 2
    torch.cuda.set_device(0)
    stream = torch.cuda.Stream()
    rstream = torch.cuda.Stream()
    ctx = binding.Context(device=0, stream=stream)
    rctx = binding.Context(device=0, stream=rstream)
    # steps with inputs of their own: the timed ones and the last few warm-up steps before them; earlier
    # warm-up steps replay those steps' graphs in turn (every step reads one generation of supports and writes
    # the other, whatever ran before it)
    own_warm = min(args.warmup, 3)
    nsteps = args.steps + own_warm
    if args.prefill_pass:
        with torch.cuda.stream(stream):
            res = prefill_measurements(ctx, wl, stream, binding)
        res["prefill_pass"] = True
        print(json.dumps(res))
        return
    with torch.cuda.stream(stream):
        st = DecodeState(ctx, wl, binding, args.layers, args.batch, nsteps)
        for l in range(args.layers):               # the recovery context keeps its own plans
            rctx.cs_plan(st.ffn_op[l], st.ffn_dict[l], st.psi[l])
            rctx.cs_plan(st.head_op[l], st.head_dict)
        torch.cuda.synchronize()
        if args.counter_pass:
            src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0").fill_(1)
            dst = torch.empty_like(src)
            dst.copy_(src)                           # known traffic: 1 GiB read + 1 GiB written
            torch.cuda.synchronize()
            decode_step(ctx, st, 0)
            torch.cuda.synchronize()
            print(json.dumps({"counter_pass": True, "calibration_copy_bytes": 1 << 30}))
            return
        # one HIP graph per step: the launches of a step (two streams, 8 kernels per layer) are
        # replayed without host work in between
        if args.recovery == "next-step":
            if args.solver != "omp":
                raise SystemExit("--recovery next-step batches the block-OMP solver; use --recovery same-step with --solver iht")
            global NEXT_INLINE
            NEXT_INLINE = args.recovery_stream == "same"
            if not NEXT_INLINE and len(st.groups) < 2:
                raise SystemExit("--groups must be at least 2: the last group's recovery is carried into the next step")
            prime_supports(ctx, st)
            for grp in st.groups:                       # the recovery context builds its device tables now
                recover_group(rctx, st, grp, 1)
            torch.cuda.synchronize()
            step_fn = decode_step_next_inline if NEXT_INLINE else decode_step_next
        else:
            step_fn = decode_step_pipelined
        graphs = None
        if not args.no_graph:
            try:
                graphs = []
                for i in range(nsteps):
                    g = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(g, stream=stream, capture_error_mode="thread_local"):
                        step_fn(ctx, rctx, st, i, stream, rstream)
                    graphs.append(g)
            except Exception as exc:                # fall back to plain launches
                print("graph capture failed (%s); running eager" % exc, file=sys.stderr)
                graphs = None
                torch.cuda.synchronize()

        def run(i):
            if graphs is not None:
                graphs[i].replay()
            else:
                step_fn(ctx, rctx, st, i, stream, rstream)

        # set-up: whatever --warmup says, at least SETTLE_STEPS replays precede the timed region, so that the
        # 60-80 slow steps after the idle gap of the graph capture are not timed
        settle = max(0, SETTLE_STEPS - args.warmup)
        for i in range(settle):
            run(i % nsteps)
        for i in range(args.warmup - own_warm):
            run(i % nsteps)
        for i in range(own_warm):
            run(i)
        torch.cuda.synchronize()
        # --- timed region: exactly `steps` steps
        t0 = time.perf_counter()
        for i in range(args.steps):
            run(own_warm + i)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        # --- after the timed region: the same steps once more with an event between them (spread of
        # the step time), and the execution stream alone (attention + FFN of every layer, no sketches and
        # no recoveries) replayed the same way: net against kernel-only time of a step
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
        marks[0].record(stream)
        for i in range(args.steps):
            run(own_warm + i)
            marks[i + 1].record(stream)
        torch.cuda.synchronize()
        step_ms = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
        pick = lambda q: step_ms[min(len(step_ms) - 1, int(q * len(step_ms)))]
        step_spread = {"p10": pick(0.1), "p50": pick(0.5), "p90": pick(0.9), "note": "one event per step; the timed region has none"}
        verify = None
        if args.recovery == "next-step" and not args.no_verify:
            verify = verify_last_step(ctx, st, wl, own_warm + args.steps - 1)
        exec_only_ms = None
        other_mode_ms = None
        if graphs is not None and args.recovery == "next-step":
            # the step with measurement and recovery on the other stream arrangement (with the number of groups
            # that suits it), replayed the same way
            other_fn = decode_step_next if NEXT_INLINE else decode_step_next_inline
            main_groups = st.groups
            other_groups = st.make_groups(binding, 2 if NEXT_INLINE else 1)
            for grp in other_groups:                      # device tables of both contexts, outside the capture
                recover_group(ctx, st, grp, 1)
                recover_group(rctx, st, grp, 1)
            torch.cuda.synchronize()
            st.groups = other_groups
            og = []
            for i in range(min(4, nsteps)):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=stream, capture_error_mode="thread_local"):
                    other_fn(ctx, rctx, st, i, stream, rstream)
                og.append(g)
            st.groups = main_groups
            for g in og:
                g.replay()
            # The step time drifts by a few per cent with the device's temperature (the first pass on an
            # idle device is the fastest), so the two arrangements are timed in alternation and compared
            # by their medians.
            mine, other = [], []
            for r in range(5):
                mine.append(time_loop(lambda i: graphs[i % len(graphs)].replay(), 8, stream))
                other.append(time_loop(lambda i: og[i % len(og)].replay(), 8, stream))
            other_mode_ms = {"this_arrangement_ms": sorted(mine)[2], "other_arrangement_ms": sorted(other)[2],
                             "this_groups": len(main_groups), "other_groups": len(other_groups),
                             "how": "medians of 5 alternating passes of 8 replayed steps each"}
            del og
        if graphs is not None and args.recovery == "next-step":
            def exec_only(i):
                cur = i % 2
                for l in range(st.layers):
                    ctx.cs_head_attn(st.q[i][l], st.K[l], st.V[l], st.H_gen[cur][l], st.o)
                    ctx.cs_block_ffn(st.Wg[l], st.Wu[l], st.Wd[l], st.x[i][l], st.S_gen[cur][l], False, st.out)
            eg = []
            for i in range(min(4, nsteps)):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=stream, capture_error_mode="thread_local"):
                    exec_only(i)
                eg.append(g)
            for g in eg:
                g.replay()
            exec_only_ms = time_loop(lambda i: eg[i % len(eg)].replay(), 3 * len(eg), stream)
            del eg
        # --- per-call durations: each call type launched back to back over all layers (fresh
        # weights and supports per layer), HIP events on the launching stream around each loop
        per, union_mean = call_loops(ctx, st, stream)
        # active bytes per call
        c, hs = st.c, st.hs
        attn_bytes = args.batch * hs.kh * 2 * hs.L * hs.dh * 2
        # union of the supports of one call stands for all (same distribution)
        # share of the step's recoveries whose selection margin clears the exact-comparison filter (all
        # layers x tokens of the last batched recovery)
        # (same-step mode recovers layer by layer: the margins of the last layer's batch stand for the step)
        margin_pass = float(((st.margin_all if args.recovery == "next-step" else st.margin) > 1e-3).float().mean())
        ffn_bytes = union_mean * 3 * c.b * c.d * 2
        # what a plain streaming read reaches on this device in this run (the K caches of the layers in turn)
        chk = torch.zeros((1,), dtype=torch.int32, device="cuda:0")
        fn = lambda i: ctx.cs_stream_read(st.K[i % st.layers], chk)
        time_loop(fn, st.layers, stream)
        read_ms = time_loop(fn, 2 * st.layers, stream)
        read_ceiling = st.K[0].numel() * 2 / (read_ms * 1e-3) / 1e9
        extra = None if args.no_extra else extra_measurements(ctx, st, wl, stream, binding)
        if extra is not None:
            extra.update(prefill_measurements(ctx, wl, stream, binding))
        torch.cuda.synchronize()

    ms_per_step = wall * 1e3 / args.steps
    tokens_per_s = args.batch / (wall / args.steps)
    calls_per_step = {"sketch": 2 * args.layers, "recover": 2 * args.layers, "attn": args.layers, "ffn": args.layers}
    step_share = {k: per[k] * calls_per_step[k] for k in calls_per_step}
    per_layer_recover_ms = step_share["recover"]
    per_layer_sketch_ms = step_share["sketch"]
    if args.recovery == "next-step":
        step_share["recover"] = per["recover_step_batched"]
        step_share["sketch"] = per["sketch_step_batched"]
    kernels = {
        "attn": {"us_per_call": per["attn"] * 1e3, "active_MB": attn_bytes / 1e6,
                 "GBs": attn_bytes / (per["attn"] * 1e-3) / 1e9,
                 "hbm_frac": attn_bytes / (per["attn"] * 1e-3) / 1e9 / HBM_PEAK_GBS,
                 "traffic": recorded_traffic("cs_head_attn")},
        "ffn": {"us_per_call": per["ffn"] * 1e3, "active_MB": ffn_bytes / 1e6,
                "GBs": ffn_bytes / (per["ffn"] * 1e-3) / 1e9,
                "hbm_frac": ffn_bytes / (per["ffn"] * 1e-3) / 1e9 / HBM_PEAK_GBS,
                "traffic": recorded_traffic("cs_block_ffn")},
        "recover_ffn": {"us_per_call": per["recover_ffn"] * 1e3},
        "recover_heads": {"us_per_call": per["recover_heads"] * 1e3},
        "sketch_ffn": {"us_per_call": per["sketch_ffn"] * 1e3},
        "sketch_heads": {"us_per_call": per["sketch_heads"] * 1e3},
    }
    for kn in ("attn", "ffn"):
        kernels[kn]["frac_of_measured_read_ceiling"] = kernels[kn]["GBs"] / read_ceiling
    dom = "attn" if step_share["attn"] >= step_share["ffn"] else "ffn"
    achieved = kernels[dom]["GBs"]
    rec_frac = step_share["recover"] / sum(step_share.values())
    result = {
        "metric": "decode tokens/s + HBM GB/s on active blocks; recovery us/token (7B-shaped)",
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "settle_steps": settle,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "config 3: full 7B-shaped decode step, %d layers, batch %d, KV length %d, "
                               "supports re-recovered every token" % (args.layers, args.batch, hs.L),
                   "global_batch": args.batch, "layers": args.layers, "kv_len": hs.L,
                   "ffn_blocks_kept": "%d/%d" % (c.k, c.G), "heads_kept": "%d/%d" % (hs.kh, hs.H),
                   "solver": args.solver if args.solver == "omp" else "iht(%d iterations)" % args.iht_iters},
        "roofline": {"bound": "hbm", "kernel": "cs_head_attn" if dom == "attn" else "cs_block_ffn",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": recorded_traffic("cs_head_attn" if dom == "attn" else "cs_block_ffn")},
        # the decode FFN is the call with a stated target (0.70 of the HBM peak on the active blocks)
        "roofline_ffn": {"bound": "hbm", "kernel": "cs_block_ffn", "achieved": kernels["ffn"]["GBs"],
                         "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": kernels["ffn"]["hbm_frac"], "target_frac": 0.70,
                         "traffic": recorded_traffic("cs_block_ffn")},
        "measured_read_ceiling": {"GBs": read_ceiling, "frac_of_peak": read_ceiling / HBM_PEAK_GBS,
                                  "how": "cs_stream_read over the layers' K caches (1.07 GB each) in turn"},
        "step_hbm": {"active_GB_per_step": (attn_bytes + ffn_bytes) * args.layers / 1e9,
                     "GBs": (attn_bytes + ffn_bytes) * args.layers / (ms_per_step * 1e-3) / 1e9,
                     "frac": (attn_bytes + ffn_bytes) * args.layers / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "tokens_per_s_at_peak": args.batch / ((attn_bytes + ffn_bytes) * args.layers / (HBM_PEAK_GBS * 1e9))},
        "oracle_check": verify,
        "kernels": kernels,
        "recovery": {"mode": args.recovery,
                     "us_per_token": step_share["recover"] * 1e3 / args.batch,
                     "ms_per_step": step_share["recover"],
                     "frac_of_serial_step": rec_frac,
                     "frac_of_step_with_sketches": (step_share["recover"] + step_share["sketch"]) / sum(step_share.values()),
                     "ms_per_step_one_call_per_layer": per_layer_recover_ms,
                     "sketch_ms_per_step": step_share["sketch"],
                     "sketch_ms_per_step_one_call_per_layer": per_layer_sketch_ms,
                     "margin_pass_rate": margin_pass,
                     "stream": args.recovery_stream if args.recovery == "next-step" else "second",
                     "note": (("the sketches of step t give the supports step t+1 executes; %d groups of layers are sketched "
                               "and recovered with one launch per group and kind on the execution stream, each right "
                               "after the group's last layer" % len(st.groups)) if NEXT_INLINE else
                              ("the sketches of step t give the supports step t+1 executes; a second stream sketches and "
                               "recovers %d groups of layers with one launch per group and kind, each after the "
                               "execution stream has issued the group's last layer (the last group's work is carried "
                               "to the start of the next step)" % len(st.groups))) if args.recovery == "next-step" else
                             "measurement and recovery run on a second stream up to 4 layers ahead of execution in the same step"},
        "step_ms_spread": step_spread,
        "ms_per_step_execution_only": exec_only_ms,
        "stream_arrangements": None if other_mode_ms is None else {
            ("one_stream_ms" if NEXT_INLINE else "two_streams_ms"): other_mode_ms["this_arrangement_ms"],
            ("two_streams_ms" if NEXT_INLINE else "one_stream_ms"): other_mode_ms["other_arrangement_ms"],
            ("one_stream_groups" if NEXT_INLINE else "two_streams_groups"): other_mode_ms["this_groups"],
            ("two_streams_groups" if NEXT_INLINE else "one_stream_groups"): other_mode_ms["other_groups"],
            "how": other_mode_ms["how"]},
        "measurement_and_recovery_overhead": None if exec_only_ms is None else (ms_per_step - exec_only_ms) / ms_per_step,
        "serial_step_breakdown_ms": step_share,
        "ms_per_step_serial_sum": sum(step_share.values()),
        "launch_mode": "hip_graph" if graphs is not None else "eager",
    }
    if extra is not None:
        result["single_layer"] = extra
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl, B=args.batch)
    ctx.close()
    rctx.close()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
