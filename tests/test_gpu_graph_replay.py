"""A captured two-stream decode step replayed several times must reproduce the eager
results every time (device-side work counters are restored by the kernels themselves,
no memset nodes are recorded)."""
import numpy as np
import pytest
import torch

from paper_2604_14156_amd import binding, workloads as wl
from gpu_util import host

pytestmark = pytest.mark.gpu


def test_pipelined_step_graph_replays_match_eager():
    dev = "cuda:0"
    c = wl.scaled(wl.CFG2, d=512, G=24, k=6, m=64)
    hs = wl.scaled(wl.CFG3_HEADS, L=300)
    B, layers = 5, 3
    s_exec, s_rec = torch.cuda.Stream(), torch.cuda.Stream()
    ctx, rctx = binding.Context(0, s_exec), binding.Context(0, s_rec)
    gen = torch.Generator(device=dev).manual_seed(9)
    bf = torch.bfloat16
    rn = lambda *shape: torch.randn(shape, generator=gen, device=dev)
    with torch.cuda.stream(s_exec):
        Wg = [rn(c.G, c.b, c.d).mul(0.05).to(bf) for _ in range(layers)]
        Wu = [rn(c.G, c.b, c.d).mul(0.05).to(bf) for _ in range(layers)]
        Wd = [rn(c.G, c.d, c.b).mul(0.05).to(bf) for _ in range(layers)]
        K = [rn(B, hs.H, hs.L, hs.dh).to(bf) for _ in range(layers)]
        V = [rn(B, hs.H, hs.L, hs.dh).to(bf) for _ in range(layers)]
        psi = []
        for _ in range(layers):
            p = rn(c.G, c.b)
            psi.append((p / p.norm(dim=1, keepdim=True)).reshape(c.G, c.b, 1).contiguous())
        z = [rn(B, c.n) for _ in range(layers)]
        u = [rn(B, hs.H) for _ in range(layers)]
        x = [rn(B, c.d).to(bf) for _ in range(layers)]
        q = [rn(B, hs.H, hs.dh).to(bf) for _ in range(layers)]
        fop = [binding.make_op(c.ens, 5, 2 * l, c.m, c.n) for l in range(layers)]
        hop = [binding.make_op(hs.ens, 5, 2 * l + 1, hs.m, hs.H) for l in range(layers)]
        fdict = [binding.make_dict(psi[l], c.G, c.b, 1) for l in range(layers)]
        hdict = binding.make_dict(None, hs.H, 1, 1)
        for cx in (ctx, rctx):
            for l in range(layers):
                cx.cs_plan(fop[l], fdict[l], psi[l])
                cx.cs_plan(hop[l], hdict)
        y = [torch.empty((B, c.m), device=dev) for _ in range(layers)]
        yh = [torch.empty((B, hs.m), device=dev) for _ in range(layers)]
        S = [torch.empty((B, c.k), dtype=torch.int32, device=dev) for _ in range(layers)]
        Hh = [torch.empty((B, hs.kh), dtype=torch.int32, device=dev) for _ in range(layers)]
        mg = [torch.empty((B,), device=dev) for _ in range(2 * layers)]
        o = [torch.empty((B, hs.H, hs.dh), device=dev, dtype=bf) for _ in range(layers)]
        out = [torch.empty((B, c.d), device=dev, dtype=bf) for _ in range(layers)]
        torch.cuda.synchronize()

        def step():
            s_rec.wait_stream(s_exec)
            for l in range(layers):
                with torch.cuda.stream(s_rec):
                    rctx.cs_sketch(hop[l], u[l], yh[l])
                    rctx.cs_recover_support(hop[l], hdict, hs.kh, yh[l], Hh[l], None, None, mg[2 * l],
                                            want_coef=False, want_resid=False)
                    rctx.cs_sketch(fop[l], z[l], y[l])
                    rctx.cs_recover_support(fop[l], fdict[l], c.k, y[l], S[l], None, None, mg[2 * l + 1],
                                            want_coef=False, want_resid=False)
                    ready = torch.cuda.Event()
                    ready.record(s_rec)
                with torch.cuda.stream(s_exec):
                    s_exec.wait_event(ready)
                    ctx.cs_head_attn(q[l], K[l], V[l], Hh[l], o[l])
                    ctx.cs_block_ffn(Wg[l], Wu[l], Wd[l], x[l], S[l], False, out[l])
            s_exec.wait_stream(s_rec)

        def snapshot():
            torch.cuda.synchronize()
            return [t.clone() for t in S + Hh + o + out]

        def scribble():
            for t in S + Hh:
                t.fill_(-7)
            for t in o + out:
                t.fill_(3.0)

        step()
        ref = snapshot()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s_exec, capture_error_mode="thread_local"):
            step()
        for rep in range(4):
            scribble()
            torch.cuda.synchronize()
            g.replay()
            got = snapshot()
            for a, b in zip(ref, got):
                assert torch.equal(a, b), rep
            # the library's own eager work in between replays
            ctx.cs_block_ffn(Wg[0], Wu[0], Wd[0], x[0], S[0], False, out[0])
            torch.cuda.synchronize()
            assert torch.equal(out[0], ref[2 * layers + layers + 0])
    ctx.close()
    rctx.close()


def test_next_step_graph_with_batched_recovery_replays_match_eager():
    """The other step shape: execution reads one generation of supports while the second stream sketches a
    group of layers with one launch per kind, after the group has been issued, and recovers it with one
    launch per kind into the other generation; the last group's work opens the next step (cross-stream
    edges in both directions in the middle of the captured step)."""
    dev = "cuda:0"
    c = wl.scaled(wl.CFG2, d=512, G=24, k=6, m=64)
    hs = wl.scaled(wl.CFG3_HEADS, L=200)
    B, layers = 4, 3
    s_exec, s_rec = torch.cuda.Stream(), torch.cuda.Stream()
    ctx, rctx = binding.Context(0, s_exec), binding.Context(0, s_rec)
    gen = torch.Generator(device=dev).manual_seed(11)
    bf = torch.bfloat16
    rn = lambda *shape: torch.randn(shape, generator=gen, device=dev)
    with torch.cuda.stream(s_exec):
        Wg = [rn(c.G, c.b, c.d).mul(0.05).to(bf) for _ in range(layers)]
        Wu = [rn(c.G, c.b, c.d).mul(0.05).to(bf) for _ in range(layers)]
        Wd = [rn(c.G, c.d, c.b).mul(0.05).to(bf) for _ in range(layers)]
        K = [rn(B, hs.H, hs.L, hs.dh).to(bf) for _ in range(layers)]
        V = [rn(B, hs.H, hs.L, hs.dh).to(bf) for _ in range(layers)]
        psi = []
        for _ in range(layers):
            p = rn(c.G, c.b)
            psi.append((p / p.norm(dim=1, keepdim=True)).reshape(c.G, c.b, 1).contiguous())
        z, u = rn(layers, B, c.n), rn(layers, B, hs.H)
        x = [rn(B, c.d).to(bf) for _ in range(layers)]
        q = [rn(B, hs.H, hs.dh).to(bf) for _ in range(layers)]
        fop = [binding.make_op(c.ens, 6, 2 * l, c.m, c.n) for l in range(layers)]
        hop = [binding.make_op(hs.ens, 6, 2 * l + 1, hs.m, hs.H) for l in range(layers)]
        fdict = [binding.make_dict(psi[l], c.G, c.b, 1) for l in range(layers)]
        hdict = [binding.make_dict(None, hs.H, 1, 1) for _ in range(layers)]
        Y = torch.empty((layers, B, c.m), device=dev)
        Yh = torch.empty((layers, B, hs.m), device=dev)
        S = [torch.zeros((layers, B, c.k), dtype=torch.int32, device=dev) for _ in range(2)]
        Hh = [torch.zeros((layers, B, hs.kh), dtype=torch.int32, device=dev) for _ in range(2)]
        mg = torch.empty((2, layers, B), device=dev)
        o = [torch.empty((B, hs.H, hs.dh), device=dev, dtype=bf) for _ in range(layers)]
        out = [torch.empty((B, c.d), device=dev, dtype=bf) for _ in range(layers)]

        def recover_rows(cx, gen_idx, l0, l1):
            cx.cs_recover_support_multi(hop[l0:l1], hdict[l0:l1], hs.kh, Yh[l0:l1], Hh[gen_idx][l0:l1], None, None,
                                        mg[0][l0:l1], want_coef=False, want_resid=False)
            cx.cs_recover_support_multi(fop[l0:l1], fdict[l0:l1], c.k, Y[l0:l1], S[gen_idx][l0:l1], None, None,
                                        mg[1][l0:l1], want_coef=False, want_resid=False)

        def sketch_rows(cx, l0, l1):
            cx.cs_sketch_multi(hop[l0:l1], u[l0:l1], Yh[l0:l1])
            cx.cs_sketch_multi(fop[l0:l1], z[l0:l1], Y[l0:l1])

        # generation 0 from the sketches themselves (eager, first stream), device tables of both contexts
        cut = layers - 1                       # two groups of layers: [0, cut) and the last layer
        for l in range(layers):
            ctx.cs_sketch(hop[l], u[l], Yh[l])
            ctx.cs_sketch(fop[l], z[l], Y[l])
        recover_rows(ctx, 0, 0, cut)
        recover_rows(ctx, 0, cut, layers)
        torch.cuda.synchronize()
        with torch.cuda.stream(s_rec):
            recover_rows(rctx, 1, 0, cut)
            recover_rows(rctx, 1, cut, layers)
        torch.cuda.synchronize()
        S0_ref, H0_ref = S[0].clone(), Hh[0].clone()

        def run_layer(l):
            ctx.cs_head_attn(q[l], K[l], V[l], Hh[0][l], o[l])
            ctx.cs_block_ffn(Wg[l], Wu[l], Wd[l], x[l], S[0][l], False, out[l])

        def step():
            # the last group's measurement and recovery (carried over from the step before) open the step
            # on the second stream and fill generation 0, which the last layer reads after a wait; the
            # first group is measured once its layers have been issued and fills generation 1
            s_rec.wait_stream(s_exec)
            with torch.cuda.stream(s_rec):
                sketch_rows(rctx, cut, layers)
                recover_rows(rctx, 0, cut, layers)
                carried = torch.cuda.Event()
                carried.record(s_rec)
            with torch.cuda.stream(s_exec):
                for l in range(cut):
                    run_layer(l)
                issued = torch.cuda.Event()
                issued.record(s_exec)
            with torch.cuda.stream(s_rec):
                s_rec.wait_event(issued)
                sketch_rows(rctx, 0, cut)
                recover_rows(rctx, 1, 0, cut)
            with torch.cuda.stream(s_exec):
                s_exec.wait_event(carried)
                for l in range(cut, layers):
                    run_layer(l)
            s_exec.wait_stream(s_rec)

        def snapshot():
            torch.cuda.synchronize()
            return [t.clone() for t in [S[1][:cut], Hh[1][:cut], S[0], Hh[0], Y, Yh] + o + out]

        step()
        ref = snapshot()
        assert torch.equal(ref[0], S0_ref[:cut]) and torch.equal(ref[1], H0_ref[:cut])      # same sketches, same supports
        assert torch.equal(ref[2], S0_ref) and torch.equal(ref[3], H0_ref)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s_exec, capture_error_mode="thread_local"):
            step()
        for rep in range(4):
            S[1].fill_(-7); Hh[1].fill_(-7); Y.fill_(0.5); Yh.fill_(0.5)
            S[0][cut:].fill_(-7); Hh[0][cut:].fill_(-7)             # the step itself refills these before the last layer reads them
            for t in o + out:
                t.fill_(3.0)
            torch.cuda.synchronize()
            g.replay()
            got = snapshot()
            for a, b in zip(ref, got):
                assert torch.equal(a, b), rep
            ctx.cs_recover_support_multi(fop, fdict, c.k, Y, S[1], None, None, mg[1], want_coef=False, want_resid=False)
            torch.cuda.synchronize()
            assert torch.equal(S[1], S0_ref)

        # the benchmark's default arrangement: everything on the execution stream, a group measured and
        # recovered (into the generation the next step reads) right after its last layer
        def step_one_stream():
            for l0, l1 in ((0, cut), (cut, layers)):
                for l in range(l0, l1):
                    run_layer(l)
                sketch_rows(ctx, l0, l1)
                recover_rows(ctx, 1, l0, l1)

        step_one_stream()
        ref1 = [t.clone() for t in [S[1], Hh[1], Y, Yh] + o + out]
        torch.cuda.synchronize()
        assert torch.equal(ref1[0], S0_ref) and torch.equal(ref1[1], H0_ref)
        g1 = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g1, stream=s_exec, capture_error_mode="thread_local"):
            step_one_stream()
        for rep in range(3):
            S[1].fill_(-7); Hh[1].fill_(-7); Y.fill_(0.5); Yh.fill_(0.5)
            for t in o + out:
                t.fill_(3.0)
            torch.cuda.synchronize()
            g1.replay()
            torch.cuda.synchronize()
            for a, b in zip(ref1, [S[1], Hh[1], Y, Yh] + o + out):
                assert torch.equal(a, b), rep
            ctx.cs_head_attn(q[0], K[0], V[0], Hh[0][0], o[0])              # eager work between the replays
            torch.cuda.synchronize()
    ctx.close()
    rctx.close()
