"""GPU parity of the rows beyond the core path: the ablation orderings of Sec. 6.3 (bit-exact against the
oracle), attention recall of Eq. 3 (against the oracle's definition), and a run of the paper's step
schedule (Sec. 6.1) through the one-call entry point."""
import math

import numpy as np
import pytest
import torch

from oracle import dfs_oracle as O
from workloads import Workload, derived_sizes, make_qkv
from workloads.synth import as_f64

pytestmark = pytest.mark.gpu

P = pytest.importorskip("paper_2605_23445_amd")
from tests import gpu_util as G  # noqa: E402

ORDER_ID = {"hilbert3d": P.DFS_ORDER_HILBERT3D, "raster": P.DFS_ORDER_RASTER, "hilbert2d": P.DFS_ORDER_HILBERT2D,
            "block3d": P.DFS_ORDER_BLOCK3D}


@pytest.mark.parametrize("kind", list(ORDER_ID))
@pytest.mark.parametrize("T,H,W,n_text,B", [(4, 8, 8, 0, 64), (13, 30, 45, 0, 128), (33, 45, 80, 256, 128), (3, 5, 7, 9, 64),
                                            (1, 1, 1, 0, 64), (9, 2, 130, 1, 128)])
def test_token_orders_bit_exact(kind, T, H, W, n_text, B):
    print(f"order {kind} {T}x{H}x{W}+{n_text}", flush=True)
    g = P.Geom(T, H, W, n_text, 1, 64, B, B)
    s = P.dfs_geom_sizes(g)
    perm_pad = torch.full((s.N_pad,), -7, dtype=torch.int32, device="cuda")
    inv = torch.full((s.N,), -7, dtype=torch.int32, device="cuda")
    blk_valid = torch.full((s.M,), -7, dtype=torch.int32, device="cuda")
    ws = G.ws_tensor(P.dfs_workspace_bytes(g, P.DFS_WS_HILBERT_PERM))
    P.dfs_token_order(g, ORDER_ID[kind], perm_pad, inv, blk_valid, ws)
    want = O.token_order(kind, T, H, W, n_text, B)
    for got, exp in zip((perm_pad, inv, blk_valid), want):
        assert np.array_equal(got.cpu().numpy(), exp)


def test_recall_against_the_definition():
    w = Workload("recall_mid", 4, 10, 12, heads=3, d=128, dtype="bf16", B=128, Bs=32, sparsity=(0.5,), seed=31, n_text=20)
    sz = derived_sizes(w)
    g, dt = G.geom_of(w), G.dtype_of(w)
    q, k, v = make_qkv(w)
    perm_pad, inv, blk_valid_d = G.gpu_perm(g)
    blk_valid = blk_valid_d.cpu().numpy()
    qp, kp, vp = (G.gpu_permute(g, dt, G.to_dev(x), perm_pad) for x in (q, k, v))
    score = G.gpu_score(g, dt, qp, kp)
    dense = G.gpu_select(g, score, P.DFS_SELECT_TOPK, 0.0)
    _, lse_d = G.gpu_attn(g, dt, qp, kp, vp, dense)
    recall = torch.empty(w.heads, dtype=torch.float32, device="cuda")
    P.dfs_recall(g, lse_d, lse_d, recall)
    assert np.allclose(recall.cpu().numpy(), 1.0, atol=1e-6)
    prev = None
    for sp in (0.25, 0.5, 0.75):
        st = G.gpu_select(g, score, P.DFS_SELECT_TOPK, sp)
        _, lse_s = G.gpu_attn(g, dt, qp, kp, vp, st)
        P.dfs_recall(g, lse_s, lse_d, recall)
        got = recall.cpu().numpy()
        want = O.attention_recall(G.as_f64_dev(qp), G.as_f64_dev(kp), st.mask.cpu().numpy(), blk_valid, w.B)
        print(f"  sparsity {sp}: recall {got} oracle {want}", flush=True)
        # recall = mean of exp(lse_sparse - lse_dense) <= 1: an lse good to 1e-4 (the parity bound) moves it by
        # at most 2e-4; the mean over the rows is taken in fp32
        assert np.abs(got - want).max() <= 2e-4
        assert np.all(got > 1.0 - sp)                            # kept blocks hold more than their share
        if prev is not None:
            assert np.all(got <= prev + 1e-3)                    # fewer kept blocks, less mass
        prev = got


def test_paper_schedule_run():
    """A short sampling run under the paper's schedule: dense first quarter, then keep 0.3 / 0.2 / 0.1 with the
    mask refreshed when the schedule says so; every step's output is checked against the oracle under the mask
    in force."""
    w = Workload("sched_mid", 4, 8, 16, heads=2, d=64, dtype="bf16", B=128, Bs=32, sparsity=(0.7,), seed=41)
    sz = derived_sizes(w)
    g, dt = G.geom_of(w), G.dtype_of(w)
    q, k, v = make_qkv(w)
    perm_pad, inv, blk_valid_d = G.gpu_perm(g)
    blk_valid = blk_valid_d.cpu().numpy()
    inv_np = inv.cpu().numpy()
    qd, kd, vd = (G.to_dev(x) for x in (q, k, v))
    K_max = sz["M"]
    st = P.MaskState(torch.zeros((w.heads, sz["M"], K_max), dtype=torch.int32, device="cuda"),
                     torch.zeros((w.heads, sz["M"]), dtype=torch.int32, device="cuda"),
                     torch.zeros((w.heads, sz["M"], sz["M"]), dtype=torch.uint8, device="cuda"), None, K_max)
    ws = G.ws_tensor(P.dfs_workspace_bytes(g, P.DFS_WS_FORWARD_BF16))
    o = torch.empty_like(qd)
    total, delta, cached, log = 8, 3, None, []
    for t in range(total):
        dense, refresh, sp = P.dfs_schedule(total, t, delta, cached)
        assert (dense, refresh, round(sp, 9)) == tuple(round(x, 9) if isinstance(x, float) else x for x in O.paper_schedule(total, t, delta, cached_keep=cached))
        kd = torch.roll(kd, 1, dims=1).contiguous()              # the inputs change every step
        if dense:
            # dense bypass: all blocks kept; the cached sparse mask (none yet) is left alone
            all_st = P.MaskState(torch.zeros_like(st.kv_idx), torch.zeros_like(st.kv_cnt), torch.zeros_like(st.mask), None, K_max)
            P.dfs_forward(g, dt, qd, kd, vd, perm_pad, inv, True, P.DFS_SELECT_TOPK, 0.0, 0.0, all_st, 1 / math.sqrt(w.d), o, ws)
            mask = all_st.mask.cpu().numpy()
        else:
            P.dfs_forward(g, dt, qd, kd, vd, perm_pad, inv, refresh, P.DFS_SELECT_TOPK, sp, 0.0, st, 1 / math.sqrt(w.d), o, ws)
            if refresh:
                cached = 1.0 - sp
            mask = st.mask.cpu().numpy()
            assert np.all(mask[:, :sz["M_v"], :sz["M_v"]].sum(axis=2) == P.dfs_keep_count(1.0 - cached, sz["M_v"]))
        log.append((dense, refresh, round(sp, 3)))
        kp = G.gpu_permute(g, dt, kd, perm_pad); qp = G.gpu_permute(g, dt, qd, perm_pad); vp = G.gpu_permute(g, dt, vd, perm_pad)
        want, _ = O.sparse_attn(G.as_f64_dev(qp), G.as_f64_dev(kp), G.as_f64_dev(vp), mask, blk_valid, w.B)
        err = np.abs(G.as_f64_dev(o) - O.unpermute(want, inv_np))
        assert err.max() <= 2e-2 and err.mean() <= 2e-3
    print("  schedule:", log, flush=True)
    assert [d for d, _, _ in log] == [True, True, False, False, False, False, False, False]
    assert [s for _, _, s in log[2:]] == [0.7, 0.7, 0.8, 0.8, 0.9, 0.9]
    assert [r for _, r, _ in log[2:]] == [True, True, True, False, True, False]


def test_attention_clock_probe_counts_every_work_group():
    """The measurement diagnostic: with the probe set, every (head, query block) work-group of the bf16
    attention kernel reports once, the output is unchanged, and the clock ratio is a plausible shader clock."""
    w = Workload("probe", 5, 12, 20, heads=3, d=128, dtype="bf16", B=128, Bs=32, sparsity=(0.6,), seed=5)
    sz = derived_sizes(w)
    g, dt = G.geom_of(w), G.dtype_of(w)
    q, k, v = make_qkv(w)
    perm_pad, inv, _ = G.gpu_perm(g)
    qp, kp, vp = (G.gpu_permute(g, dt, G.to_dev(x), perm_pad) for x in (q, k, v))
    st = G.gpu_select(g, G.gpu_score(g, dt, qp, kp), P.DFS_SELECT_TOPK, 0.6)
    o_ref, _ = G.gpu_attn(g, dt, qp, kp, vp, st)
    probe = torch.zeros(3, dtype=torch.int64, device="cuda")
    P.dfs_attn_clock_probe(probe)
    try:
        o_probe, _ = G.gpu_attn(g, dt, qp, kp, vp, st)
        torch.cuda.synchronize()
    finally:
        P.dfs_attn_clock_probe(None)
    cycles, ticks, groups = (int(x) for x in probe.cpu())
    assert groups == w.heads * sz["M"]
    assert torch.equal(o_ref.view(torch.int16), o_probe.view(torch.int16))
    assert ticks > 0 and 300.0 < cycles / ticks * 100.0 < 3000.0
    o_again, _ = G.gpu_attn(g, dt, qp, kp, vp, st)
    torch.cuda.synchronize()
    assert int(probe.cpu()[2]) == groups          # switched off again


def test_measurement_probes_run_and_report_sane_rates():
    """The probes behind `bench.py --probe`: a short matrix-instruction chain, a copy and a read-only pass."""
    sink = torch.empty(64 * 256, dtype=torch.float32, device="cuda")
    counters = torch.zeros(2, dtype=torch.int64, device="cuda")
    P.dfs_probe_mfma(64, 2000, sink, counters)
    torch.cuda.synchronize()
    cycles, ticks = (int(x) for x in counters.cpu())
    assert torch.isfinite(sink).all()
    assert ticks > 0 and 300.0 < cycles / ticks * 100.0 < 3000.0            # a plausible shader clock in MHz
    assert 28.0 < cycles / (2000 * 4) < 80.0                                 # about 32 cycles per matrix instruction
    src = torch.arange(1 << 20, dtype=torch.int32, device="cuda")
    dst = torch.zeros_like(src)
    P.dfs_probe_copy(src, dst)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    with pytest.raises(P.DfsError):
        P.dfs_probe_mfma(0, 10, sink, None)
    region = torch.ones(4 << 20, dtype=torch.uint8, device="cuda")
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    P.dfs_probe_read(region, 64, 8, flag)
    torch.cuda.synchronize()
    assert int(flag) == 0                                                     # all-ones words cancel in the checksum
    with pytest.raises(P.DfsError):
        P.dfs_probe_read(region[:1000], 64, 8, flag)                          # not a multiple of 64 KB


def test_whole_step_under_graph_capture_replays_bit_identical():
    """The library neither allocates, copies, clears memory with the runtime, nor waits: a whole step (token order,
    V reorder, fused scoring with the K reorder, selection through the built-in scratch, attention written in
    source order) and the one-call entry point are each captured into a HIP graph and replayed four times on inputs
    that change between replays, with eager runs of the same calls and synchronisations in between; every replay
    must equal the eager run bit for bit."""
    w = Workload("graph_mid", 5, 12, 20, heads=3, d=128, dtype="bf16", B=128, Bs=32, sparsity=(0.6,), seed=77, n_text=70)
    sz = derived_sizes(w)
    g, dt = G.geom_of(w), G.dtype_of(w)
    q, k, v = make_qkv(w)
    qd, kd, vd = (G.to_dev(x) for x in (q, k, v))
    s = P.dfs_geom_sizes(g)
    i32 = dict(dtype=torch.int32, device="cuda")
    K_max, scale = sz["M"], 1 / math.sqrt(w.d)
    ws = G.ws_tensor(max(P.dfs_workspace_bytes(g, c) for c in (P.DFS_WS_HILBERT_PERM, P.DFS_WS_BLOCK_SCORE, P.DFS_WS_FORWARD_BF16)))

    class Bufs:
        def __init__(self):
            self.perm_pad, self.inv, self.bv = torch.zeros(s.N_pad, **i32), torch.zeros(s.N, **i32), torch.zeros(s.M, **i32)
            self.kp = torch.zeros((w.heads, s.N_pad, w.d), dtype=torch.bfloat16, device="cuda")
            self.vp = torch.zeros_like(self.kp)
            self.score = torch.zeros((w.heads, s.M_v, s.M_v), device="cuda")
            self.st = P.MaskState(torch.zeros((w.heads, s.M, K_max), **i32), torch.zeros((w.heads, s.M), **i32),
                                  torch.zeros((w.heads, s.M, s.M), dtype=torch.uint8, device="cuda"),
                                  torch.zeros(w.heads, **i32), K_max)
            self.o, self.o1 = torch.zeros_like(qd), torch.zeros_like(qd)

    def step(b, mode, sparsity, mass):
        P.dfs_hilbert_perm(g, b.perm_pad, b.inv, b.bv, ws)
        P.dfs_permute(g, dt, vd, b.perm_pad, b.vp)
        P.dfs_block_score_fused(g, dt, qd, kd, b.perm_pad, b.kp, b.score, ws)
        P.dfs_select_mask_static(g, b.score, mode, sparsity, mass, b.st.mask, b.st.kv_idx, b.st.kv_cnt, K_max, b.st.k_head)
        P.dfs_sparse_attn_fwd_src(g, dt, qd, b.perm_pad, b.kp, b.vp, b.st.kv_idx, b.st.kv_cnt, K_max, scale, b.o)
        P.dfs_forward(g, dt, qd, kd, vd, b.perm_pad, b.inv, True, mode, sparsity, mass, b.st, scale, b.o1, ws)

    for mode, sparsity, mass in ((P.DFS_SELECT_TOPK, 0.6, 0.0), (P.DFS_SELECT_MASS_HEAD, 0.9, 0.8)):
        eager, cap = Bufs(), Bufs()
        step(eager, mode, sparsity, mass)                      # also looks up the built-in scratch outside the capture
        torch.cuda.synchronize()
        graph, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
        with torch.cuda.graph(graph, stream=side):
            step(cap, mode, sparsity, mass)
        for rep in range(4):
            kd.copy_(torch.roll(kd, 7 + rep, dims=1)); qd.copy_(torch.roll(qd, 3, dims=0))   # inputs change in place
            step(eager, mode, sparsity, mass)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            for name in ("perm_pad", "inv", "bv", "kp", "vp", "score", "o", "o1"):
                assert torch.equal(getattr(eager, name), getattr(cap, name)), (mode, rep, name)
            assert torch.equal(eager.st.kv_cnt, cap.st.kv_cnt) and torch.equal(eager.st.mask, cap.st.mask), (mode, rep)
            assert torch.equal(eager.st.k_head, cap.st.k_head) or mode == P.DFS_SELECT_TOPK
            assert torch.equal(eager.o, eager.o1), "one-call entry point and staged calls differ"
            assert bool(torch.isfinite(cap.o.float()).all())


def test_two_streams_share_no_hidden_state():
    """Two one-call forwards on two streams at the same time, each with its own inputs, mask state, workspace and
    output: each must give bit for bit what it gives alone (the library keeps no state between calls besides what the
    caller passes in)."""
    w = Workload("streams_mid", 5, 12, 20, heads=3, d=128, dtype="bf16", B=128, Bs=32, sparsity=(0.6,), seed=91)
    sz = derived_sizes(w)
    g, dt = G.geom_of(w), G.dtype_of(w)
    q, k, v = make_qkv(w)
    perm_pad, inv, _ = G.gpu_perm(g)
    i32 = dict(dtype=torch.int32, device="cuda")
    K_max, scale = sz["M"], 1 / math.sqrt(w.d)

    class Job:
        def __init__(self, shift):
            self.q, self.k, self.v = (torch.roll(G.to_dev(x), shift, dims=1).contiguous() for x in (q, k, v))
            self.st = P.MaskState(torch.zeros((w.heads, sz["M"], K_max), **i32), torch.zeros((w.heads, sz["M"]), **i32),
                                  torch.zeros((w.heads, sz["M"], sz["M"]), dtype=torch.uint8, device="cuda"), None, K_max)
            self.ws = G.ws_tensor(P.dfs_workspace_bytes(g, P.DFS_WS_FORWARD_BF16))
            self.o = torch.zeros_like(self.q)

        def run(self, sparsity):
            P.dfs_forward(g, dt, self.q, self.k, self.v, perm_pad, inv, True, P.DFS_SELECT_TOPK, sparsity, 0.0, self.st, scale, self.o, self.ws)

    alone = [Job(0), Job(37)]
    alone[0].run(0.6); alone[1].run(0.8)
    torch.cuda.synchronize()
    both = [Job(0), Job(37)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    for rep in range(3):
        for job, stream, sp in zip(both, streams, (0.6, 0.8)):
            with torch.cuda.stream(stream):
                job.run(sp)
    torch.cuda.synchronize()
    for a, b in zip(alone, both):
        assert torch.equal(a.o, b.o) and torch.equal(a.st.kv_cnt, b.st.kv_cnt) and torch.equal(a.st.mask, b.st.mask)
