"""GPU tests of pipelined calls: large bf16 batches are cut into segments of tiles, and the
walk over a segment's load-dependent tokens runs inside the gate kernel while the later
segments are still being projected (Algorithm 1 orders the tokens of a batch, so a segment
needs nothing of the tokens behind it).  The results must not depend on the segmentation:
every case is compared with the oracle and with the same call run in one piece.  Small
segments (`pipeline_tiles` of a few tiles) put many segment boundaries into small batches."""
from __future__ import annotations

import numpy as np
import pytest

from synth import workloads as wl

pytestmark = pytest.mark.gpu


def _util():
    import gpu_util
    return gpu_util


def _mixed_gate(seed, T, H, E, flat_frac, flat_tiles=None):
    """Zipf-biased rows (decided by the top-k mass test) with a share of flat rows (which
    go to the load-aware branch); flat_tiles: restrict the flat rows to these tiles."""
    rng = np.random.default_rng(seed)
    rank_of = rng.permutation(E) + 1
    zipf = (-1.3 * np.log(rank_of)).astype(np.float32)
    flat = rng.random(T) < flat_frac
    if flat_tiles is not None:
        allowed = np.zeros(T, dtype=bool)
        for t in flat_tiles:
            allowed[t * 64:(t + 1) * 64] = True
        flat &= allowed
    bias = np.where(flat[:, None], np.float32(0.0), zipf[None, :]).astype(np.float32)
    natural = 0.02 * np.sqrt(H)
    sigma = np.where(flat, np.float32(0.05 / natural), np.float32(1.0)).astype(np.float32)
    hidden, w = wl.make_gate(rng, T, H, E, wl.DTYPE_BF16, bias=bias, sigma=sigma)
    return hidden, w, flat


def _same(a, b, label):
    for key in ("expert_ids", "loads", "expert_offsets", "permutation", "weights", "logits"):
        assert np.array_equal(a[key], b[key]), f"{label}: {key} depends on the segmentation"


CASES = [
    # T, H, E, k, c, share of flat rows, tiles per segment
    (1000, 512, 64, 6, 8, 0.10, 2),
    (1000, 512, 64, 6, 8, 0.10, 5),
    (4097, 256, 64, 6, 8, 0.50, 3),     # window evaluation in every segment, ragged last tile
    (4097, 256, 64, 6, 8, 0.50, 17),
    (3000, 512, 8, 2, 4, 0.30, 4),
    (3000, 512, 8, 2, 4, 1.00, 7),      # every token load-dependent
    (2048, 256, 16, 4, 12, 0.20, 8),
    (2500, 1000, 33, 3, 9, 0.40, 6),
    (130, 2048, 64, 6, 8, 0.30, 2),     # two segments, the second one ragged tile only
    (6000, 128, 64, 6, 8, 0.90, 31),
]


@pytest.mark.parametrize("T,H,E,k,c,frac,seg", CASES)
def test_segmented_calls_against_oracle(T, H, E, k, c, frac, seg):
    u = _util()
    hidden, w, flat = _mixed_gate(T + 7 * seg, T, H, E, frac)
    loads = np.random.default_rng(seg).integers(0, 9, E).astype(np.int32)
    eps, tfix = 0.9, 0.05
    gpu, ref = u.check_route(hidden, w, wl.DTYPE_BF16, k, c, eps, tfix, loads,
                             label=f"seg{seg} T{T} E{E}", pipeline_tiles=seg)
    if frac > 0:
        assert ref["expanded"].any()
    whole = u.run_route(hidden, w, wl.DTYPE_BF16, k, c, eps, tfix, loads, pipeline_tiles=1)
    _same(gpu, whole, f"seg{seg} T{T} E{E}")


@pytest.mark.parametrize("flat_tiles", [
    [],                       # no load-dependent token anywhere
    [0],                      # only in the first segment
    [9, 10, 11],              # only in one middle segment (segments of 3 tiles: tiles 9..11)
    [3, 4, 20],               # segments without any in between
    [22],                     # only in the last, ragged segment
    [-5],                     # a handful of load-dependent tokens in one tile
])
def test_segments_with_and_without_flexible_tokens(flat_tiles):
    u = _util()
    T, H, E, k, c = 23 * 64 - 11, 256, 64, 6, 8
    few = flat_tiles == [-5]
    hidden, w, flat = _mixed_gate(99 + len(flat_tiles), T, H, E, 0.06 if few else 0.8,
                                  [5] if few else flat_tiles)
    assert not few or 1 <= flat.sum() <= 8
    loads = np.arange(E, dtype=np.int32) % 5
    # (Zipf rows pass the top-k mass test at 0.40 but for a few; with no flat rows the
    # threshold is lowered until every token keeps its top-k)
    eps, tfix = (0.40, 0.80) if flat_tiles else (1e-6, 0.80)
    gpu, ref = u.check_route(hidden, w, wl.DTYPE_BF16, k, c, eps, tfix, loads,
                             label=f"flat tiles {flat_tiles}", pipeline_tiles=3)
    flexible = (ref["expanded"] != 0) & (ref["cstar"] > k)
    assert bool(flexible.any()) == bool(flat_tiles)
    if flat_tiles:
        assert flexible[flat].mean() > 0.5 and flexible[~flat].mean() < 0.1
    whole = u.run_route(hidden, w, wl.DTYPE_BF16, k, c, eps, tfix, loads, pipeline_tiles=1)
    _same(gpu, whole, f"flat tiles {flat_tiles}")


@pytest.mark.parametrize("nflex", [31, 32, 33, 64, 96, 255, 256, 257])
def test_flexible_token_counts_around_word_boundaries(nflex):
    """The flexible tokens of a segment are numbered from a multiple of 32; counts of
    exactly one or several words per segment are the edge of that numbering."""
    u = _util()
    T, H, E, k, c = 16 * 64, 256, 64, 6, 8
    rng = np.random.default_rng(nflex)
    rank_of = rng.permutation(E) + 1
    zipf = (-1.3 * np.log(rank_of)).astype(np.float32)
    flat = np.zeros(T, dtype=bool)
    # nflex flat rows in each segment of 4 tiles (256 tokens), at random places
    for s0 in range(0, T, 256):
        flat[s0 + rng.permutation(256)[:nflex]] = True
    bias = np.where(flat[:, None], np.float32(0.0), zipf[None, :]).astype(np.float32)
    sigma = np.where(flat, np.float32(0.05 / (0.02 * np.sqrt(H))), np.float32(1.0)).astype(np.float32)
    hidden, w = wl.make_gate(rng, T, H, E, wl.DTYPE_BF16, bias=bias, sigma=sigma)
    loads = np.zeros(E, dtype=np.int32)
    gpu, ref = u.check_route(hidden, w, wl.DTYPE_BF16, k, c, 0.40, 0.80, loads,
                             label=f"{nflex} per segment", pipeline_tiles=4)
    flexible = (ref["expanded"] != 0) & (ref["cstar"] > k)
    assert flexible[flat].mean() > 0.5
    whole = u.run_route(hidden, w, wl.DTYPE_BF16, k, c, 0.40, 0.80, loads, pipeline_tiles=1)
    _same(gpu, whole, f"{nflex} per segment")


def test_default_segmentation_of_a_large_batch():
    """98 304 tokens (six rounds of the persistent grid and a few tiles): pipelined by the
    library's own choice -- a segment of one round, two of two, a short last one --
    compared with the oracle and with the call in one piece."""
    u = _util()
    T, H, E, k, c = 98304, 256, 64, 6, 8
    hidden, w, flat = _mixed_gate(5, T, H, E, 0.10)
    loads = np.zeros(E, dtype=np.int32)
    rows = np.random.default_rng(2).choice(T, size=2048, replace=False)
    gpu, ref = u.check_route(hidden, w, wl.DTYPE_BF16, k, c, 0.40, 0.80, loads,
                             label="T98304 default", logit_rows=rows)
    assert 0.05 < ref["expanded"].mean() < 0.2
    whole = u.run_route(hidden, w, wl.DTYPE_BF16, k, c, 0.40, 0.80, loads, pipeline_tiles=1)
    _same(gpu, whole, "T98304 default")


def test_segmented_call_twice_on_one_workspace():
    """The counters a pipelined call keeps in the workspace are cleared by the call itself:
    a second call on the same buffers (other thresholds, so other segments hold the
    flexible tokens) gives the oracle's result again."""
    import torch
    from paper_2510_03293_amd import binding as B
    import oracle
    u = _util()
    T, H, E, k, c = 3000, 256, 64, 6, 8
    hidden, w, flat = _mixed_gate(17, T, H, E, 0.3)
    hd, wd = u.to_device(hidden), u.to_device(w)
    buf = None
    for eps, tfix, seg in [(0.9, 0.05, 5), (0.4, 0.5, 3), (2.0, 1e-30, 9)]:
        params = B.make_params(k, c, eps, tfix, pipeline_tiles=seg)
        loads = torch.zeros(E, dtype=torch.int32, device="cuda")
        if buf is None:
            buf = B.RouteBuffers(T, H, E, params, want_logits=True)
        B.laser_route(hd, wd, T, H, E, params, loads, buf.expert_ids, buf.weights, buf.permutation,
                      buf.expert_offsets, buf.logits, buf.workspace)
        torch.cuda.synchronize()
        gpu = u._collect(buf, loads, buf.logits)
        ref = oracle.route(gpu["logits"], k, c, eps, tfix, np.zeros(E, dtype=np.int32), True)
        u.assert_discrete_equal(gpu, ref, f"second call eps {eps}")


@pytest.mark.parametrize("T,H,E,k,c,seg", [(3000, 2048, 64, 6, 8, 5), (1500, 512, 8, 2, 4, 3), (2100, 4096, 33, 3, 9, 7)])
def test_segmented_call_with_statistics(T, H, E, k, c, seg):
    """laser_route_stats is pipelined like laser_route: routing against the oracle, the
    statistics bit-equal to those of the call in one piece (which test_token_statistics
    checks against the oracle's)."""
    import oracle
    u = _util()
    hidden, w, flat = _mixed_gate(T + seg, T, H, E, 0.3)
    loads = np.zeros(E, dtype=np.int32)
    eps, tfix = 0.40, 0.80
    gpu = u.run_route_stats(hidden, w, wl.DTYPE_BF16, k, c, eps, tfix, loads, pipeline_tiles=seg)
    ref = oracle.route(gpu["logits"], k, c, eps, tfix, loads, True)
    u.assert_discrete_equal(gpu, ref, f"stats seg{seg}")
    whole = u.run_route_stats(hidden, w, wl.DTYPE_BF16, k, c, eps, tfix, loads, pipeline_tiles=1)
    _same(gpu, whole, f"stats seg{seg}")
    for key in ("topk_mass", "entropy", "pool_size"):
        assert np.array_equal(gpu[key], whole[key]), key


def test_pipelined_calls_side_by_side_on_two_streams():
    """Two pipelined calls at the same time: each brings a persistent grid that wants every
    compute unit, and a chain workgroup that waits (bounded) for its own grid's tiles.
    Whatever the hardware interleaves, both calls finish and give what they give alone."""
    import torch
    from paper_2510_03293_amd import binding as B
    u = _util()
    T, H, E, k, c = 20000, 256, 64, 6, 8          # 313 tiles: more than one round of workgroups
    params = B.make_params(k, c, 0.40, 0.80, dtype=wl.DTYPE_BF16, pipeline_tiles=40)
    prob = []
    for i in range(4):
        h, w, _ = _mixed_gate(300 + i, T, H, E, 0.2)
        prob.append((u.to_device(h), u.to_device(w)))

    def run(streams):
        bufs = [B.RouteBuffers(T, H, E, params) for _ in prob]
        loads = [torch.zeros(E, dtype=torch.int32, device="cuda") for _ in prob]
        torch.cuda.synchronize()
        for rep in range(3):
            for i, (hd, wd) in enumerate(prob):
                st = streams[i % len(streams)]
                B.laser_route(hd, wd, T, H, E, params, loads[i], bufs[i].expert_ids, bufs[i].weights,
                              bufs[i].permutation, bufs[i].expert_offsets, None, bufs[i].workspace, st)
        torch.cuda.synchronize()
        for b in bufs:
            assert B.laser_status(b.workspace) == B.STATUS_COMPLETE
        return [(b.expert_ids.clone(), b.permutation.clone(), l.clone()) for b, l in zip(bufs, loads)]

    one = run([torch.cuda.current_stream()])
    two = run([torch.cuda.Stream(), torch.cuda.Stream()])
    for (i1, p1, l1), (i2, p2, l2) in zip(one, two):
        assert torch.equal(i1, i2) and torch.equal(p1, p2) and torch.equal(l1, l2)


def test_pipelined_call_replayed_from_a_hip_graph():
    """A pipelined call is three launches (its counters are cleared by a kernel): captured
    once, replayed on new inputs with eager work in between, every replay must give what
    the eager call gives."""
    import torch
    from paper_2510_03293_amd import binding as B
    u = _util()
    T, H, E, k, c = 6000, 256, 64, 6, 8
    params = B.make_params(k, c, 0.40, 0.80, dtype=wl.DTYPE_BF16, pipeline_tiles=13)
    hid = torch.empty((T, H), dtype=torch.bfloat16, device="cuda")
    inputs = [_mixed_gate(500 + i, T, H, E, 0.25) for i in range(4)]
    wd = u.to_device(inputs[0][1])
    buf = B.RouteBuffers(T, H, E, params)
    loads = torch.zeros(E, dtype=torch.int32, device="cuda")
    side = torch.cuda.Stream()

    def enqueue(stream):
        B.laser_route(hid, wd, T, H, E, params, loads, buf.expert_ids, buf.weights, buf.permutation,
                      buf.expert_offsets, None, buf.workspace, stream)

    def fill(rep):
        hid.copy_(u.to_device(inputs[rep % len(inputs)][0]))
        loads.zero_()

    fill(0)
    with torch.cuda.stream(side):
        enqueue(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    fill(0)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        enqueue(side)
    torch.cuda.synchronize()
    for rep in range(1, 5):
        fill(rep)
        torch.cuda.synchronize()
        enqueue(torch.cuda.current_stream())
        torch.cuda.synchronize()
        want = (buf.expert_ids.clone(), buf.weights.clone(), buf.permutation.clone(), buf.expert_offsets.clone(),
                loads.clone())
        buf.expert_ids.fill_(-1)
        buf.permutation.fill_(-1)
        fill(rep)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = (buf.expert_ids, buf.weights, buf.permutation, buf.expert_offsets, loads)
        for x, y in zip(want, got):
            assert torch.equal(x.view(torch.int32), y.view(torch.int32)), f"replay {rep}"
        assert B.laser_status(buf.workspace) == B.STATUS_COMPLETE
