"""GPU parity on whole stages of the benchmark workloads: blocks chained on one map, the score
taken once on the stage input and shared by the stage's blocks, one keep ratio per block pair."""
import numpy as np
import pytest
import torch

from paper_2507_19131_amd import synth

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import gpu_harness as gh
    import oracle_api as O
    from paper_2507_19131_amd import binding as M


def run_stage(spec, shifts, keep, seed, blobs, outliers, ranges):
    """Returns (y_gpu, y_oracle, perm_gpu, perm_oracle) after the chain of blocks."""
    dev = torch.device("cuda:0")
    x_np = synth.make_feature_map(spec, seed, blobs=blobs, outlier_channels=outliers)
    inputs = [synth.make_block_inputs(spec, seed + 10 * i, ranges=ranges) for i in range(len(shifts))]
    k = M.mixaq_keep_count(spec.nW, keep)
    x = torch.from_numpy(x_np).to(dev)
    blocks = [gh.GpuBlock(inp, shift) for inp, shift in zip(inputs, shifts)]
    try:
        _, perm = blocks[0].score_select(x, k)
        cur = x
        for gb in blocks:
            cur = gb.forward(cur, perm, k)
        torch.cuda.synchronize()
        y_gpu, perm_gpu = cur.cpu().numpy(), perm.cpu().numpy()
    finally:
        for gb in blocks:
            gb.close()
    perm_o = O.select_windows(O.score_windows(inputs[0], x_np), k)
    cur = x_np
    for inp, shift in zip(inputs, shifts):
        cur, _ = O.block_forward(inp, cur, perm_o, k, shift, threads=16)
    return y_gpu, cur, perm_gpu, perm_o


def check(y_gpu, y_or, perm_gpu, perm_or):
    assert np.array_equal(perm_gpu, perm_or)
    assert not np.isnan(y_gpu).any()
    rms = float(np.sqrt(np.mean(y_or.astype(np.float64) ** 2)))
    err = float(np.max(np.abs(y_gpu.astype(np.float64) - y_or)))
    print("max abs err", err, "rms", rms, "bit identical", np.array_equal(y_gpu, y_or), flush=True)
    assert err <= 1e-3 * rms


def test_config2_stage_pair():
    wl = synth.workload("cfg2")
    st = wl["stages"][0]
    check(*run_stage(st["spec"], st["shifts"], wl["keep"][0], wl["seed"], wl["blobs"], wl["outliers"], wl.get("ranges")))


def test_config2_shape_on_a_batch_of_four():
    """The benchmark's context entry: config 2's stage on four maps at once (5568 windows per block, the selection
    taken per image)."""
    import dataclasses
    wl = synth.workload("cfg2")
    st = wl["stages"][0]
    spec = dataclasses.replace(st["spec"], B=4)
    print("config 2 shape, batch 4", flush=True)
    y_gpu, y_or, perm_gpu, perm_or = run_stage(spec, st["shifts"], wl["keep"][0], wl["seed"], wl["blobs"], wl["outliers"], wl.get("ranges"))
    assert perm_gpu.shape == (4, spec.nW) and all(sorted(row) == list(range(spec.nW)) for row in perm_gpu.tolist())
    check(y_gpu, y_or, perm_gpu, perm_or)


@pytest.mark.parametrize("keep", [0.25, 0.5, 0.75])
def test_config3_six_blocks(keep):
    wl = synth.workload("cfg3")
    st = wl["stages"][0]
    print("config 3 keep", keep, flush=True)
    check(*run_stage(st["spec"], st["shifts"], keep, wl["seed"], wl["blobs"], wl["outliers"], wl.get("ranges")))


@pytest.mark.parametrize("stage", [0, 1, 2, 3])
def test_config4_stage_shapes(stage):
    """W4A4 with 2-bit low windows; every stage of Swin-T at 800x1344 on its own synthetic map."""
    wl = synth.workload("cfg4")
    st = wl["stages"][stage]
    print("config 4 stage", stage, flush=True)
    check(*run_stage(st["spec"], st["shifts"], wl["keep"][0], wl["seed"] + stage, wl["blobs"], wl["outliers"], wl.get("ranges")))


@pytest.mark.parametrize("stage", [0, 1])
def test_config5_swin_b_stages(stage):
    wl = synth.workload("cfg5")
    st = wl["stages"][stage]
    print("config 5 stage", stage, flush=True)
    check(*run_stage(st["spec"], st["shifts"], wl["keep"][0], wl["seed"] + stage, wl["blobs"], wl["outliers"], wl.get("ranges")))


@pytest.mark.parametrize("fused", [True, False])
def test_stage_entry_point_with_a_ratio_per_pair_and_pruning(fused):
    """mixaq_stage_forward (one C call for the stage: score once, select inside the first block, every
    pair with its own counts, Sec. 3.2-3.4) against the oracle's chain of blocks."""
    spec = synth.BlockSpec(2, 33, 40, 96, 3)
    shifts = [0, 3, 0, 3, 0]                                      # two pairs and a single last block
    k_high, k_low = [12, 5, 20], [10, 25, 0]                       # nW = 30: pair 0 prunes 8 windows, pair 2 prunes 10
    x_np = synth.make_feature_map(spec, 77, blobs=True)
    inputs = [synth.make_block_inputs(spec, 700 + i) for i in range(len(shifts))]
    assert spec.nW == 30
    dev = torch.device("cuda:0")
    x = torch.from_numpy(x_np).to(dev)
    blocks = [gh.GpuBlock(inp, shift, fused) for inp, shift in zip(inputs, shifts)]
    try:
        y, tmp = torch.empty_like(x), torch.empty_like(x)
        scores = torch.empty((spec.B, spec.nW), dtype=torch.float64, device=dev)
        perm = torch.empty((spec.B, spec.nW), dtype=torch.int32, device=dev)
        M.mixaq_stage_forward([gb.blk for gb in blocks], x, k_high, k_low, y, tmp, scores, perm, blocks[0].ws)
        torch.cuda.synchronize()
        assert torch.equal(x.cpu(), torch.from_numpy(x_np))        # the input is left alone
        y_gpu, perm_gpu, scores_gpu = y.cpu().numpy(), perm.cpu().numpy(), scores.cpu().numpy()
        with pytest.raises(M.MixaqError) as e:
            M.mixaq_stage_forward([gb.blk for gb in blocks], x, [12, 5, 31], None, y, tmp, scores, perm, blocks[0].ws)
        assert e.value.code == -2
    finally:
        for gb in blocks:
            gb.close()
    sc_o = O.score_windows(inputs[0], x_np)
    assert np.array_equal(scores_gpu, sc_o) or np.allclose(scores_gpu, sc_o, rtol=1e-12, atol=0)
    cur = x_np
    for i, (inp, shift) in enumerate(zip(inputs, shifts)):
        perm_o = O.select_windows(sc_o, k_high[i // 2], k_low=k_low[i // 2])
        assert np.array_equal(perm_gpu, perm_o)                   # the list is the full sort: the same for every pair
        cur, _ = O.block_forward(inp, cur, perm_o, k_high[i // 2], shift, threads=16, k_low=k_low[i // 2])
    check(y_gpu, cur, perm_gpu, perm_o)
    assert np.array_equal(y_gpu, cur)


@pytest.mark.parametrize("B,C,heads", [(2, 384, 12), (3, 96, 3), (5, 192, 6)])
def test_stage_on_a_batch_of_small_maps_runs_as_two_chains(B, C, heads):
    """A batch of small maps (at most 4096 windows in all) goes through the stage call as two chains of blocks, one per
    half of the images (uneven halves for an odd batch), the second on the library's side stream; the result is the
    oracle's, the same bits as block after block on the whole batch, and repeated calls agree."""
    spec = synth.BlockSpec(B, 30, 37, C, heads)
    shifts = [0, 3, 0, 3]
    assert B * spec.nW <= 4096
    x_np = synth.make_feature_map(spec, 78, blobs=True)
    inputs = [synth.make_block_inputs(spec, 800 + i) for i in range(len(shifts))]
    k_high, k_low = [spec.nW // 2, spec.nW // 3], [spec.nW - spec.nW // 2, spec.nW // 3]      # the second pair prunes a third
    dev = torch.device("cuda:0")
    x = torch.from_numpy(x_np).to(dev)
    print("two chains, batch", B, "C", C, flush=True)
    blocks = [gh.GpuBlock(inp, shift) for inp, shift in zip(inputs, shifts)]
    try:
        y, tmp = torch.full_like(x, float("nan")), torch.empty_like(x)
        scores = torch.empty((B, spec.nW), dtype=torch.float64, device=dev)
        perm = torch.full((B, spec.nW), -1, dtype=torch.int32, device=dev)
        handles = [gb.blk for gb in blocks]
        M.mixaq_stage_forward(handles, x, k_high, k_low, y, tmp, scores, perm, blocks[0].ws)
        torch.cuda.synchronize()
        y1, perm1 = y.clone(), perm.clone()
        for _ in range(3):                                         # the side stream joins every call: no call sees the last one's state
            M.mixaq_stage_forward(handles, x, k_high, k_low, y, tmp, scores, perm, blocks[0].ws)
        torch.cuda.synchronize()
        assert torch.equal(y, y1) and torch.equal(perm, perm1)
        cur = x                                                    # block after block on the whole batch, one stream
        for i, gb in enumerate(blocks):
            cur = gb.forward_pruned(cur, perm, k_high[i // 2], k_low[i // 2])
        torch.cuda.synchronize()
        assert torch.equal(cur, y1)
        y_gpu, perm_gpu = y1.cpu().numpy(), perm1.cpu().numpy()
    finally:
        for gb in blocks:
            gb.close()
    sc_o = O.score_windows(inputs[0], x_np)
    cur = x_np
    for i, (inp, shift) in enumerate(zip(inputs, shifts)):
        perm_o = O.select_windows(sc_o, k_high[i // 2], k_low=k_low[i // 2])
        assert np.array_equal(perm_gpu, perm_o)
        cur, _ = O.block_forward(inp, cur, perm_o, k_high[i // 2], shift, threads=16, k_low=k_low[i // 2])
    assert np.array_equal(y_gpu, cur)


def test_two_chains_at_config2_shape_on_two_maps():
    """2 x 1392 windows at C = 96: the largest kind of batch the stage call still runs as two chains."""
    import dataclasses
    wl = synth.workload("cfg2")
    st = wl["stages"][0]
    spec = dataclasses.replace(st["spec"], B=2)
    assert spec.B * spec.nW <= 4096
    y_blocks, y_or, perm_blocks, perm_or = run_stage(spec, st["shifts"], wl["keep"][0], wl["seed"], wl["blobs"], wl["outliers"], wl.get("ranges"))
    check(y_blocks, y_or, perm_blocks, perm_or)
    k = M.mixaq_keep_count(spec.nW, wl["keep"][0])
    dev = torch.device("cuda:0")
    x = torch.from_numpy(synth.make_feature_map(spec, wl["seed"], blobs=wl["blobs"], outlier_channels=wl["outliers"])).to(dev)
    inputs = [synth.make_block_inputs(spec, wl["seed"] + 10 * i, ranges=wl.get("ranges")) for i in range(len(st["shifts"]))]
    blocks = [gh.GpuBlock(inp, shift) for inp, shift in zip(inputs, st["shifts"])]
    try:
        y, tmp = torch.full_like(x, float("nan")), torch.empty_like(x)
        scores = torch.empty((spec.B, spec.nW), dtype=torch.float64, device=dev)
        perm = torch.empty((spec.B, spec.nW), dtype=torch.int32, device=dev)
        M.mixaq_stage_forward([gb.blk for gb in blocks], x, [k], None, y, tmp, scores, perm, blocks[0].ws)
        torch.cuda.synchronize()
        assert np.array_equal(y.cpu().numpy(), y_or) and np.array_equal(perm.cpu().numpy(), perm_or)
    finally:
        for gb in blocks:
            gb.close()


@pytest.mark.parametrize("B", [1, 3])
def test_stage_on_a_side_stream_matches_the_default_stream(B):
    """All work of a call is ordered on the stream it is given: a stage run on a second stream (default
    priority) while the default stream is kept busy gives the same bits, and is complete as soon as that
    stream is; with a batch also when the call runs as two chains (the second on the library's own stream)."""
    wl = synth.workload("cfg2")
    st = wl["stages"][0]
    spec = synth.BlockSpec(B, 60, 75, 96, 3)
    dev = torch.device("cuda:0")
    x = torch.from_numpy(synth.make_feature_map(spec, 88, blobs=True)).to(dev)
    blocks = [gh.GpuBlock(synth.make_block_inputs(spec, 880 + i), shift) for i, shift in enumerate(st["shifts"])]
    try:
        k = M.mixaq_keep_count(spec.nW, 0.5)
        outs = []
        side = torch.cuda.Stream()
        for stream in (None, side):
            y, tmp = torch.full_like(x, float("nan")), torch.empty_like(x)
            scores = torch.empty((spec.B, spec.nW), dtype=torch.float64, device=dev)
            perm = torch.empty((spec.B, spec.nW), dtype=torch.int32, device=dev)
            ws = M.alloc_workspace(blocks[0].blk)
            torch.cuda.synchronize()
            if stream is not None:
                busy = torch.empty(1 << 26, device=dev)
                for _ in range(8):
                    busy.normal_()                                  # keeps the default stream occupied meanwhile
            M.mixaq_stage_forward([gb.blk for gb in blocks], x, [k], None, y, tmp, scores, perm, ws, stream=stream)
            if stream is not None:
                stream.synchronize()
                assert not torch.isnan(y).any()                     # complete as soon as ITS stream is
            torch.cuda.synchronize()
            outs.append(y.clone())
        assert torch.equal(outs[0], outs[1])
    finally:
        for gb in blocks:
            gb.close()


BENCH_STAGES = [("cfg1", 0), ("cfg2", 0), ("cfg3", 0), ("cfg4", 1), ("cfg4", 2), ("cfg4", 3), ("cfg5", 0), ("cfg5", 1)]


@pytest.mark.parametrize("name,stage", BENCH_STAGES, ids=[f"{n}-stage{s + 1}" for n, s in BENCH_STAGES])
def test_stage_call_as_the_benchmark_launches_it(name, stage):
    """Every benchmark workload at full size through mixaq_stage_forward, the one call a benchmark step makes
    (score, selection inside the first block's first kernel, list handed on to the later blocks; config 3's two
    maps go through it as two chains, config 4's last stage on the seven-kernel path)."""
    wl = synth.workload(name)
    st = wl["stages"][stage]
    spec, shifts = st["spec"], st["shifts"]
    keep = wl["keep"][len(wl["keep"]) // 2]
    seed = wl["seed"] + stage
    print("stage call", name, "stage", stage + 1, "C", spec.C, "B", spec.B, "windows", spec.B * spec.nW, flush=True)
    x_np = synth.make_feature_map(spec, seed, blobs=wl["blobs"], outlier_channels=wl["outliers"])
    inputs = [synth.make_block_inputs(spec, seed + 10 * i, ranges=wl.get("ranges")) for i, _ in enumerate(shifts)]
    k = M.mixaq_keep_count(spec.nW, keep)
    pairs = (len(shifts) + 1) // 2
    dev = torch.device("cuda:0")
    x = torch.from_numpy(x_np).to(dev)
    blocks = [gh.GpuBlock(inp, shift) for inp, shift in zip(inputs, shifts)]
    try:
        y, tmp = torch.full_like(x, float("nan")), torch.empty_like(x)
        scores = torch.empty((spec.B, spec.nW), dtype=torch.float64, device=dev)
        perm = torch.empty((spec.B, spec.nW), dtype=torch.int32, device=dev)
        for _ in range(3):                                          # repeated calls reuse workspace, scores and list
            M.mixaq_stage_forward([gb.blk for gb in blocks], x, [k] * pairs, None, y, tmp, scores, perm, blocks[0].ws)
        torch.cuda.synchronize()
        y_gpu, perm_gpu = y.cpu().numpy(), perm.cpu().numpy()
    finally:
        for gb in blocks:
            gb.close()
    perm_o = O.select_windows(O.score_windows(inputs[0], x_np), k)
    cur = x_np
    for inp, shift in zip(inputs, shifts):
        cur, _ = O.block_forward(inp, cur, perm_o, k, shift, threads=16)
    check(y_gpu, cur, perm_gpu, perm_o)
    assert np.array_equal(y_gpu, cur)


def test_random_sweep_of_stage_calls():
    """Thirty seeded random stage calls: width, batch (one or two chains), map size, 1-4 blocks, bit widths, score mode,
    shared or independent biases and, per pair, any split into high, low and pruned windows (none and all included);
    maps and selection lists must equal the oracle's bit for bit."""
    dev = torch.device("cuda:0")
    for case in range(30):
        rng = np.random.default_rng(61000 + case)
        C, heads = [(96, 3), (128, 4), (192, 6), (256, 8), (384, 12)][int(rng.choice([0, 0, 1, 2, 3, 4]))]
        B, H, W = int(rng.integers(1, 7)), int(rng.integers(14, 60)), int(rng.integers(14, 60))
        shifts = [0, 3, 0, 3][:int(rng.integers(1, 5))]
        hi = int(rng.integers(4, 9))
        spec = synth.BlockSpec(B, H, W, C, heads, act_bits_high=hi, act_bits_low=int(rng.integers(2, hi + 1)),
                               weight_bits=int(rng.choice([4, 8])), score_mode=int(rng.integers(0, 2)))
        k_high, k_low = [], []
        for _ in range((len(shifts) + 1) // 2):
            kh = int(rng.integers(0, spec.nW + 1))
            kl = int(rng.integers(0, spec.nW - kh + 1))
            if rng.integers(0, 2):
                kl = spec.nW - kh                                   # no pruning
            k_high.append(kh)
            k_low.append(kl)
        print("stage sweep case", case, "B", B, H, W, "C", C, "blocks", len(shifts), "k_high", k_high, "k_low", k_low, flush=True)
        x_np = synth.make_feature_map(spec, 62000 + case, blobs=bool(rng.integers(0, 2)))
        inputs = [synth.make_block_inputs(spec, 63000 + 10 * case + i, per_branch_bias=bool(rng.integers(0, 2))) for i in range(len(shifts))]
        x = torch.from_numpy(x_np).to(dev)
        blocks = [gh.GpuBlock(inp, shift) for inp, shift in zip(inputs, shifts)]
        try:
            y, tmp = torch.full_like(x, float("nan")), torch.empty_like(x)
            scores = torch.empty((B, spec.nW), dtype=torch.float64, device=dev)
            perm = torch.full((B, spec.nW), -1, dtype=torch.int32, device=dev)
            for _ in range(2):
                M.mixaq_stage_forward([gb.blk for gb in blocks], x, k_high, k_low, y, tmp, scores, perm, blocks[0].ws)
            torch.cuda.synchronize()
            y_gpu, perm_gpu = y.cpu().numpy(), perm.cpu().numpy()
        finally:
            for gb in blocks:
                gb.close()
        sc_o = O.score_windows(inputs[0], x_np)
        cur = x_np
        for i, (inp, shift) in enumerate(zip(inputs, shifts)):
            perm_o = O.select_windows(sc_o, k_high[i // 2], k_low=k_low[i // 2])
            cur, _ = O.block_forward(inp, cur, perm_o, k_high[i // 2], shift, threads=16, k_low=k_low[i // 2])
        assert np.array_equal(perm_gpu, perm_o), case
        assert np.array_equal(y_gpu, cur), case


@pytest.mark.parametrize("name", ["cfg2", "cfg3"])
def test_repeated_stage_calls_are_bit_stable(name):
    """The same stage call a hundred times over (one chain at config 2, two chains at config 3): every result has the
    bits of the first, which a missing barrier or a race between the chains would not survive."""
    wl = synth.workload(name)
    st = wl["stages"][0]
    spec, shifts = st["spec"], st["shifts"]
    dev = torch.device("cuda:0")
    x = torch.from_numpy(synth.make_feature_map(spec, wl["seed"], blobs=wl["blobs"], outlier_channels=wl["outliers"])).to(dev)
    blocks = [gh.GpuBlock(synth.make_block_inputs(spec, wl["seed"] + 10 * i, ranges=wl.get("ranges")), shift) for i, shift in enumerate(shifts)]
    try:
        k = M.mixaq_keep_count(spec.nW, 0.5)
        pairs = (len(shifts) + 1) // 2
        y, tmp = torch.empty_like(x), torch.empty_like(x)
        scores = torch.empty((spec.B, spec.nW), dtype=torch.float64, device=dev)
        perm = torch.empty((spec.B, spec.nW), dtype=torch.int32, device=dev)
        handles = [gb.blk for gb in blocks]
        M.mixaq_stage_forward(handles, x, [k] * pairs, None, y, tmp, scores, perm, blocks[0].ws)
        torch.cuda.synchronize()
        first, first_perm = y.clone(), perm.clone()
        print("repeating the stage call of", name, flush=True)
        for it in range(100):
            y.fill_(float("nan"))
            M.mixaq_stage_forward(handles, x, [k] * pairs, None, y, tmp, scores, perm, blocks[0].ws)
            if it % 5 == 4:
                assert torch.equal(y, first) and torch.equal(perm, first_perm), it
        torch.cuda.synchronize()
    finally:
        for gb in blocks:
            gb.close()


def test_stage_call_can_be_captured_in_a_graph():
    """The stage call allocates nothing and never synchronises, so a caller may capture it; every replay, with
    eager work and synchronisations in between, reproduces the eager result."""
    spec = synth.BlockSpec(2, 40, 47, 96, 3)
    dev = torch.device("cuda:0")
    xs = [torch.from_numpy(synth.make_feature_map(spec, 90 + i, blobs=True)).to(dev) for i in range(3)]
    blocks = [gh.GpuBlock(synth.make_block_inputs(spec, 900 + i), shift) for i, shift in enumerate([0, 3])]
    try:
        k = M.mixaq_keep_count(spec.nW, 0.5)
        x = xs[0].clone()
        y, tmp = torch.empty_like(x), torch.empty_like(x)
        scores = torch.empty((spec.B, spec.nW), dtype=torch.float64, device=dev)
        perm = torch.empty((spec.B, spec.nW), dtype=torch.int32, device=dev)
        ws = blocks[0].ws
        handles = [gb.blk for gb in blocks]

        def step():
            M.mixaq_stage_forward(handles, x, [k], None, y, tmp, scores, perm, ws)
        eager = []
        for xi in xs:
            x.copy_(xi)
            step()
            torch.cuda.synchronize()
            eager.append(y.clone())
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()                                                  # warm-up on the capture stream
        torch.cuda.current_stream().wait_stream(side)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        for rep in range(2):
            for xi, want in zip(xs, eager):
                x.copy_(xi)                                         # eager work between the replays
                y.fill_(float("nan"))
                graph.replay()
                torch.cuda.synchronize()
                assert torch.equal(y, want), rep
    finally:
        for gb in blocks:
            gb.close()
