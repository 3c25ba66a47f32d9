#!/usr/bin/env python3
"""Benchmark of the Two-Branch Swin Block hot path on one MI355X.

One step = one pass of the whole path over the Swin-T stage-1 pair at detection
scale (BASELINE config 2): score the 1392 windows of a 200x336x96 map once,
run the regular block and then the shifted block (A8 high / A4 low, int8
per-channel weights), all through one mixaq_stage_forward call: the first
block takes the selection (keep ratio 0.5) from the scores inside its first
kernel and leaves the list for the shifted block.  Inputs are seeded synthetic
tensors already resident in HBM; block creation (weight packing) is outside the
timed region.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_INT8_TOPS = 5000.0      # MI355X dense int8 MFMA, TOP/s
PEAK_HBM_GBS = 8000.0        # MI355X HBM3E, GB/s
PEAK_VALU_TLOPS = 39.32      # 256 CU x 4 SIMD x 16 lanes x 2.4 GHz, non-packed fp32 lane-ops/s (T)


def macs_per_window(C):
    return 588 * C * C + 4802 * C


# VALU instructions per element of the pinned arithmetic (one lane-operation each): dequantize = cvt + fma,
# quantize = fma + med3 + 3/4 pack, GELU = 9, LayerNorm = 8 (+ quantize), softmax element = 17 (+ quantize)
ALU_DEQ, ALU_Q, ALU_GELU, ALU_LN, ALU_SOFTMAX = 2.0, 2.75, 9.0, 8.0, 17.0


def kernel_model(name, C, F, heads, n_windows):
    """Algorithmic work of one launch over n_windows windows as (bound, amount): HBM kernels in bytes,
    MFMA kernels in int8 operations (2 per MAC), ALU kernels in fp32 vector lane-operations.
    The fused kernels are given BOTH their MFMA and their ALU work; the ALU side is the one that binds."""
    T = 49
    mfma = None
    if name == "score":
        return "hbm", n_windows * (4 * T * C + 8), mfma
    if name == "select":
        return "hbm", n_windows * (8 + 4), mfma
    if name in ("gather_ln1_quant", "ln2_quant"):
        return "hbm", n_windows * (4 * T * C + T * C), mfma
    if name == "qkv_gemm":
        return "mfma", n_windows * 2 * T * C * 3 * C, mfma
    if name == "window_attention":
        return "mfma", n_windows * 2 * 2 * T * T * C, mfma
    if name == "proj_gemm_residual":
        return "mfma", n_windows * 2 * T * C * C, mfma
    if name in ("fc1_gemm_gelu", "fc2_gemm_residual_scatter"):
        return "mfma", n_windows * 2 * T * C * F, mfma
    if name == "window_ln1_qkv_attention":
        mfma = n_windows * 2 * (T * C * 3 * C + 2 * T * T * C)
        alu = T * C * (ALU_LN + ALU_Q) + T * 3 * C * (ALU_DEQ + ALU_Q) + heads * T * T * (ALU_SOFTMAX + ALU_Q) + \
            T * C * (ALU_DEQ + 1 + ALU_Q)
        return "alu", n_windows * alu, mfma
    if name == "token_proj_ln2_ffn_scatter":
        mfma = n_windows * 2 * (T * C * C + 2 * T * C * F)
        alu = T * C * (ALU_DEQ + 1) + T * C * (ALU_LN + ALU_Q) + T * F * (ALU_DEQ + ALU_GELU + ALU_Q) + T * C * (ALU_DEQ + 1)
        return "alu", n_windows * alu, mfma
    raise KeyError(name)


def kernel_hbm_bytes(name, C, n_windows):
    """Algorithmic HBM bytes of one launch of a fused kernel (the gather / scatter side of it): the window
    kernel reads the map and writes the attention-output codes; the token kernel reads the shortcut and the
    codes and writes the map."""
    T = 49
    if name == "window_ln1_qkv_attention":
        return n_windows * (4 * T * C + T * C)
    if name == "token_proj_ln2_ffn_scatter":
        return n_windows * (4 * T * C + T * C + 4 * T * C)
    return None


def read_traffic(kernel):
    """HBM bytes per launch of `kernel` from the committed counter summary (profiles/), or None."""
    path = os.path.join(ROOT, "profiles", "cfg2_hbm_traffic.txt")
    try:
        for line in open(path):
            parts = line.split()
            if len(parts) >= 3 and parts[0] == "traffic_bytes_per_launch" and parts[1] == kernel:
                return int(float(parts[2]))
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=500)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the path has no collectives); run with --gpus 1",
              file=sys.stderr)
        return 2

    import torch
    from paper_2507_19131_amd import binding as M
    from paper_2507_19131_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    M.load()
    dev = torch.device("cuda:0")
    wl = synth.workload("cfg2")
    stage = wl["stages"][0]
    spec = stage["spec"]
    keep = wl["keep"][0]
    k_high = M.mixaq_keep_count(spec.nW, keep)
    x_np = synth.make_feature_map(spec, wl["seed"], blobs=wl["blobs"], outlier_channels=wl["outliers"])
    inputs = [synth.make_block_inputs(spec, wl["seed"] + 10 * i) for i, _ in enumerate(stage["shifts"])]
    x = torch.from_numpy(x_np).to(dev)
    blocks = []
    for inp, shift in zip(inputs, stage["shifts"]):
        sh, br = M.to_device(inp)
        blocks.append(M.mixaq_block_create(M.make_desc(spec, shift), sh, br))
    ws = M.alloc_workspace(blocks[0])
    scores = torch.empty((spec.B, spec.nW), dtype=torch.float64, device=dev)
    perm = torch.empty((spec.B, spec.nW), dtype=torch.int32, device=dev)
    bufs = [torch.empty_like(x), torch.empty_like(x)]

    def step():
        # one C call for the stage: score once; the first block takes the selection from the scores inside
        # its first kernel and leaves the list for the stage's other blocks
        return M.mixaq_stage_forward(blocks, x, [k_high], None, bufs[0], bufs[1], scores, perm, ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    # per-kernel durations with HIP events on the launch stream, same steps again
    names = [M.mixaq_kernel_name(i) for i in range(M.NUM_KERNELS)]
    acc = {n: 0.0 for n in names}
    launches = {n: 0 for n in names}
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    REP = 4                      # launches between an event pair (amortises the events' own cost)
    prof_steps = min(args.steps, 200)
    for _ in range(prof_steps):
        ev0.record()
        for _r in range(REP):
            M.mixaq_score_windows(blocks[0], x, scores)
        ev1.record()
        ev1.synchronize()
        acc["score"] += ev0.elapsed_time(ev1) / REP
        launches["score"] += 1
        cur = x
        for i, blk in enumerate(blocks):
            if i == 0:
                ms = M.mixaq_block_forward_profile(blk, cur, None, k_high, bufs[i % 2], ws, repeats=REP, scores=scores)
            else:
                ms = M.mixaq_block_forward_profile(blk, cur, perm, k_high, bufs[i % 2], ws, repeats=REP)
            cur = bufs[i % 2]
            for n, v in ms.items():
                if v > 0:
                    acc[n] += v
                    launches[n] += 1
    n_win = spec.B * spec.nW
    C, F = spec.C, spec.C * spec.mlp_ratio
    kernels = {}
    for n in names:
        if not launches[n]:
            continue
        avg_ms = acc[n] / launches[n]
        bound, amount, mfma_ops = kernel_model(n, C, F, spec.heads, n_win)
        if bound == "hbm":
            ach, peak, unit = amount / (avg_ms * 1e-3) / 1e9, PEAK_HBM_GBS, "GB/s"
        elif bound == "mfma":
            ach, peak, unit = amount / (avg_ms * 1e-3) / 1e12, PEAK_INT8_TOPS, "TOP/s"
        else:
            ach, peak, unit = amount / (avg_ms * 1e-3) / 1e12, PEAK_VALU_TLOPS, "Tlane-op/s"
        kernels[n] = dict(avg_ms=round(avg_ms, 5), launches_per_step=launches[n] // prof_steps, bound=bound,
                          achieved=round(ach, 3), peak=peak, unit=unit, frac=round(ach / peak, 5))
        if mfma_ops is not None:        # the same launch against the int8 MFMA peak
            t = mfma_ops / (avg_ms * 1e-3) / 1e12
            kernels[n].update(int8_tops=round(t, 3), frac_int8_mfma_peak=round(t / PEAK_INT8_TOPS, 5))
        hb = kernel_hbm_bytes(n, C, n_win)
        if hb is not None:              # ... and its gather / scatter traffic against the HBM peak
            gbs = hb / (avg_ms * 1e-3) / 1e9
            kernels[n].update(hbm_gbs=round(gbs, 1), frac_hbm_peak=round(gbs / PEAK_HBM_GBS, 5))
    per_step = {n: kernels[n]["avg_ms"] * kernels[n]["launches_per_step"] for n in kernels}
    dom = max(per_step, key=per_step.get)
    kd = kernels[dom]
    roofline = dict(kernel=dom, bound=kd["bound"], achieved=kd["achieved"], peak=kd["peak"], unit=kd["unit"],
                    frac=kd["frac"], traffic=read_traffic(dom), avg_ms=kd["avg_ms"])
    if "frac_int8_mfma_peak" in kd:
        roofline.update(int8_tops=kd["int8_tops"], frac_int8_mfma_peak=kd["frac_int8_mfma_peak"])

    # The same step with the score taken after a LayerNorm (score_mode 1: the scoring LayerNorm's parameters are
    # the high branch's LN1 here); only the score kernel differs, and with it which windows are selected.
    d1 = M.make_desc(spec, stage["shifts"][0])
    d1.score_mode = 1
    sh1, br1 = M.to_device(inputs[0])
    blocks_m1 = [M.mixaq_block_create(d1, sh1, br1)] + blocks[1:]

    def step_m1():
        return M.mixaq_stage_forward(blocks_m1, x, [k_high], None, bufs[0], bufs[1], scores, perm, ws)
    for _ in range(args.warmup):
        step_m1()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step_m1()
    torch.cuda.synchronize()
    ms_per_step_m1 = (time.perf_counter() - t0) * 1e3 / args.steps
    M.mixaq_block_destroy(blocks_m1[0])

    windows_per_step = n_win * len(blocks)
    ops_per_step = 2 * macs_per_window(C) * windows_per_step
    value = windows_per_step / (ms_per_step * 1e-3)
    int_tops = ops_per_step / (ms_per_step * 1e-3) / 1e12

    cpu = None
    if not args.no_cpu_baseline:
        sys.path.insert(0, os.path.join(ROOT, "tests"))
        import oracle_api as O              # the oracle is used for this leg only
        t0 = time.perf_counter()
        o_scores = O.score_windows(inputs[0], x_np)
        o_perm = O.select_windows(o_scores, k_high)
        cur = x_np
        for inp, shift in zip(inputs, stage["shifts"]):
            cur, _ = O.block_forward(inp, cur, o_perm, k_high, shift, threads=1)
        dt = time.perf_counter() - t0
        cpu = dict(value=round(windows_per_step / dt, 2), unit="windows/s", cores=1, kind="oracle",
                   sample="one full step of the same workload (score + select + both blocks, 2784 windows), single thread",
                   seconds=round(dt, 2), int_tops=round(ops_per_step / dt / 1e12, 5))

    out = dict(metric="windows/sec & effective int-TOPS per two-branch Swin block; % int8 MFMA peak",
               value=round(value, 1), unit="windows/s", n_gpus=1, steps=args.steps, warmup=args.warmup,
               ms_per_step=round(ms_per_step, 5), higher_is_better=True, scaling="weak", vs_baseline=None,
               dtype="int8 (int32 accumulate, fp32 epilogues)", data="synthetic",
               config=dict(workload="cfg2: Swin-T stage-1 pair (regular + shifted block), B=1, 200x336x96 padded to 203x336, "
                                    "1392 windows, 3 heads, keep 0.5, A8/A4, W8", blocks_per_step=len(blocks),
                           windows_per_step=windows_per_step, k_high=k_high, score_mode=0),
               score_after_layernorm=dict(score_mode=1, ms_per_step=round(ms_per_step_m1, 5),
                                          value=round(windows_per_step / (ms_per_step_m1 * 1e-3), 1)),
               int_tops=round(int_tops, 3), pct_int8_mfma_peak=round(100 * int_tops / PEAK_INT8_TOPS, 3),
               ms_per_block=round(ms_per_step / len(blocks), 5),
               roofline=roofline, kernels=kernels, cpu_baseline=cpu)
    # a plain copy of known size, so that a counter run of this same command can calibrate
    # FETCH_SIZE / WRITE_SIZE against bytes (64 MiB read + 64 MiB written)
    calib_src = torch.empty(64 * 1024 * 1024, dtype=torch.uint8, device=dev)
    calib_dst = torch.empty_like(calib_src)
    calib_dst.copy_(calib_src)
    torch.cuda.synchronize()
    print(json.dumps(out))
    for blk in blocks:
        M.mixaq_block_destroy(blk)
    return 0


if __name__ == "__main__":
    sys.exit(main())
