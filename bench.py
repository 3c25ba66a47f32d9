#!/usr/bin/env python3
"""Benchmark of the Two-Branch Swin Block hot path on one MI355X.

Headline: one step = one pass of the whole path over the Swin-T stage-1 pair at detection scale
(BASELINE config 2): score the 1392 windows of a 200x336x96 map once, run the regular block and
then the shifted block (A8 high / A4 low, int8 per-channel weights), all through one
mixaq_stage_forward call: the first block takes the selection (keep ratio 0.5) from the scores
inside its first kernel and leaves the list for the shifted block.  Inputs are seeded synthetic
tensors already resident in HBM; block creation (weight packing) is outside the timed region.

The other four workloads (config 1, 3, 4, 5) are timed the same way, stage by stage, and reported
under "configs"; every kernel is priced against the roofline that bounds its algorithmic work
(HBM bytes for the fused kernels up to C = 192 and the gather / scatter kernels, int8 MFMA
operations from C = 256 and for the GEMM kernels).  The CPU oracle is timed beside it on bounded
samples.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
# Kernel arguments in device memory (the HIP runtime's default on this image; stated here because the step is five short
# kernels and each one starts by reading its arguments: with the arguments in host memory the step measures 0.142 ms
# instead of 0.122).  Has to be in the environment before the runtime library is loaded, i.e. before torch is imported.
os.environ.setdefault("HIP_FORCE_DEV_KERNARG", "1")

PEAK_INT8_TOPS = 5000.0      # MI355X dense int8 MFMA, TOP/s
PEAK_HBM_GBS = 8000.0        # MI355X HBM3E, GB/s
PEAK_VALU_TLOPS = 39.32      # 256 CU x 4 SIMD x 16 lanes x 2.4 GHz, non-packed fp32 lane-ops/s (T)
T = 49                       # tokens per window


def macs_per_window(C):
    return 588 * C * C + 4802 * C


def ideal_windows_per_s(C):
    """Fused ideal of one block: one fp32 read and one fp32 write of the map (392 C bytes per window)
    against 2 (588 C^2 + 4802 C) int8 operations per window, whichever binds."""
    return min(PEAK_HBM_GBS * 1e9 / (392 * C), PEAK_INT8_TOPS * 1e12 / (2 * macs_per_window(C)))


# VALU instructions per element of the pinned arithmetic (one lane-operation each): dequantize = cvt + fma,
# quantize = fma + med3 + 3/4 pack, GELU = 9, LayerNorm = 8 (+ quantize), softmax element = 17 (+ quantize)
ALU_DEQ, ALU_Q, ALU_GELU, ALU_LN, ALU_SOFTMAX = 2.0, 2.75, 9.0, 8.0, 17.0


def kernel_work(name, C, F, heads, n_windows):
    """Algorithmic work of one launch over n_windows windows: dict(hbm_bytes, mfma_ops, alu_lane_ops); None where
    a kind of work does not apply.  HBM bytes are the per-window figures of the scope table: a score or gather
    kernel reads the fp32 map (196 C), codes are 49 C bytes, the scatter writes 196 C."""
    w = dict(hbm_bytes=None, mfma_ops=None, alu_lane_ops=None)
    if name == "score":
        w["hbm_bytes"] = n_windows * (4 * T * C + 8)
    elif name == "select":
        w["hbm_bytes"] = n_windows * (8 + 4)
    elif name in ("gather_ln1_quant", "ln2_quant"):
        w["hbm_bytes"] = n_windows * (4 * T * C + T * C)
    elif name == "qkv_gemm":
        w["mfma_ops"] = n_windows * 2 * T * C * 3 * C
    elif name == "window_attention":
        w["mfma_ops"] = n_windows * 2 * 2 * T * T * C
    elif name == "proj_gemm_residual":
        w["mfma_ops"] = n_windows * 2 * T * C * C
    elif name in ("fc1_gemm_gelu", "fc2_gemm_residual_scatter"):
        w["mfma_ops"] = n_windows * 2 * T * C * F
    elif name == "window_ln1_qkv_attention":     # reads the map, writes the attention-output codes
        w["hbm_bytes"] = n_windows * (4 * T * C + T * C)
        w["mfma_ops"] = n_windows * 2 * (T * C * 3 * C + 2 * T * T * C)
        w["alu_lane_ops"] = n_windows * (T * C * (ALU_LN + ALU_Q) + T * 3 * C * (ALU_DEQ + ALU_Q) +
                                         heads * T * T * (ALU_SOFTMAX + ALU_Q) + T * C * (ALU_DEQ + 1 + ALU_Q))
    elif name == "token_proj_ln2_ffn_scatter":   # reads the shortcut and the codes, writes the map
        w["hbm_bytes"] = n_windows * (4 * T * C + T * C + 4 * T * C)
        w["mfma_ops"] = n_windows * 2 * (T * C * C + 2 * T * C * F)
        w["alu_lane_ops"] = n_windows * (T * C * (ALU_DEQ + 1) + T * C * (ALU_LN + ALU_Q) +
                                         T * F * (ALU_DEQ + ALU_GELU + ALU_Q) + T * C * (ALU_DEQ + 1))
    else:
        raise KeyError(name)
    return w


def price_kernel(name, avg_ms, C, F, heads, n_windows):
    """The launch against the roofline that bounds its algorithmic work: HBM for the memory kernels and for the
    fused kernels up to C = 192 (their intensity is below the machine balance of 625 op/B), int8 MFMA otherwise.
    The other views of the same launch are kept beside it."""
    w = kernel_work(name, C, F, heads, n_windows)
    sec = avg_ms * 1e-3
    out = dict(avg_ms=round(avg_ms, 5))
    fused = w["hbm_bytes"] is not None and w["mfma_ops"] is not None
    bound = "hbm" if (w["mfma_ops"] is None or (fused and C <= 192)) else "mfma"
    if bound == "hbm":
        ach = w["hbm_bytes"] / sec / 1e9
        out.update(bound="hbm", achieved=round(ach, 1), peak=PEAK_HBM_GBS, unit="GB/s", frac=round(ach / PEAK_HBM_GBS, 5),
                   algorithmic_bytes=w["hbm_bytes"])
    else:
        ach = w["mfma_ops"] / sec / 1e12
        out.update(bound="mfma", achieved=round(ach, 2), peak=PEAK_INT8_TOPS, unit="TOP/s", frac=round(ach / PEAK_INT8_TOPS, 5),
                   algorithmic_ops=w["mfma_ops"])
    if fused:
        t = w["mfma_ops"] / sec / 1e12
        g = w["hbm_bytes"] / sec / 1e9
        a = w["alu_lane_ops"] / sec / 1e12
        out.update(int8_tops=round(t, 2), frac_int8_mfma_peak=round(t / PEAK_INT8_TOPS, 5), hbm_gbs=round(g, 1),
                   frac_hbm_peak=round(g / PEAK_HBM_GBS, 5),
                   alu_model=dict(lane_ops=int(w["alu_lane_ops"]), achieved_tlops=round(a, 3), peak_tlops=PEAK_VALU_TLOPS,
                                  frac=round(a / PEAK_VALU_TLOPS, 5)))
    return out


def read_traffic(kernel, workload):
    """HBM bytes per launch of `kernel` from the committed counter summary of that workload (two rocprofv3 --pmc
    runs of this command, FETCH_SIZE and WRITE_SIZE), or None when no summary is there."""
    path = os.path.join(ROOT, "profiles", "%s_hbm_traffic.txt" % workload)
    try:
        for line in open(path):
            parts = line.split()
            if len(parts) >= 3 and parts[0] == "traffic_bytes_per_launch" and parts[1] == kernel:
                return int(float(parts[2]))
    except OSError:
        pass
    return None


class Stage:
    """One stage of a workload on the GPU: blocks, buffers, the stage call and its per-kernel profile."""

    def __init__(self, M, synth, torch, wl, si, keep):
        st = wl["stages"][si]
        self.M, self.torch = M, torch
        self.spec, self.shifts = st["spec"], st["shifts"]
        spec = self.spec
        self.k_high = M.mixaq_keep_count(spec.nW, keep)
        self.keep = keep
        self.x_np = synth.make_feature_map(spec, wl["seed"] + si, blobs=wl["blobs"], outlier_channels=wl["outliers"])
        self.inputs = [synth.make_block_inputs(spec, wl["seed"] + 10 * i, ranges=wl.get("ranges")) for i, _ in enumerate(self.shifts)]
        dev = torch.device("cuda:0")
        self.x = torch.from_numpy(self.x_np).to(dev)
        self.blocks = []
        for inp, shift in zip(self.inputs, self.shifts):
            sh, br = M.to_device(inp)
            self.blocks.append(M.mixaq_block_create(M.make_desc(spec, shift), sh, br))
        self.ws = M.alloc_workspace(self.blocks[0])
        self.scores = torch.empty((spec.B, spec.nW), dtype=torch.float64, device=dev)
        self.perm = torch.empty((spec.B, spec.nW), dtype=torch.int32, device=dev)
        self.bufs = [torch.empty_like(self.x), torch.empty_like(self.x)]
        self.n_pairs = (len(self.blocks) + 1) // 2
        self.n_win = spec.B * spec.nW

    def step(self):
        # one C call for the stage: score once; the first block takes the selection from the scores inside its
        # first kernel and leaves the list for the stage's other blocks
        return self.M.mixaq_stage_forward(self.blocks, self.x, [self.k_high] * self.n_pairs, None, self.bufs[0], self.bufs[1],
                                          self.scores, self.perm, self.ws)

    def spin_up(self, seconds=0.15):
        """Untimed steps until the shader clock has settled (about 50 ms of work)."""
        t0 = time.perf_counter()
        while time.perf_counter() - t0 < seconds:
            for _ in range(20):
                self.step()
            self.torch.cuda.synchronize()

    def time_steps(self, steps, warmup):
        for _ in range(warmup):
            self.step()
        self.torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step()
        self.torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    def profile(self, prof_steps, rep=4):
        """Per-kernel durations with HIP events on the launch stream (each kernel launched `rep` times between an
        event pair); returns {kernel: dict(avg_ms, launches_per_step, roofline fields)}."""
        M, torch = self.M, self.torch
        names = [M.mixaq_kernel_name(i) for i in range(M.NUM_KERNELS)]
        acc = {n: 0.0 for n in names}
        launches = {n: 0 for n in names}
        for _ in range(prof_steps):
            cur = self.x
            for i, blk in enumerate(self.blocks):
                dst = self.bufs[i % 2]
                if i == 0:      # scores and selection inside the call: the score kernel is timed like the others
                    ms = M.mixaq_block_forward_profile(blk, cur, None, self.k_high, dst, self.ws, repeats=rep)
                else:           # self.perm holds the stage's list since the timed steps
                    ms = M.mixaq_block_forward_profile(blk, cur, self.perm, self.k_high, dst, self.ws, repeats=rep)
                cur = dst
                for n, v in ms.items():
                    if v > 0:
                        acc[n] += v
                        launches[n] += 1
        spec = self.spec
        kernels = {}
        for n in names:
            if launches[n]:
                k = price_kernel(n, acc[n] / launches[n], spec.C, spec.C * spec.mlp_ratio, spec.heads, self.n_win)
                k["launches_per_step"] = round(launches[n] / prof_steps, 2)
                kernels[n] = k
        return kernels

    def summary(self, ms_per_pass, kernels):
        spec = self.spec
        windows = self.n_win * len(self.blocks)
        ops = 2 * macs_per_window(spec.C) * windows
        wps = windows / (ms_per_pass * 1e-3)
        tops = ops / (ms_per_pass * 1e-3) / 1e12
        out = dict(C=spec.C, B=spec.B, heads=spec.heads, windows_per_block=self.n_win, blocks=len(self.blocks), keep=self.keep,
                   k_high=self.k_high, bits="W%dA%d/A%d" % (spec.weight_bits, spec.act_bits_high, spec.act_bits_low),
                   ms_per_pass=round(ms_per_pass, 5), windows_per_s=round(wps, 1), int_tops=round(tops, 2),
                   pct_int8_mfma_peak=round(100 * tops / PEAK_INT8_TOPS, 3),
                   ideal_windows_per_s=round(ideal_windows_per_s(spec.C), 1),
                   frac_of_fused_ideal=round(wps / ideal_windows_per_s(spec.C), 5))
        if spec.B >= 2 and self.n_win <= 4096 and spec.C <= 384 and len(self.blocks) > 1:
            out["two_chains"] = ("the stage call runs the two halves of the batch as two chains of blocks on two streams; the per-kernel "
                                 "durations below are whole-batch launches on one stream and add up to more than ms_per_pass")
        if kernels:
            per_step = {n: kernels[n]["avg_ms"] * kernels[n]["launches_per_step"] for n in kernels}
            dom = max(per_step, key=per_step.get)
            out["kernels"] = kernels
            out["dominant"] = dict(kernel=dom, **{k: kernels[dom][k] for k in ("bound", "achieved", "peak", "unit", "frac", "avg_ms")})
        return out

    def close(self):
        for blk in self.blocks:
            self.M.mixaq_block_destroy(blk)
        self.blocks = []


def oracle_stage(O, stage, n_blocks, threads):
    """The oracle on the first n_blocks blocks of a stage (score + select + blocks); returns (seconds, windows)."""
    t0 = time.perf_counter()
    scores = O.score_windows(stage.inputs[0], stage.x_np)
    perm = O.select_windows(scores, stage.k_high)
    cur = stage.x_np
    for inp, shift in list(zip(stage.inputs, stage.shifts))[:n_blocks]:
        cur, _ = O.block_forward(inp, cur, perm, stage.k_high, shift, threads=threads)
    return time.perf_counter() - t0, stage.n_win * n_blocks


def backbone_chain(M, synth, torch, steps):
    """Config 4 as one chain: patch embedding, four stages, a patch merging between stages; ms per image."""
    bb = synth.backbone("cfg4")
    B, Hi, Wi = bb["image"]
    seed = bb["seed"]
    dev = torch.device("cuda:0")
    img = torch.from_numpy(synth.make_image(B, Hi, Wi, seed)).to(dev)
    downs = [M.mixaq_downsample_create(M.make_downsample_desc(sp), M.downsample_to_device(synth.make_downsample_inputs(sp, seed + 1 + i)))
             for i, sp in enumerate([bb["embed"]] + bb["merges"])]
    stages = []
    for si, st in enumerate(bb["stages"]):
        spec = st["spec"]
        blocks = []
        for i, sh in enumerate(st["shifts"]):
            s_, b_ = M.to_device(synth.make_block_inputs(spec, seed + 100 * si + 10 * i))
            blocks.append(M.mixaq_block_create(M.make_desc(spec, sh), s_, b_))
        x = torch.empty((spec.B, spec.H, spec.W, spec.C), device=dev)
        stages.append(dict(blocks=blocks, ws=M.alloc_workspace(blocks[0]), x=x, y=torch.empty_like(x), tmp=torch.empty_like(x),
                           scores=torch.empty((spec.B, spec.nW), dtype=torch.float64, device=dev),
                           perm=torch.empty((spec.B, spec.nW), dtype=torch.int32, device=dev),
                           k=M.mixaq_keep_count(spec.nW, bb["keep"][0]), pairs=(len(blocks) + 1) // 2))

    def run():
        cur = img
        for si, S in enumerate(stages):
            M.mixaq_downsample_forward(downs[si], cur, S["x"])
            M.mixaq_stage_forward(S["blocks"], S["x"], [S["k"]] * S["pairs"], None, S["y"], S["tmp"], S["scores"], S["perm"], S["ws"])
            cur = S["y"]
    for _ in range(30):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        run()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    for S in stages:
        for b in S["blocks"]:
            M.mixaq_block_destroy(b)
    for d in downs:
        M.mixaq_downsample_destroy(d)
    windows = sum(st["spec"].B * st["spec"].nW * len(st["shifts"]) for st in bb["stages"])
    ops = sum(2 * macs_per_window(st["spec"].C) * st["spec"].B * st["spec"].nW * len(st["shifts"]) for st in bb["stages"])
    return dict(ms_per_image=round(ms, 4), windows_per_s=round(windows / (ms * 1e-3), 1), int_tops_blocks_only=round(ops / (ms * 1e-3) / 1e12, 2),
                note="patch embedding + 4 stages + 3 patch mergings per image; the int-TOPS count the blocks' operations only")


def calibration_copy(torch, dev):
    """A plain copy of known size, so that a counter run of this same command can calibrate FETCH_SIZE /
    WRITE_SIZE against bytes (64 MiB read + 64 MiB written)."""
    calib_src = torch.empty(64 * 1024 * 1024, dtype=torch.uint8, device=dev)
    calib_dst = torch.empty_like(calib_src)
    calib_dst.copy_(calib_src)
    torch.cuda.synchronize()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=500)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--headline-only", action="store_true", help="skip configs 1, 3, 4, 5")
    ap.add_argument("--workload", default=None, help="run ONE workload's stage only (cfg1..cfg5), e.g. under rocprofv3")
    ap.add_argument("--stage", type=int, default=0, help="stage of --workload")
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
    threads = int(os.environ.get("OMP_NUM_THREADS", "0")) or min(16, os.cpu_count() or 1)
    O = None
    if not args.no_cpu_baseline:
        sys.path.insert(0, os.path.join(ROOT, "tests"))
        import oracle_api as O              # the oracle is used for the cpu_baseline legs only

    if args.workload:            # one stage on its own: what a profiler run of a single workload executes
        wln = synth.workload(args.workload)
        stg = Stage(M, synth, torch, wln, args.stage, wln["keep"][len(wln["keep"]) // 2])
        stg.spin_up()
        ms = stg.time_steps(args.steps, args.warmup)
        s = stg.summary(ms, stg.profile(min(args.steps, 50)))
        s.update(workload=args.workload, stage=args.stage, steps=args.steps, warmup=args.warmup)
        stg.close()
        calibration_copy(torch, dev)
        print(json.dumps(s))
        return 0

    # ---------------------------------------------------------------- headline: config 2
    wl = synth.workload("cfg2")
    head = Stage(M, synth, torch, wl, 0, wl["keep"][0])
    spec = head.spec
    head.spin_up()
    ms_per_step = head.time_steps(args.steps, args.warmup)
    kernels = head.profile(min(args.steps, 200))
    per_step = {n: kernels[n]["avg_ms"] * kernels[n]["launches_per_step"] for n in kernels}
    dom = max(per_step, key=per_step.get)
    kd = kernels[dom]
    roofline = dict(kernel=dom, bound=kd["bound"], achieved=kd["achieved"], peak=kd["peak"], unit=kd["unit"], frac=kd["frac"],
                    traffic=read_traffic(dom, "cfg2"), traffic_source="profiles/cfg2_hbm_traffic.txt (rocprofv3 --pmc runs of this command)",
                    avg_ms=kd["avg_ms"])
    for k in ("algorithmic_bytes", "algorithmic_ops", "int8_tops", "frac_int8_mfma_peak", "alu_model"):
        if k in kd:
            roofline[k] = kd[k]

    # The same step with the score taken after a LayerNorm (score_mode 1: the scoring LayerNorm's parameters are
    # the high branch's LN1 here); only the score kernel differs, and with it which windows are selected.
    d1 = M.make_desc(spec, head.shifts[0])
    d1.score_mode = 1
    sh1, br1 = M.to_device(head.inputs[0])
    first = head.blocks[0]
    head.blocks[0] = M.mixaq_block_create(d1, sh1, br1)
    ms_per_step_m1 = head.time_steps(args.steps, args.warmup)
    M.mixaq_block_destroy(head.blocks[0])
    head.blocks[0] = first

    windows_per_step = head.n_win * len(head.blocks)
    ops_per_step = 2 * macs_per_window(spec.C) * windows_per_step
    value = windows_per_step / (ms_per_step * 1e-3)
    int_tops = ops_per_step / (ms_per_step * 1e-3) / 1e12

    cpu = None
    if O is not None:
        dt, nwin = oracle_stage(O, head, len(head.blocks), 1)
        dt_mp, _ = oracle_stage(O, head, len(head.blocks), threads)
        cpu = dict(value=round(nwin / dt, 2), unit="windows/s", cores=1, kind="oracle",
                   sample="one full step of the same workload (score + select + both blocks, 2784 windows), single thread",
                   seconds=round(dt, 2), int_tops=round(ops_per_step / dt / 1e12, 5),
                   openmp=dict(value=round(nwin / dt_mp, 2), unit="windows/s", cores=threads, seconds=round(dt_mp, 2),
                               sample="the same step, windows split over OpenMP threads"))

    configs = {}
    configs["cfg2"] = dict(workload="Swin-T stage-1 pair, 200x336x96, keep 0.5", stages=[head.summary(ms_per_step, kernels)])
    head.close()

    # ---------------------------------------------------------------- the other workloads
    if not args.headline_only:
        descr = dict(cfg1="single regular block, 56x56x96, keep 0.5",
                     cfg3="Swin-T stage-3 stack of 6 blocks, batch 2, 50x84x384, keep swept",
                     cfg4="Swin-T backbone stages at 800x1344, W4A4 with 2-bit low windows, keep 0.5",
                     cfg5="Swin-B-shaped stages 1 and 2, batch 4, 256x256x128 and 128x128x256, keep 0.4, outlier channels")
        for name in ("cfg1", "cfg3", "cfg4", "cfg5"):
            wln = synth.workload(name)
            entry = dict(workload=descr[name], stages=[])
            for si in range(len(wln["stages"])):
                for ki, keep in enumerate(wln["keep"]):
                    stg = Stage(M, synth, torch, wln, si, keep)
                    stg.spin_up(0.05)
                    ms = stg.time_steps(200, 50)
                    last = ki == len(wln["keep"]) // 2
                    kern = stg.profile(20) if last else None
                    s = stg.summary(ms, kern)
                    s["stage"] = si
                    if O is not None and last:          # the oracle on one block of this stage, OpenMP over windows
                        dt, nwin = oracle_stage(O, stg, 1, threads)
                        s["cpu_oracle"] = dict(windows_per_s=round(nwin / dt, 2), cores=threads, seconds=round(dt, 2),
                                               sample="score + select + the first block of the stage (%d windows)" % nwin)
                    entry["stages"].append(s)
                    stg.close()
            if name == "cfg4":
                entry["chain"] = backbone_chain(M, synth, torch, 100)
            configs[name] = entry

    # ---------------------------------------------------------------- config 2's shape at larger batches (context, not the headline)
    # One 200x336 map gives every CU five or six windows per kernel, so each of the five kernels of a step runs
    # mostly in its ramp-up and its tail; the same kernels on a batch show the rate they sustain once the chip is full.
    batch_scaling = None
    if not args.headline_only:
        import dataclasses
        batch_scaling = []
        for b in (2, 4, 8):
            st0 = wl["stages"][0]
            wlb = dict(wl, stages=[dict(st0, spec=dataclasses.replace(st0["spec"], B=b))])
            stg = Stage(M, synth, torch, wlb, 0, wl["keep"][0])
            stg.spin_up(0.05)
            ms = stg.time_steps(300, 50)
            wps = stg.n_win * len(stg.blocks) / (ms * 1e-3)
            batch_scaling.append(dict(B=b, ms_per_pass=round(ms, 5), windows_per_s=round(wps, 1),
                                      int_tops=round(2 * macs_per_window(spec.C) * wps / 1e12, 2)))
            stg.close()

    out = dict(metric="windows/sec & effective int-TOPS per two-branch Swin block; % int8 MFMA peak",
               value=round(value, 1), unit="windows/s", n_gpus=1, steps=args.steps, warmup=args.warmup,
               ms_per_step=round(ms_per_step, 5), higher_is_better=True, scaling="weak", vs_baseline=None,
               dtype="int8 (int32 accumulate, fp32 epilogues)", data="synthetic",
               config=dict(workload="cfg2: Swin-T stage-1 pair (regular + shifted block), B=1, 200x336x96 padded to 203x336, "
                                    "1392 windows, 3 heads, keep 0.5, A8/A4, W8", blocks_per_step=2,
                           windows_per_step=windows_per_step, k_high=configs["cfg2"]["stages"][0]["k_high"], score_mode=0),
               score_after_layernorm=dict(score_mode=1, ms_per_step=round(ms_per_step_m1, 5),
                                          value=round(windows_per_step / (ms_per_step_m1 * 1e-3), 1)),
               int_tops=round(int_tops, 3), pct_int8_mfma_peak=round(100 * int_tops / PEAK_INT8_TOPS, 3),
               ms_per_block=round(ms_per_step / 2, 5), frac_of_fused_ideal=round(value / ideal_windows_per_s(spec.C), 5),
               roofline=roofline, kernels=kernels, cpu_baseline=cpu, configs=configs,
               cfg2_shape_at_larger_batches=batch_scaling)
    calibration_copy(torch, dev)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
