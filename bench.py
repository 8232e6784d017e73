#!/usr/bin/env python3
"""Benchmark of the FB4 online quantizer on one MI355X.

A step is one pass of the hot path -- fb4_quantize with the paper's online
selector (Qerror over 8 group-wise maxima, all 32 dialects, block 32) -- over
one 16384 x 3072 bf16 activation tensor already resident in HBM.  Steps rotate
through several input/output buffer sets (more than 512 MB in total) so that
the 129 MB working set is streamed from HBM and not served by the 256 MB
Infinity Cache.  Prints ONE JSON line.

The other entry points (exhaustive selector, g = 32, SeDA, decomposition,
dequantize, MXFP8 repack) and the other workloads (cfg1, cfg5 activation and
weight) are timed the same way and reported under "extras".
"""

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# HBM bytes per launch of the headline kernel (rocprofv3 FETCH_SIZE / WRITE_SIZE, each scaled by what the same
# counter reads for a plain copy of known size) and the kernel's name come from this summary, which
# paper_2603_02883_amd/profile_summary.py writes from raw rocprofv3 output; without the file both are null.
TRAFFIC_SUMMARY = os.path.join(ROOT, "profiles", "headline_kernel_traffic.txt")
ROWS, COLS, BLOCK = 16384, 3072, 32
N_SETS = 6
SETTLE_S = 0.05   # untimed load before a timed graph replay


def algorithmic_bytes(rows, cols, block=32):
    """bf16 in + 4-bit codes out + 16-bit metadata per block out."""
    return rows * cols * 2 + rows * cols // 2 + rows * (cols // block) * 2


def time_graph(fn_steps, steps, warmup):
    """Run a few eager steps (at most 100), capture `steps` steps into one HIP graph, replay it untimed (until `warmup`
    steps have been replayed and the card has been under load for SETTLE_S seconds: the capture leaves it idle
    for a moment, and from idle the clocks take 20 to 25 ms of load to come back up), then once timed.
    Returns (wall seconds, event seconds) for the timed replay."""
    import torch
    for i in range(min(warmup, 100)):
        fn_steps(i)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            for i in range(steps):
                fn_steps(i)
    torch.cuda.synchronize()
    replays, t_load = 0, time.perf_counter()
    while replays * steps < warmup or time.perf_counter() - t_load < SETTLE_S:
        g.replay()
        g.replay()
        torch.cuda.synchronize()
        replays += 2
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    g.replay()
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return wall, e0.elapsed_time(e1) * 1e-3


def time_eager(fn_steps, steps, warmup):
    import torch
    for i in range(warmup):
        fn_steps(i)
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for i in range(steps):
        fn_steps(i)
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return wall, e0.elapsed_time(e1) * 1e-3


def selector_agreement(F, luts, synth):
    """Per workload: fraction of blocks on which a selector picks the same dialect as the exhaustive one, and
    its total squared error relative to the exhaustive selector's (>= 1).  Evaluation only: the comparison
    runs in torch on the dequantized fp32 tensors."""
    import torch
    work = {
        "cfg1": lambda: synth.gaussian_outlier(rows=1024, cols=3072, seed=1, device="cuda"),
        "cfg2": lambda: synth.vdit_activation(rows=16384, cols=3072, seed=2, device="cuda"),
        "cfg4": lambda: synth.mixture_activation(rows=16384, cols=3072, seed=4, device="cuda")[0],
        "cfg5_activation": lambda: synth.vdit_activation(rows=65536, cols=12288, seed=5, device="cuda",
                                                         outlier_frac=0.01),
        "cfg5_weight": lambda: synth.weight_matrix(rows=12288, cols=3072, seed=5, device="cuda"),
    }
    variants = {"lut_g8": F.opts(selector=F.SEL_LUT, num_groups=8),
                "lut_g8_two_stage": F.opts(selector=F.SEL_LUT, num_groups=8, flags=F.FLAG_TWO_STAGE),
                "lut_g16": F.opts(selector=F.SEL_LUT, num_groups=16),
                "lut_g32": F.opts(selector=F.SEL_LUT, num_groups=32)}

    def sq_err(x, c, m):
        total = 0.0
        for r0 in range(0, x.shape[0], 8192):           # in row chunks: the fp32 copies stay small
            y = F.fb4_dequantize(luts, c[r0:r0 + 8192], m[r0:r0 + 8192], out_dtype=F.DTYPE_F32)
            d = (x[r0:r0 + 8192].float() - y).double()
            d = torch.where(torch.isfinite(d), d, torch.zeros_like(d))
            total += float((d * d).sum())
        return total

    out = {}
    for name, make in work.items():
        x = make()
        c0, m0 = F.fb4_quantize(luts, F.opts(selector=F.SEL_SSE), x)
        e0 = sq_err(x, c0, m0)
        res = {"blocks": int(m0.numel())}
        for vname, o in variants.items():
            c, m = F.fb4_quantize(luts, o, x)
            same = float(((m & 0xFF) == (m0 & 0xFF)).float().mean())
            res[vname] = {"same_dialect": round(same, 4), "squared_error_ratio": round(sq_err(x, c, m) / e0, 4)}
            del c, m
        out[name] = res
        del x, c0, m0
        torch.cuda.empty_cache()
    return {"selector_agreement": out, "reference": "exhaustive squared-error selector", "block": 32}


def pruning_study(n_wavefronts=512):
    """CPU only (numpy, no library, no oracle): how much work exact early-exit pruning of the exhaustive selector
    could save on the first n_wavefronts * 64 blocks of cfg2.  A dialect is dropped for a block once its partial
    squared error exceeds the total of the best dialect (the most favourable incumbent there is); a wavefront,
    which holds 64 blocks in its lanes, executes the union of their surviving dialects."""
    import numpy as np

    from fb4_inputs import DEFAULT_FORMATBOOK, synth
    fbk = np.asarray(DEFAULT_FORMATBOOK, dtype=np.float64)
    n_blocks = 64 * n_wavefronts
    rows = (n_blocks * 32 + 3071) // 3072
    x = synth.vdit_activation(rows=rows, cols=3072, seed=2, device="cpu").float().numpy().astype(np.float64)
    blocks = np.abs(x.reshape(-1, 32))[:n_blocks]
    per_block = np.zeros(32)
    union = np.zeros(32)
    gaps = []
    for lo in range(0, n_blocks, 64 * 32):                                            # 32 wavefronts at a time
        blk = blocks[lo:lo + 64 * 32]
        e = np.floor(np.log2(np.maximum(blk.max(1), 1e-30)))
        xn = blk * 2.0 ** (3 - e)[:, None]
        err = np.abs(xn[:, :, None, None] - fbk[None, None, :, :]).min(-1) ** 2      # [block][element][dialect]
        srt = np.sort(err.sum(1), 1)
        gaps.append((srt[:, 1] - srt[:, 0]) / np.maximum((xn ** 2).sum(1) - srt[:, 0], 1e-300))
        alive = np.cumsum(err, 1) <= srt[:, :1, None] + 1e-12                        # [block][elements seen][dialect]
        per_block += alive.sum(2).sum(0)
        union += alive.reshape(-1, 64, 32, 32).any(1).sum(2).sum(0)
    per_block /= n_blocks
    union /= n_wavefronts
    work = lambda a: float(np.concatenate([[32.0], a[:-1]]).sum() / 1024)
    return {"pruning_study": {
        "blocks": int(n_blocks),
        "median_gap_best_to_runner_up_rel_to_Z": float(np.median(np.concatenate(gaps))),
        "alive_dialects_per_block_after_8_16_24_32_elements": [float(per_block[k]) for k in (7, 15, 23, 31)],
        "alive_in_wavefront_union_after_8_16_24_32_elements": [float(union[k]) for k in (7, 15, 23, 31)],
        "work_fraction_per_block_pruning": work(per_block), "work_fraction_wavefront_union": work(union)}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=1000)
    ap.add_argument("--eager", action="store_true", help="time eager launches instead of one HIP graph")
    ap.add_argument("--no-extras", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--selector-agreement", action="store_true",
                    help="instead of timing: how often the online selectors pick the exhaustive selector's "
                         "dialect, and what the difference costs in squared error, on the five workloads")
    ap.add_argument("--pruning-study", action="store_true",
                    help="CPU only: what exact early-exit pruning of the exhaustive selector could save on cfg2")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="for `rocprofv3 --pmc ...`: a few plain device copies of known size, then a few "
                         "launches of the headline kernel, of the exhaustive selector and of the other streaming "
                         "kernels; prints a marker line")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (the path has no multi-GPU part); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    if args.pruning_study:
        print(json.dumps(pruning_study()))
        return

    import numpy as np
    import torch

    import paper_2603_02883_amd as F
    from fb4_inputs import DEFAULT_FORMATBOOK, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    timer = time_eager if args.eager else time_graph
    luts = F.fb4_build_luts(DEFAULT_FORMATBOOK)

    if args.selector_agreement:
        print(json.dumps(selector_agreement(F, luts, synth)))
        luts.free()
        return

    x0 = synth.vdit_activation(rows=ROWS, cols=COLS, seed=2, device="cuda")
    xs = [x0] + [x0.clone() for _ in range(N_SETS - 1)]
    codes = [torch.empty((ROWS, COLS // 2), dtype=torch.uint8, device="cuda") for _ in range(N_SETS)]
    metas = [torch.empty((ROWS, COLS // BLOCK), dtype=torch.int16, device="cuda") for _ in range(N_SETS)]
    n_el = ROWS * COLS
    abytes = algorithmic_bytes(ROWS, COLS)

    if args.traffic_probe:
        # plain copy kernel of known size: reads 100,663,296 B and writes 100,663,296 B per launch
        dst = torch.empty_like(x0)
        o = F.opts(block=BLOCK, selector=F.SEL_LUT, num_groups=8)
        for i in range(10):
            dst.copy_(xs[i % N_SETS])
        for i in range(10):
            F.fb4_quantize(luts, o, xs[i % N_SETS], codes=codes[i % N_SETS], meta=metas[i % N_SETS])
        # the exhaustive selector, for its instruction and LDS counters
        o_sse = F.opts(block=BLOCK, selector=F.SEL_SSE)
        for i in range(4):
            F.fb4_quantize(luts, o_sse, xs[i % N_SETS], codes=codes[i % N_SETS], meta=metas[i % N_SETS])
        # the other streaming kernels: both planes in one pass, the second plane alone, decode, repack
        sal_d = torch.from_numpy(synth.salient_rows_from_attention(ROWS, frac=0.05, heads=24, seed=3,
                                                                   device="cuda")).cuda()
        c2 = torch.empty((sal_d.numel(), COLS // 2), dtype=torch.uint8, device="cuda")
        m2 = torch.empty((sal_d.numel(), COLS // BLOCK), dtype=torch.int16, device="cuda")
        outs = [torch.empty((ROWS, COLS), dtype=torch.bfloat16, device="cuda") for _ in range(2)]
        els = [torch.empty((ROWS, COLS), dtype=torch.uint8, device="cuda") for _ in range(2)]
        scs = [torch.empty((ROWS, COLS // 32), dtype=torch.uint8, device="cuda") for _ in range(2)]
        for i in range(4):
            k = i % N_SETS
            F.fb4_quantize_decompose(luts, o, xs[k], sal_d, codes1=codes[k], meta1=metas[k], codes2=c2, meta2=m2)
            F.fb4_decompose(luts, o, xs[k], codes[k], metas[k], sal_d, codes2=c2, meta2=m2)
            F.fb4_dequantize(luts, codes[k], metas[k], out=outs[i % 2])
            F.fb4_dequantize(luts, codes[k], metas[k], codes2=c2, meta2=m2, salient_rows=sal_d, out=outs[i % 2])
            F.fb4_repack_mxfp8(luts, codes[k], metas[k], elems=els[i % 2], scales=scs[i % 2])
        # attention scores of 384 groups x 1024 tokens x 128 channels, and the per-tile choice
        qa, ka = synth.attention_qk(16 * 24, 1024, 128, seed=7, device="cuda")
        att = torch.empty((16 * 24, 1024), dtype=torch.float32, device="cuda")
        for i in range(4):
            F.fb4_attention_scores(qa, ka, 0, scores=att)
            F.fb4_select_salient_tokens(att.view(16, 24, 1024), 32, 32)
        # GeLU + quantizer in one pass
        for i in range(4):
            k = i % N_SETS
            F.fb4_gelu_quantize(luts, o, xs[k], 1, codes=codes[k], meta=metas[k])
        # LayerNorm + quantizer in one pass
        gamma_h, beta_h = synth.layernorm_affine(COLS)
        gamma_d, beta_d = torch.from_numpy(gamma_h).cuda(), torch.from_numpy(beta_h).cuda()
        for i in range(4):
            k = i % N_SETS
            F.fb4_layernorm_quantize(luts, o, xs[k], gamma_d, beta_d, 1e-6, codes=codes[k], meta=metas[k])
        torch.cuda.synchronize()
        print(json.dumps({"traffic_probe": True, "copy_bytes_read": x0.numel() * 2, "copy_bytes_written": x0.numel() * 2,
                          "quantize_algorithmic_bytes": abytes}))
        luts.free()
        return

    def quant_step(o):
        def f(i):
            k = i % N_SETS
            F.fb4_quantize(luts, o, xs[k], codes=codes[k], meta=metas[k])
        return f

    # ---- headline: the paper's online selector
    o_main = F.opts(block=BLOCK, selector=F.SEL_LUT, num_groups=8)
    from paper_2603_02883_amd.profile_summary import read_summary
    summary = read_summary(TRAFFIC_SUMMARY)
    wall, ev = timer(quant_step(o_main), args.steps, args.warmup)
    ms_per_step = wall * 1e3 / args.steps
    kern_s = ev / args.steps
    result = {
        "metric": "G elements/s quantized + achieved HBM GB/s (% of peak), 16384x3072 bf16",
        "value": n_el / (wall / args.steps) / 1e9,
        "unit": "G elements/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u16",
        "data": "synthetic",
        "config": {
            "workload": "cfg2: Open-Sora-2.0-like VDiT activation 16384x3072 bf16, Student-t(3), per-frame "
                        "scale drift, 0.5% outlier channels x100",
            "entry_point": "fb4_quantize", "selector": "lut", "num_groups": 8, "block": BLOCK,
            "formatbook": "32 dialects (default table)", "buffer_sets": N_SETS,
            "launch": "eager" if args.eager else "hip_graph",
        },
        "roofline": {
            "bound": "hbm", "achieved": abytes / kern_s / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": abytes / kern_s / 1e9 / HBM_PEAK_GBS,
            "traffic": int(summary["traffic_bytes_per_launch"]) if "traffic_bytes_per_launch" in summary else None,
            "kernel": summary.get("kernel"), "kernel_us": kern_s * 1e6, "algorithmic_bytes": abytes,
            "traffic_source": os.path.relpath(TRAFFIC_SUMMARY, ROOT) if summary else None,
        },
    }

    # ---- other entry points, same protocol
    if not args.no_extras:
        extras = {}
        steps2 = max(10, args.steps // 4)

        def add(name, fn, nbytes, nelem, steps=steps2):
            w, e = timer(fn, steps, 2 * steps)
            extras[name] = {"us": e / steps * 1e6, "G_elements_per_s": nelem / (e / steps) / 1e9,
                            "GB_per_s": nbytes / (e / steps) / 1e9, "hbm_frac": nbytes / (e / steps) / 1e9 / HBM_PEAK_GBS}

        # the same launch on ONE buffer set: its 129 MB fit the 256 MB Infinity Cache (reported apart from the headline)
        def resident_step(i):
            F.fb4_quantize(luts, o_main, xs[0], codes=codes[0], meta=metas[0])
        add("quantize_lut_g8_one_buffer_set_cache_resident", resident_step, abytes, n_el)
        add("quantize_lut_g16", quant_step(F.opts(selector=F.SEL_LUT, num_groups=16)), abytes, n_el)
        add("quantize_lut_g32", quant_step(F.opts(selector=F.SEL_LUT, num_groups=32)), abytes, n_el)
        metas16 = [torch.empty((ROWS, COLS // 16), dtype=torch.int16, device="cuda") for _ in range(N_SETS)]
        o16 = F.opts(block=16, selector=F.SEL_LUT, num_groups=8)

        def b16_step(i):
            k = i % N_SETS
            F.fb4_quantize(luts, o16, xs[k], codes=codes[k], meta=metas16[k])
        add("quantize_block16_lut_g8", b16_step, algorithmic_bytes(ROWS, COLS, 16), n_el)
        add("quantize_lut_g8_two_stage", quant_step(F.opts(selector=F.SEL_LUT, num_groups=8,
                                                           flags=F.FLAG_TWO_STAGE)), abytes, n_el)
        # LayerNorm fused in front of the quantizer: x read once, the normalized tensor never written ...
        gamma_h, beta_h = synth.layernorm_affine(COLS)
        gamma_d, beta_d = torch.from_numpy(gamma_h).cuda(), torch.from_numpy(beta_h).cuda()

        def ln_step(i):
            k = i % N_SETS
            F.fb4_layernorm_quantize(luts, o_main, xs[k], gamma_d, beta_d, 1e-6, codes=codes[k], meta=metas[k])
        add("layernorm_quantize_one_pass", ln_step, abytes + 2 * COLS * 4, n_el)
        # ... against the two-pass form: the framework's LayerNorm writing bf16 (into a buffer that is reused at
        # once, so part of it is still in the Infinity Cache), then the quantizer reading that back
        gamma_b, beta_b = gamma_d.bfloat16(), beta_d.bfloat16()

        def ln_unfused_step(i):
            k = i % N_SETS
            y = torch.nn.functional.layer_norm(xs[k], (COLS,), gamma_b, beta_b, 1e-6)
            F.fb4_quantize(luts, o_main, y, codes=codes[k], meta=metas[k])
        add("layernorm_by_torch_then_quantize", ln_unfused_step, abytes + 2 * n_el * 2, n_el)
        # GeLU fused in front of the quantizer, against the framework's GeLU followed by the quantizer
        def gelu_step(i):
            k = i % N_SETS
            F.fb4_gelu_quantize(luts, o_main, xs[k], 1, codes=codes[k], meta=metas[k])
        add("gelu_quantize_one_pass", gelu_step, abytes, n_el)

        def gelu_unfused_step(i):
            k = i % N_SETS
            y = torch.nn.functional.gelu(xs[k], approximate="tanh")
            F.fb4_quantize(luts, o_main, y, codes=codes[k], meta=metas[k])
        add("gelu_by_torch_then_quantize", gelu_unfused_step, abytes + 2 * n_el * 2, n_el)
        # the fused producers with a scale per 16 elements and with 16 groups per block
        o_g16 = F.opts(block=BLOCK, selector=F.SEL_LUT, num_groups=16)

        def ln16_step(i):
            k = i % N_SETS
            F.fb4_layernorm_quantize(luts, o16, xs[k], gamma_d, beta_d, 1e-6, codes=codes[k], meta=metas16[k])
        add("layernorm_quantize_block16", ln16_step, algorithmic_bytes(ROWS, COLS, 16) + 2 * COLS * 4, n_el)

        def ln_g16_step(i):
            k = i % N_SETS
            F.fb4_layernorm_quantize(luts, o_g16, xs[k], gamma_d, beta_d, 1e-6, codes=codes[k], meta=metas[k])
        add("layernorm_quantize_g16", ln_g16_step, abytes + 2 * COLS * 4, n_el)

        def gelu16_step(i):
            k = i % N_SETS
            F.fb4_gelu_quantize(luts, o16, xs[k], 1, codes=codes[k], meta=metas16[k])
        add("gelu_quantize_block16", gelu16_step, algorithmic_bytes(ROWS, COLS, 16), n_el)

        def gelu_g16_step(i):
            k = i % N_SETS
            F.fb4_gelu_quantize(luts, o_g16, xs[k], 1, codes=codes[k], meta=metas[k])
        add("gelu_quantize_g16", gelu_g16_step, abytes, n_el)
        # SeDA (cfg4)
        xm, comp = synth.mixture_activation(rows=ROWS, cols=COLS, seed=4, device="cuda")
        xms = [xm] + [xm.clone() for _ in range(N_SETS - 1)]
        tg = torch.from_numpy(comp).cuda()
        sub = torch.from_numpy(synth.seda_sub_formatbooks(DEFAULT_FORMATBOOK, 64, 4)).cuda()

        def seda_step(i):
            k = i % N_SETS
            F.fb4_quantize_seda(luts, o_main, xms[k], tg, sub, codes=codes[k], meta=metas[k])
        add("quantize_seda_lut_g8", seda_step, abytes + ROWS * 4, n_el)
        # SeDA bookkeeping (Sec. 3.4): dialect counts of the anchor rows (every tenth row here) per group and
        # the eight-dialect sub-formatbooks from them; reads the metadata of the anchor rows only
        anchors = torch.from_numpy(np.where(np.arange(ROWS) % 10 == 0, comp, -1).astype(np.int32)).cuda()
        counts = torch.zeros((64, 32), dtype=torch.int32, device="cuda")
        subs = torch.zeros((64, 8), dtype=torch.uint8, device="cuda")

        def profile_step(i):
            F.fb4_seda_profile(luts, metas[i % N_SETS], anchors, 64, counts=counts, sub_formatbooks=subs)
        add("seda_profile_10pct_anchor_rows", profile_step, ROWS * 4 + (ROWS // 10) * (COLS // BLOCK) * 2,
            (ROWS // 10) * COLS)
        # attention-guided salient tokens (Sec. 3.3) for this tensor: 16 frames x 24 heads, 32 x 32 tokens per frame,
        # 128 channels per head; one token per 4 x 4 tile = 1024 rows
        qa, ka = synth.attention_qk(16 * 24, 1024, 128, seed=7, device="cuda")
        att = torch.empty((16 * 24, 1024), dtype=torch.float32, device="cuda")
        sal_rows = torch.empty((16, 64), dtype=torch.int32, device="cuda")

        def scores_step(i):
            F.fb4_attention_scores(qa, ka, 0, scores=att)
        w_s, e_s = timer(scores_step, steps2, 2 * steps2)
        flops = 2.0 * 16 * 24 * 1024 * 1024 * 128
        extras["attention_scores_384x1024x128"] = {"us": e_s / steps2 * 1e6, "TFLOP_per_s": flops / (e_s / steps2) / 1e12,
                                                   "mfma_frac": flops / (e_s / steps2) / 1e12 / 2500.0}

        # what the matrix cores sustain on operands held in registers (no memory traffic): with one bit pattern in
        # every element, and with random signs and mantissas -- the power management lowers the clock for the latter
        probe_out = torch.empty(512 * 256, dtype=torch.float32, device="cuda")
        for rnd in (0, 1):
            def probe_step(i, rnd=rnd):
                F.fb4_probe_mfma_rate(512, 400, rnd, out=probe_out)
            w_p, e_p = timer(probe_step, steps2, 4 * steps2)
            pflop = F.fb4_probe_mfma_rate(512, 400, rnd, out=probe_out)[1]
            extras["mfma_bf16_register_loop_%s_operands" % ("random" if rnd else "constant")] = {
                "us": e_p / steps2 * 1e6, "TFLOP_per_s": pflop / (e_p / steps2) / 1e12, "mfma_frac": pflop / (e_p / steps2) / 1e12 / 2500.0}
        extras["attention_scores_384x1024x128"]["frac_of_register_loop_random_operands"] = (
            extras["attention_scores_384x1024x128"]["TFLOP_per_s"] / extras["mfma_bf16_register_loop_random_operands"]["TFLOP_per_s"])

        def select_step(i):
            F.fb4_select_salient_tokens(att.view(16, 24, 1024), 32, 32, rows_out=sal_rows)
        add("select_salient_tokens_16x24x1024", select_step, 16 * 24 * 1024 * 4 + 16 * 64 * 4, 16 * 1024)
        # ... and the tokens each of those 1024 anchors is correlated with (5 x 5 window, Sec. 3.4)
        q4, k4 = qa.view(16, 24, 1024, 128), ka.view(16, 24, 1024, 128)

        def assign_step(i):
            F.fb4_seda_assign(q4, k4, sal_rows, 16, 32, 32, window=5, threshold=5.0)
        add("seda_assign_16x24x1024_window5", assign_step, 1024 * 26 * 24 * 128 * 2 + 2 * 16384 * 4, 16 * 1024)
        # step 2 of Sec. 3.4 for the same clip: temporal attention (1024 positions x 24 heads, 16 frames), the main
        # anchor of each of the 64 tiles among its 16 candidates and the pruning of weakly correlated frames
        qt, kt = synth.attention_qk(1024 * 24, 16, 128, seed=8, device="cuda")
        att_t = torch.empty((1024 * 24, 16), dtype=torch.float32, device="cuda")
        F.fb4_attention_scores(qt, kt, 1, scores=att_t)
        qt4, kt4 = qt.view(1024, 24, 16, 128), kt.view(1024, 24, 16, 128)

        def main_anchor_step(i):
            F.fb4_seda_main_anchor(att_t.view(1024, 24, 16), qt4, kt4, sal_rows, 32, 32, prune_threshold=3.0)
        add("seda_main_anchor_64_tiles_16_frames", main_anchor_step, 64 * 17 * 24 * 128 * 2 + 1024 * 24 * 4, 1024)
        # ... and the 3D variant's main anchors from per-head scores of all 16384 tokens
        att3 = att.view(16, 24, 1024).transpose(0, 1).contiguous().view(24, 16384)

        def main_anchor_3d_step(i):
            F.fb4_seda_main_anchor_3d(att3, 16, 32, 32)
        add("seda_main_anchor_3d_24x16384", main_anchor_3d_step, 24 * 16384 * 4, 16384)
        del qa, ka, q4, k4, qt, kt, qt4, kt4
        # decomposition (cfg3): 5 % salient rows
        sal = synth.salient_rows_from_attention(ROWS, frac=0.05, heads=24, seed=3, device="cuda")
        sal_d = torch.from_numpy(sal).cuda()
        n_sal = sal.size
        F.fb4_quantize(luts, o_main, xs[0], codes=codes[0], meta=metas[0])
        for k in range(1, N_SETS):
            codes[k].copy_(codes[0]); metas[k].copy_(metas[0])
        c2 = torch.empty((n_sal, COLS // 2), dtype=torch.uint8, device="cuda")
        m2 = torch.empty((n_sal, COLS // BLOCK), dtype=torch.int16, device="cuda")

        def decomp_step(i):
            k = i % N_SETS
            F.fb4_decompose(luts, o_main, xs[k], codes[k], metas[k], sal_d, codes2=c2, meta2=m2)
        dbytes = n_sal * COLS * 2 + 2 * (n_sal * COLS // 2 + n_sal * (COLS // BLOCK) * 2)
        add("decompose_5pct_lut_g8", decomp_step, dbytes, n_sal * COLS)

        def fused_step(i):
            k = i % N_SETS
            F.fb4_quantize_decompose(luts, o_main, xs[k], sal_d, codes1=codes[k], meta1=metas[k], codes2=c2, meta2=m2)
        add("quantize_decompose_5pct_one_pass", fused_step,
            abytes + n_sal * COLS // 2 + n_sal * (COLS // BLOCK) * 2 + n_sal * 4, n_el)
        outs = [torch.empty((ROWS, COLS), dtype=torch.bfloat16, device="cuda") for _ in range(N_SETS)]

        def deq_plain_step(i):
            k = i % N_SETS
            F.fb4_dequantize(luts, codes[k], metas[k], out=outs[k])
        add("dequantize_bf16", deq_plain_step, abytes, n_el)

        def deq_step(i):
            k = i % N_SETS
            F.fb4_dequantize(luts, codes[k], metas[k], codes2=c2, meta2=m2, salient_rows=sal_d, out=outs[k])
        add("dequantize_bf16_with_5pct_second_plane", deq_step, abytes + dbytes, n_el)
        els = [torch.empty((ROWS, COLS), dtype=torch.uint8, device="cuda") for _ in range(N_SETS)]
        scs = [torch.empty((ROWS, COLS // 32), dtype=torch.uint8, device="cuda") for _ in range(N_SETS)]

        def repack_step(i):
            k = i % N_SETS
            F.fb4_repack_mxfp8(luts, codes[k], metas[k], elems=els[k], scales=scs[k])
        add("repack_mxfp8", repack_step, n_el // 2 + n_el // 16 + n_el + n_el // 32, n_el)
        # (the exhaustive selector runs last of the cfg2 extras: it heats the chip for whatever follows it)
        add("quantize_sse", quant_step(F.opts(selector=F.SEL_SSE)), abytes, n_el, steps=max(5, args.steps // 10))
        add("quantize_sse_two_stage", quant_step(F.opts(selector=F.SEL_SSE, flags=F.FLAG_TWO_STAGE)), abytes, n_el,
            steps=max(5, args.steps // 10))
        # the headline kernel on a four times larger tensor (65536 x 3072): the fixed cost of a launch (table
        # set-up, pipeline fill and drain) weighs less
        del els, scs, outs
        big = [x0.repeat(4, 1) for _ in range(3)]
        bc = [torch.empty((4 * ROWS, COLS // 2), dtype=torch.uint8, device="cuda") for _ in range(3)]
        bm = [torch.empty((4 * ROWS, COLS // BLOCK), dtype=torch.int16, device="cuda") for _ in range(3)]

        def big_step(i):
            k = i % 3
            F.fb4_quantize(luts, o_main, big[k], codes=bc[k], meta=bm[k])
        add("quantize_lut_g8_65536x3072", big_step, 4 * abytes, 4 * n_el)
        del big, bc, bm
        # cfg1 (1024 x 3072: 8 MB per launch, bound by the launch, not by the memory) ...
        x1 = synth.gaussian_outlier(rows=1024, cols=COLS, seed=1, device="cuda")
        x1s = [x1] + [x1.clone() for _ in range(63)]          # 64 sets = 516 MB: not served from the cache
        c1s = [torch.empty((1024, COLS // 2), dtype=torch.uint8, device="cuda") for _ in range(64)]
        m1s = [torch.empty((1024, COLS // BLOCK), dtype=torch.int16, device="cuda") for _ in range(64)]

        def cfg1_step(i):
            k = i % 64
            F.fb4_quantize(luts, o_main, x1s[k], codes=c1s[k], meta=m1s[k])
        add("cfg1_quantize_lut_g8_1024x3072", cfg1_step, algorithmic_bytes(1024, COLS), 1024 * COLS, steps=128)
        del x1s, c1s, m1s
        # ... and cfg5: the 65536 x 12288 activation (online selector, both planes in one pass with 3276
        # salient rows) and the 12288 x 3072 weight (exhaustive selector)
        R5, C5 = synth.CONFIG_SHAPES["cfg5"]
        x5 = synth.vdit_activation(rows=R5, cols=C5, seed=5, device="cuda", outlier_frac=0.01)
        c5 = torch.empty((R5, C5 // 2), dtype=torch.uint8, device="cuda")
        m5 = torch.empty((R5, C5 // BLOCK), dtype=torch.int16, device="cuda")

        def cfg5_step(i):
            F.fb4_quantize(luts, o_main, x5, codes=c5, meta=m5)
        add("cfg5_quantize_lut_g8_65536x12288", cfg5_step, algorithmic_bytes(R5, C5), R5 * C5, steps=10)

        def cfg5_gelu_step(i):
            F.fb4_gelu_quantize(luts, o_main, x5, 1, codes=c5, meta=m5)
        add("cfg5_gelu_quantize_one_pass", cfg5_gelu_step, algorithmic_bytes(R5, C5), R5 * C5, steps=10)
        sal5 = synth.salient_rows_from_attention(R5, frac=0.05, heads=24, seed=5, device="cuda", window=1024)
        sal5_d = torch.from_numpy(sal5).cuda()
        c52 = torch.empty((sal5.size, C5 // 2), dtype=torch.uint8, device="cuda")
        m52 = torch.empty((sal5.size, C5 // BLOCK), dtype=torch.int16, device="cuda")

        def cfg5_fused_step(i):
            F.fb4_quantize_decompose(luts, o_main, x5, sal5_d, codes1=c5, meta1=m5, codes2=c52, meta2=m52)
        add("cfg5_quantize_decompose_5pct_one_pass", cfg5_fused_step,
            algorithmic_bytes(R5, C5) + sal5.size * (C5 // 2 + (C5 // BLOCK) * 2 + 4), R5 * C5, steps=10)

        def cfg5_decomp_step(i):
            F.fb4_decompose(luts, o_main, x5, c5, m5, sal5_d, codes2=c52, meta2=m52)
        add("cfg5_decompose_5pct_lut_g8", cfg5_decomp_step,
            sal5.size * (C5 * 2 + 2 * (C5 // 2 + (C5 // BLOCK) * 2) + 4), sal5.size * C5, steps=20)
        del x5, c5, m5, c52, m52
        RW, CW = synth.CONFIG_SHAPES["cfg5_weight"]
        w5 = synth.weight_matrix(rows=RW, cols=CW, seed=5, device="cuda")
        w5s = [w5] + [w5.clone() for _ in range(7)]
        cws = [torch.empty((RW, CW // 2), dtype=torch.uint8, device="cuda") for _ in range(8)]
        mws = [torch.empty((RW, CW // BLOCK), dtype=torch.int16, device="cuda") for _ in range(8)]
        o_sse = F.opts(selector=F.SEL_SSE)

        def cfg5_weight_step(i):
            k = i % 8
            F.fb4_quantize(luts, o_sse, w5s[k], codes=cws[k], meta=mws[k])
        add("cfg5_weight_quantize_sse_12288x3072", cfg5_weight_step, algorithmic_bytes(RW, CW), RW * CW, steps=16)
        result["extras"] = extras

    # ---- CPU oracle on the host cores of this machine (a baseline for context, not a target)
    if not args.no_cpu_baseline:
        from oracle import fb4_oracle as O
        xb = synth.bf16_bits(x0)
        nthr = O.max_threads()
        t0 = time.perf_counter()
        cr, mr = O.quantize(DEFAULT_FORMATBOOK, xb, selector=O.SEL_LUT, num_groups=8, nthreads=nthr)
        dt = time.perf_counter() - t0
        same = bool(np.array_equal(cr, codes[0].cpu().numpy()) if args.no_extras else True)
        # one thread, on the first 1024 rows, for scale
        t0 = time.perf_counter()
        O.quantize(DEFAULT_FORMATBOOK, xb[:1024], selector=O.SEL_LUT, num_groups=8, nthreads=1)
        dt1 = time.perf_counter() - t0
        result["cpu_baseline"] = {
            "value": n_el / dt / 1e9, "unit": "G elements/s", "cores": nthr, "kind": "oracle",
            "sample": "the whole 16384x3072 cfg2 tensor, selector lut g=8, %.2f s wall on %d threads" % (dt, nthr),
            "one_thread_value": 1024 * COLS / dt1 / 1e9,
            "one_thread_sample": "its first 1024 rows, %.2f s" % dt1,
        }
        if args.no_extras:
            result["cpu_baseline"]["matches_gpu_codes"] = same

    luts.free()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
