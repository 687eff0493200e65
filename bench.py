#!/usr/bin/env python3
"""Benchmark of the sparse-sparse MoE expert-FFN path on one MI355X.

A step = one pass of the whole hot path over one batch: route + bucket + SSMM gate/up
(+SiLU*up) + SSMM down (+routing weight) + combine, inputs and encoded weights already
resident in HBM.  Headline workload: the Mixtral-shaped layer (hidden 4096, FFN 14336, 8 experts,
top-2, 2:4 weights) at 4096 tokens; its 16- and 256-token points are reported in "sweep", the
other layer shapes of the benchmark set (tiny, Qwen-MoE-shaped, DeepSeek-MoE-shaped, the 75 %
sparse variant at 4096 and 16 tokens) in "configs", each timed the same way with a roofline
object for its first product and one for its down projection.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 matrix peak


def bytes_per_weight(fmt):
    """Encoded bytes per dense weight element: 2:4 keeps half the values (1 B) plus 2 bits each (1/8 B);
    an (N,M,V) level keeps N/M of that, plus its kernel-ready Sub-Row section ((1,2,V): 2 bits per lane
    and k block = 1/32 B per dense element of the stored half; gathered: one byte per dense row and k block)."""
    N, M, V = fmt
    if N == M:
        return 1.125
    if N == 1 and M == 2:
        return 0.5625 + 1.0 / 32
    return 1.125 * N / M + 1.0 / 32


def algorithmic_bytes(cfg, active_experts):
    """Bytes the method itself must move per layer pass: encoded weights of the experts that
    have tokens (1 B of values + 1/8 B of metadata per dense element for 2:4), each token row
    once per pair, h written and read once, yp written and read once, y written."""
    H, F, P, T = cfg.H, cfg.F, cfg.pairs, cfg.T
    per_w = bytes_per_weight(cfg.fmt)
    weights = 3 * H * F * per_w * active_experts
    acts = P * (2 * H + 4 * F + 4 * H) + 2 * T * H
    return weights, acts


def kernel_bytes(cfg, active_experts):
    """Algorithmic bytes of each kernel of the path (gate/up, down, combine)."""
    H, F, P, T = cfg.H, cfg.F, cfg.pairs, cfg.T
    per_w = bytes_per_weight(cfg.fmt)
    gu = 2 * H * F * per_w * active_experts + P * (2 * H + 2 * F)
    dn = H * F * per_w * active_experts + P * (2 * F + 2 * H)
    cb = P * 2 * H + 2 * T * H
    return gu, dn, cb


def measured_traffic(kernel, tokens=4096, config="mixtral"):
    """HBM-side bytes per launch from the committed counter summary (collected with rocprofv3
    --pmc in separate runs of this script; None if there is no summary for this layer and token count)."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_ssmm_{config}_T{tokens}.txt")
    try:
        for line in open(path):
            if line.startswith(kernel + "_traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def sustained_mfma_share():
    """Share of the published sparse MFMA peak that back-to-back v_smfmac_f32_32x32x32_bf16 on random bf16
    operands sustain on this chip (committed table of `bench.py --mfma-probe`; None if absent)."""
    path = os.path.join(ROOT, "profiles", "sparse_mfma_rate_by_operand_bits.txt")
    try:
        vals = []
        for line in open(path):
            c = [v.strip() for v in line.split("|")]
            if line.startswith("#") or len(c) < 6:
                continue
            if len(c) == 7 and c[0].startswith("v_smfmac_f32_32x32x32") and c[1].startswith("random") and c[2] == "0":
                vals.append(float(c[6]))
            elif len(c) == 6 and c[0].startswith("random") and c[1] == "0":   # table without the instruction column
                vals.append(float(c[5]))
        return sum(vals) / len(vals) if vals else None
    except (OSError, ValueError, IndexError):
        return None


def sustained_hbm_share():
    """Share of the published HBM bandwidth that a kernel which only reads sustains on this chip: the best row
    of the committed table of `bench.py --hbm-probe` (None if absent)."""
    path = os.path.join(ROOT, "profiles", "hbm_stream_rate.txt")
    try:
        vals = [float(line.split("|")[5]) for line in open(path) if not line.startswith("#") and line.count("|") == 5]
        return max(vals) if vals else None
    except (OSError, ValueError, IndexError):
        return None


def run_point(cfg, enc, steps, warmup, B, synth, torch):
    """Time `steps` passes of the hot path at cfg.T tokens.  Returns a dict of measurements."""
    dev = "cuda"
    x = synth.make_tokens(cfg, dev)
    logits = synth.make_logits(cfg, dev)
    route = B.RouteBuffers(cfg.T, cfg.E, cfg.topk, cfg.S, dev)
    y = torch.empty((cfg.T, cfg.H), dtype=torch.bfloat16, device=dev)
    ws = torch.empty((B.ffn_workspace_bytes(cfg.T, cfg.H, cfg.F, cfg.E_total, cfg.slots, cfg.fmt),), dtype=torch.uint8,
                     device=dev)
    # HIP events between the kernels on every fourth step of the timed region: an event record
    # holds the stream up for a few microseconds (measured: 20 us per step with four of them, 7 %
    # of a 16-token step), which a caller of the library does not pay
    stride = 4 if steps >= 8 else 1
    events = B.HipEvents((steps + stride - 1) // stride)

    def step(ev=None):
        B.route_bucket(logits, cfg.topk, cfg.S, cfg.renormalize, route)
        B.expert_ffn(x, cfg.F, cfg.fmt, enc[0], enc[1], enc[2], route, y=y, workspace=ws, events=ev)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(events.steps[i // stride] if i % stride == 0 else None)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    k_ms = events.elapsed_ms()
    events.close()
    t1 = time.perf_counter()                 # outside the timed region: route + bucket alone, back to back
    for _ in range(steps):
        B.route_bucket(logits, cfg.topk, cfg.S, cfg.renormalize, route)
    torch.cuda.synchronize()
    rb_ms = (time.perf_counter() - t1) / steps * 1e3
    off = route.expert_offsets.cpu().numpy()
    active = int(((off[1:] - off[:-1]) > 0).sum())
    flops_dense_equiv = 6.0 * cfg.H * cfg.F * cfg.pairs
    wbytes, abytes = algorithmic_bytes(cfg, active)
    return {"T": cfg.T, "ms_per_step": dt * 1e3, "kernel_ms": {"gate_up": k_ms[0], "down": k_ms[1], "combine": k_ms[2]},
            "route_bucket_ms": rb_ms, "active_experts": active,
            "tflops_dense_equiv": flops_dense_equiv / dt / 1e12, "tokens_per_s": cfg.T / dt,
            "algorithmic_GB": (wbytes + abytes) / 1e9, "hbm_GBs": (wbytes + abytes) / dt / 1e9,
            "hbm_frac": (wbytes + abytes) / dt / 1e9 / HBM_PEAK_GBS,
            "mfma_frac_sparse_peak": flops_dense_equiv / dt / 1e12 / (2 * MFMA_BF16_PEAK_TFLOPS),
            "x": x, "logits": logits, "y": y, "route": route}


def cpu_baseline(cfg, dense, point, torch, synth, max_pairs=512, repeats=16):
    """The fp64 oracle, as it stands, timed on this host: the first expert that has tokens, with the
    first `max_pairs` tokens of its bucket (decode of its three matrices + gate/up + SiLU + down +
    combine), run `repeats` times back to back (about 10-20 s of CPU work in all; the figure is the
    mean).  Returns the cpu_baseline object and the GPU-vs-oracle error on those tokens."""
    import numpy as np
    import threadpoolctl
    from oracle import ssmm_oracle as O

    route = point["route"]
    off = route.expert_offsets.cpu().numpy()
    sel = route.sel.cpu().numpy()
    e = int(np.argmax((off[1:] - off[:-1]) > 0))
    toks = sel[off[e]:off[e + 1]][:max_pairs]
    fmt = O.Format(*cfg.fmt)
    enc = [[O.compress(synth.bits(w[e]), fmt)] for w in dense]          # offline step, not timed
    xb = synth.bits(point["x"][torch.from_numpy(toks).long().cuda()])
    lg = np.zeros((len(toks), 1), dtype=np.float32)
    t0 = time.perf_counter()
    for _ in range(repeats):
        out = O.moe_layer(xb, lg, enc[0], enc[1], enc[2], cfg.H, cfg.F, fmt, 1, 0, True)
    total = time.perf_counter() - t0
    dt = total / repeats
    threads = max([p["num_threads"] for p in threadpoolctl.threadpool_info()] + [1])
    flops = 6.0 * cfg.H * cfg.F * len(toks)
    # the same one-expert sub-layer through the HIP path, as a sanity check beside the timing
    from paper_2503_10725_amd import binding as B
    sub = [B.compress_weights(w[e:e + 1].contiguous(), cfg.fmt, canonical=False, tiled=True)["tiled"] for w in dense]
    r = B.route_bucket(torch.from_numpy(lg).cuda(), 1, 0, True)
    y = B.expert_ffn(synth.from_bits(xb, "cuda"), cfg.F, cfg.fmt, sub[0], sub[1], sub[2], r)
    torch.cuda.synchronize()
    got = O.bf16_bits_to_f64(synth.bits(y))
    rel = float(np.linalg.norm(got - out["y"]) / np.linalg.norm(out["y"]))
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s (dense-equivalent)", "cores": threads, "kind": "oracle",
            "seconds": dt, "seconds_total": total, "tokens_per_s": len(toks) / dt,
            "sample": f"expert {e} of the layer with the first {len(toks)} tokens of its bucket: decode of its 3 "
                      f"weight matrices, gate/up, SiLU*up, down in fp64 (numpy/OpenBLAS), {repeats} passes, mean",
            "gpu_vs_oracle_rel_fro_on_sample": rel}


PROBE_KINDS = [   # (constant of mfma_probe.h, instruction, dense-equivalent FLOPs per instruction, published peak TFLOP/s)
    (0, "v_smfmac_f32_32x32x32_bf16", 2 * 32 * 32 * 32, 5000.0),
    (1, "v_smfmac_f32_16x16x64_bf16", 2 * 16 * 16 * 64, 5000.0),
    (2, "v_mfma_f32_32x32x16_bf16 (dense)", 2 * 32 * 32 * 16, 2500.0),
]


def probe_library():
    """libssmm_probe.so (built by `python -m paper_2503_10725_amd.build`): bench-only, not part of the library."""
    import ctypes
    path = os.path.join(ROOT, "paper_2503_10725_amd", "libssmm_probe.so")
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: run `python -m paper_2503_10725_amd.build` first")
    lib = ctypes.CDLL(path)
    lib.ssmm_probe_operand_bytes.restype = ctypes.c_size_t
    lib.ssmm_probe_mfma.restype = ctypes.c_int
    lib.ssmm_probe_mfma.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                    ctypes.c_void_p, ctypes.POINTER(ctypes.c_float), ctypes.c_void_p]
    lib.ssmm_probe_hbm_read.restype = ctypes.c_int
    lib.ssmm_probe_hbm_read.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_int, ctypes.c_void_p,
                                        ctypes.POINTER(ctypes.c_float), ctypes.c_void_p]
    return lib


def hbm_probe(torch, out_path=None, gib=8):
    """What a kernel that only reads reaches: streaming read of a buffer far larger than the memory-side cache,
    by blocks per compute unit and 16-byte loads in flight per thread.  The roof the small-token SSMM kernels
    (which read their weights once) are read against is the published 8 TB/s; this table says how much of it
    the memory system gives to any kernel.  Returns rows."""
    import ctypes
    lib = probe_library()
    nbytes = gib << 30
    buf = torch.empty((nbytes,), dtype=torch.uint8, device="cuda")
    buf.view(torch.int32).random_()
    sink = torch.zeros((4,), dtype=torch.int32, device="cuda")
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    rows = []
    for rep in range(2):
        for blocks_per_cu in (1, 2, 4, 8):
            for in_flight in (1, 2, 4, 8):
                ms = ctypes.c_float(0.0)
                st = lib.ssmm_probe_hbm_read(ctypes.c_void_p(buf.data_ptr()), nbytes, blocks_per_cu, in_flight,
                                             ctypes.c_void_p(sink.data_ptr()), ctypes.byref(ms), stream)
                if st != 0:
                    raise RuntimeError(f"ssmm_probe_hbm_read: status {st}")
                span = in_flight * 256 * 16
                read = nbytes // span * span
                rows.append({"blocks_per_cu": blocks_per_cu, "loads_in_flight": in_flight, "repeat": rep, "ms": ms.value,
                             "GBs": read / ms.value * 1e-6, "share_of_published_peak": read / ms.value * 1e-6 / HBM_PEAK_GBS})
    if out_path:
        with open(out_path, "w") as f:
            f.write("# streaming read of %d GiB of device memory (memory-side cache: 256 MB), one MI355X\n" % gib)
            f.write("# command: python3 bench.py --hbm-probe <this file>\n")
            f.write("# blocks of 256 threads per compute unit | 16-byte loads in flight per thread | repeat | ms | GB/s | share of the published 8000 GB/s\n")
            for r in rows:
                f.write("%d | %d | %d | %7.3f | %7.1f | %.3f\n" % (r["blocks_per_cu"], r["loads_in_flight"], r["repeat"], r["ms"],
                                                                r["GBs"], r["share_of_published_peak"]))
    return rows


def mfma_probe(torch, out_path=None):
    """What the matrix pipes sustain, back to back, one wavefront per SIMD: the SSMM kernels' instruction
    (v_smfmac_f32_32x32x32_bf16) by operand bits and idle issue slots -- the chip is power-limited under
    matrix load, so the published peak (clock 2.4 GHz) is not what a kernel multiplying real data can
    reach -- and, on the same random operands, the other sparse shape and the dense MFMA a kernel working
    on expanded tiles would issue (the A/B the instruction choice rests on).  Returns rows."""
    import ctypes
    lib = probe_library()
    nbytes = int(lib.ssmm_probe_operand_bytes())
    g = torch.Generator(device="cuda").manual_seed(7)
    n_ab = 8 * 64 * 48
    one = torch.full((n_ab // 2,), 1.0, dtype=torch.bfloat16, device="cuda").view(torch.uint8)
    ix1 = torch.full((8 * 64,), 0x44444444, dtype=torch.int32, device="cuda").view(torch.uint8)
    rnd = torch.randn((n_ab // 2,), generator=g, device="cuda").to(torch.bfloat16).view(torch.uint8)
    ixr = torch.randint(0, 256, (8 * 64 * 4,), generator=g, device="cuda", dtype=torch.uint8)
    operands = {
        "zeros": torch.zeros((nbytes,), dtype=torch.uint8, device="cuda"),
        "ones (bf16 1.0, index bits 0x4 per group)": torch.cat([one, ix1]),
        "random (bf16 N(0,1), random index bits)": torch.cat([rnd, ixr]),
    }
    sink = torch.zeros((1,), dtype=torch.float32, device="cuda")
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)

    def run(buf, iters, idle, kind):
        ms = ctypes.c_float(0.0)
        st = lib.ssmm_probe_mfma(ctypes.c_void_p(buf.data_ptr()), buf.numel(), iters, idle, kind,
                                 ctypes.c_void_p(sink.data_ptr()), ctypes.byref(ms), stream)
        if st != 0:
            raise RuntimeError(f"ssmm_probe_mfma: status {st}")
        return ms.value

    cus = torch.cuda.get_device_properties(0).multi_processor_count
    iters = 12000
    rows = []
    rand = operands["random (bf16 N(0,1), random index bits)"]
    for _ in range(6):                       # ~30 ms of the heaviest load first: a cold chip runs faster for a while
        run(rand, iters, 0, 0)
    for rep in range(2):
        for kind, instr, flops, peak in PROBE_KINDS:
            for name, buf in operands.items():
                for idle in (0, -4, 1, 2, 4):      # -4: no idle slots, four consecutive MFMAs share their B operand
                    if idle and (kind != 0 or not name.startswith("random")):
                        continue
                    ns = run(buf, iters, idle, kind) * 1e6 / (iters * 8)
                    tf = cus * 4 * flops / ns * 1e-3
                    rows.append({"instruction": instr, "operands": name, "s_nop7_per_mfma": idle, "repeat": rep,
                                 "ns_per_mfma": ns, "tflops_dense_equiv": tf, "share_of_published_peak": tf / peak})
    if out_path:
        with open(out_path, "w") as f:
            f.write("# back-to-back matrix instructions, one wavefront per SIMD, %d CUs, one MI355X\n" % cus)
            f.write("# command: python3 bench.py --mfma-probe <this file>\n")
            f.write("# published peaks: sparse bf16 5000 TFLOP/s dense-equivalent (32 cycles per 32x32x32, 16 per 16x16x64, at 2.4 GHz = 13.3 / 6.7 ns); dense bf16 2500 TFLOP/s (32 cycles per 32x32x16)\n")
            f.write("# s_nop 7 = 8 wait states = 32 cycles of the wave's issue; the first one behind an MFMA hides under the MFMA's own 32 cycles\n")
            f.write("# -4 in the third column: no idle slots, four consecutive MFMAs share their B operand (the order of the SSMM kernels)\n")
            f.write("# instruction | operands | s_nop 7 behind each MFMA | repeat | ns per MFMA | dense-equiv TFLOP/s | share of its published peak\n")
            for r in rows:
                f.write("%-34s | %-44s | %2d | %d | %6.2f | %7.1f | %.3f\n" % (
                    r["instruction"], r["operands"], r["s_nop7_per_mfma"], r["repeat"], r["ns_per_mfma"],
                    r["tflops_dense_equiv"], r["share_of_published_peak"]))
    return rows


def subrow_ab(torch, B, synth, steps, warmup, out_path=None, tokens=4096):
    """Sub-Row compute skipping against the masked scheme (sections 4.1 / 4.3 on this hardware), Mixtral
    shape, formats (1,2,V)+2:4 for V = 32 ... 1024: the layer on (a) the default kernels (hand-scheduled,
    every stored operand multiplied once per source row, masked), (b) the same masked scheme on the
    compiler-scheduled kernels with 64-token tiles and (c) the compute-skipping kernels (same family, same
    tiles: one MFMA per stored operand into intermediate sums, merged by source-row bit every V/32 k
    blocks).  (b) and (c) differ in the scheme only.  The knobs that choose (b) and (c) exist in the
    tuning build of the library (libssmm_tune.so), which this leg loads."""
    import dataclasses
    rows = []
    base = synth.CONFIGS["mixtral75"]
    variants = [("masked, hand-scheduled (default)", {}),
                ("masked, compiler-scheduled, 64-token tiles", {"SSMM_PIPE": "1", "SSMM_TILE_SHAPE": "1"}),
                ("compute skipping, compiler-scheduled, 64-token tiles", {"SSMM_SUBROW_SKIP": "1", "SSMM_TILE_SHAPE": "1"})]
    with B.tuning_library():
        for V in (32, 64, 128, 256, 512, 1024):
            cfg = dataclasses.replace(base, fmt=(1, 2, V)).with_tokens(tokens)
            dense = synth.make_weights(cfg, "cuda")
            enc = [B.compress_weights(w, cfg.fmt, canonical=True, tiled=True)["tiled"] for w in dense]
            del dense
            torch.cuda.synchronize()
            for name, env in variants:
                for k, v in env.items():
                    os.environ[k] = v
                try:
                    pt = run_point(cfg, enc, steps, warmup, B, synth, torch)
                finally:
                    for k in env:
                        del os.environ[k]
                rows.append({"V": V, "variant": name, "ms_per_step": pt["ms_per_step"], "gate_up_ms": pt["kernel_ms"]["gate_up"],
                             "down_ms": pt["kernel_ms"]["down"], "tflops_dense_equiv": pt["tflops_dense_equiv"]})
            del enc
            torch.cuda.empty_cache()
    if out_path:
        with open(out_path, "w") as f:
            f.write("# Sub-Row compute skipping against the masked scheme: Mixtral-shaped layer (H 4096, F 14336, 8 experts top-2), %d tokens, (1,2,V)+2:4 weights, one MI355X\n" % tokens)
            f.write("# command: python3 bench.py --steps %d --warmup %d --subrow-ab <this file>\n" % (steps, warmup))
            f.write("# whole step (route .. combine) and its two SSMM kernels from HIP events; mean of %d steps\n" % steps)
            f.write("# V | variant | ms per step | gate/up ms | down ms | dense-equiv TFLOP/s\n")
            for r in rows:
                f.write("%4d | %-52s | %7.4f | %7.4f | %7.4f | %7.1f\n" % (r["V"], r["variant"], r["ms_per_step"], r["gate_up_ms"],
                                                                          r["down_ms"], r["tflops_dense_equiv"]))
    return rows


def ssmm_grid(torch, B, out_path=None):
    """Stand-alone kernel benchmark (the paper's section 6.1): C = A x B[:, SEL] over a grid of
    (m, k, n) in 256..16384 (the paper's own 238 sizes are not listed; powers of four and the
    expert shapes of its Table 2 models are used) and over the share of B's columns that SEL
    picks.  Returns a list of rows; dense-equivalent FLOPs = 2 m k n."""
    rows_out = []
    g = torch.Generator(device="cuda").manual_seed(6)
    shapes = [(m, k, n) for m in (256, 1024, 4096, 16384) for k in (256, 1024, 4096, 16384) for n in (256, 1024, 4096, 16384)
              if m * k <= 16384 * 4096]
    named = [("mixtral gate/up", 14336, 4096, 4096), ("mixtral down", 4096, 14336, 4096),
             ("qwen-moe gate/up", 2560, 3584, 4096), ("qwen-moe down", 3584, 2560, 4096),
             ("deepseek-moe gate/up", 1408, 2048, 4096), ("deepseek-moe down", 2048, 1408, 4096)]
    cases = [("grid", m, k, n, 1.0) for m, k, n in shapes]
    cases += [(name, m, k, n, r) for name, m, k, n in named for r in (1.0, 0.5, 0.25)]
    for name, m, k, n, ratio in cases:
        a = (torch.randn((1, m, k), generator=g, device="cuda") * 0.02).to(torch.bfloat16)
        tiled = B.compress_weights(a, (1, 1, 0), canonical=False, tiled=True)["tiled"]
        del a
        n_b = int(round(n / ratio))
        b = torch.randn((n_b, k), generator=g, device="cuda").to(torch.bfloat16)
        sel = torch.randperm(n_b, generator=g, device="cuda")[:n].sort().values.to(torch.int32)
        c = torch.empty((n, m), dtype=torch.bfloat16, device="cuda")
        ws = torch.empty((int(B.lib().ssmm_matmul_workspace_bytes(m, k, n, B.Format(1, 1, 0))),), dtype=torch.uint8, device="cuda")
        for _ in range(3):
            B.matmul(tiled, m, k, (1, 1, 0), b, sel=sel, c=c, workspace=ws)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        iters = 10
        e0.record()
        for _ in range(iters):
            B.matmul(tiled, m, k, (1, 1, 0), b, sel=sel, c=c, workspace=ws)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / iters
        bytes_alg = m * k * 1.125 + n * k * 2 + n * m * 2
        rows_out.append({"case": name, "m": m, "k": k, "n": n, "selected_share": ratio, "ms": ms,
                         "tflops_dense_equiv": 2.0 * m * k * n / (ms * 1e-3) / 1e12,
                         "GBs_algorithmic": bytes_alg / (ms * 1e-3) / 1e9})
        del tiled, b, sel, c
    if out_path:
        with open(out_path, "w") as f:
            f.write("# stand-alone SSMM  C = A x B[:, SEL]  (ssmm_matmul), 2:4 weights, bf16, one MI355X\n")
            f.write("# command: python3 bench.py --ssmm-grid <this file>\n")
            f.write("# time = mean of 10 back-to-back calls (torch events on the launch stream)\n")
            f.write("# case | m (rows of A) | k | n (selected columns) | share of B selected | ms | dense-equiv TFLOP/s | algorithmic GB/s\n")
            for r in rows_out:
                f.write(f"{r['case']:22s} | {r['m']:6d} | {r['k']:6d} | {r['n']:6d} | {r['selected_share']:.2f} | {r['ms']:8.4f} | "
                        f"{r['tflops_dense_equiv']:8.1f} | {r['GBs_algorithmic']:8.1f}\n")
    return rows_out


def kernel_rooflines(cfg, pt, config_name):
    """Roofline objects of the two SSMM kernels of a measured point: each is read against the roof that
    bounds it at this shape -- the larger of its ideal times at the published peaks (dense bf16 MFMA on
    the FLOPs it executes on the kept half of the weights; HBM on its algorithmic bytes) -- and carries
    the other view beside it."""
    gu_b, dn_b, cb_b = kernel_bytes(cfg, pt["active_experts"])
    out = {}
    for key, ms, nbytes, flops, what in (
            ("roofline", pt["kernel_ms"]["gate_up"], gu_b, 2.0 * cfg.H * cfg.F * cfg.pairs, "gate/up"),
            ("roofline_down", pt["kernel_ms"]["down"], dn_b, 1.0 * cfg.H * cfg.F * cfg.pairs, "down")):
        t = ms * 1e-3
        tf, gbs = flops / t / 1e12, nbytes / t / 1e9
        mfma_bound = flops / (MFMA_BF16_PEAK_TFLOPS * 1e12) >= nbytes / (HBM_PEAK_GBS * 1e9)
        r = {"kernel": f"SSMM {what} (v_smfmac_f32_32x32x32_bf16)", "bound": "mfma" if mfma_bound else "hbm",
             "achieved": tf if mfma_bound else gbs, "peak": MFMA_BF16_PEAK_TFLOPS if mfma_bound else HBM_PEAK_GBS,
             "unit": "TFLOP/s" if mfma_bound else "GB/s",
             "frac": tf / MFMA_BF16_PEAK_TFLOPS if mfma_bound else gbs / HBM_PEAK_GBS,
             "avg_launch_ms": ms, "executed_TFLOPs": tf, "frac_mfma": tf / MFMA_BF16_PEAK_TFLOPS,
             "algorithmic_GBs": gbs, "frac_hbm": gbs / HBM_PEAK_GBS,
             "traffic": measured_traffic("gate_up" if key == "roofline" else "down", cfg.T, config_name)}
        # context, not the peak: what back-to-back sparse MFMAs on random operands / a kernel that only reads sustain here
        share = sustained_mfma_share() if mfma_bound else sustained_hbm_share()
        if share:
            r["sustained"] = {"share_of_peak": share, "frac_of_sustained": r["frac"] / share,
                              "source": "profiles/sparse_mfma_rate_by_operand_bits.txt (bench.py --mfma-probe)" if mfma_bound
                              else "profiles/hbm_stream_rate.txt (bench.py --hbm-probe)"}
        out[key] = r
    out["combine_GBs"] = cb_b / (pt["kernel_ms"]["combine"] * 1e-3) / 1e9
    return out


def public(pt):
    return {k: v for k, v in pt.items() if k not in ("x", "logits", "y", "route")}


WORKLOADS = {
    "tiny": "tiny MoE layer: 128 tokens, hidden 512, FFN 1024, 8 experts top-2, 2:4 weights, N(0,1) router logits",
    "mixtral": "Mixtral-shaped MoE layer: hidden 4096, FFN 14336, 8 experts top-2, 2:4 weights N(0,0.02), {T} tokens, uniform router logits",
    "qwen": "Qwen-MoE-shaped layer: hidden 3584, FFN 2560, 64 experts top-8, 2:4 weights, {T} tokens, per-expert logit bias N(0,1) (skewed loads)",
    "deepseek": "DeepSeek-MoE-shaped layer: hidden 2048, FFN 1408, 64 routed experts top-6 + 2 shared, 2:4 weights, {T} tokens",
    "mixtral75": "Mixtral shape at 75 % weight sparsity: (1,2,8) Sub-Rows by L2 norm stacked on 2:4, {T} tokens, top-2",
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50,
                    help="untimed steps before the timed ones; the first ~25 steps after idle run 5-10 %% slower (clock ramp)")
    ap.add_argument("--tokens", type=int, default=None, help="token count of the headline point (default: the layer's own, 4096 for the headline layer)")
    ap.add_argument("--config", default="mixtral", help="layer of synth.CONFIGS to time as the headline (default: the Mixtral-shaped one)")
    ap.add_argument("--format", default=None, metavar="N,M,V",
                    help="time the chosen layer shape with another weight format, e.g. 4,8,32 (1,1,0 = plain 2:4)")
    ap.add_argument("--pre-expand", action="store_true",
                    help="with a gathered --format: expand the weights once, before the timed region, to plain 2:4 operands "
                         "(ssmm_expand_tiled_weights) and run the layer on those")
    ap.add_argument("--no-sweep", action="store_true", help="skip the 16- and 256-token points of the headline layer")
    ap.add_argument("--no-configs", action="store_true", help="skip the other layer shapes of the benchmark set")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy (reference point for the FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--mfma-probe", metavar="FILE", default=None,
                    help="instead of the layer benchmark: time back-to-back matrix instructions (the kernels' sparse MFMA by "
                         "operand bits, the other sparse shape, the dense MFMA), write the table to FILE")
    ap.add_argument("--hbm-probe", metavar="FILE", default=None,
                    help="instead of the layer benchmark: streaming-read rate of the device memory (8 GiB buffer) by blocks "
                         "per compute unit and loads in flight, write the table to FILE")
    ap.add_argument("--subrow-ab", metavar="FILE", default=None,
                    help="instead of the layer benchmark: Sub-Row compute skipping against the masked scheme for (1,2,V), "
                         "V = 32..1024, on the Mixtral shape; write the table to FILE")
    ap.add_argument("--ssmm-grid", metavar="FILE", default=None,
                    help="instead of the layer benchmark: time the stand-alone SSMM over a shape grid, write the table to FILE")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2503_10725_amd import binding as B
    from paper_2503_10725_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    if args.mfma_probe:
        rows = mfma_probe(torch, args.mfma_probe)
        print(json.dumps({"metric": "sustained matrix-instruction rate by instruction and operand bits", "rows": rows}))
        return
    if args.hbm_probe:
        rows = hbm_probe(torch, args.hbm_probe)
        print(json.dumps({"metric": "streaming-read rate of the device memory, GB/s", "rows": rows}))
        return
    if args.subrow_ab:
        rows = subrow_ab(torch, B, synth, args.steps, args.warmup, args.subrow_ab)
        print(json.dumps({"metric": "Sub-Row compute skipping vs the masked scheme, ms per layer step", "rows": rows}))
        return
    if args.ssmm_grid:
        rows = ssmm_grid(torch, B, args.ssmm_grid)
        print(json.dumps({"metric": "stand-alone SSMM dense-equiv TFLOP/s over a shape grid", "rows": rows}))
        return
    import dataclasses
    base = synth.CONFIGS[args.config]
    if args.format:
        base = dataclasses.replace(base, fmt=tuple(int(v) for v in args.format.split(",")))
    default_run = args.config == "mixtral" and not args.format and not args.pre_expand and args.tokens is None
    if not default_run:
        args.no_sweep = args.no_configs = True
    tokens = args.tokens if args.tokens is not None else base.T

    def encode(cfg):
        dense = synth.make_weights(cfg, "cuda")
        enc = [B.compress_weights(w, cfg.fmt, canonical=False, tiled=True)["tiled"] for w in dense]
        torch.cuda.synchronize()
        return dense, enc

    dense, enc = encode(base)
    run_base = base                       # what the timed calls are given; `base` stays the pruning format (oracle leg)
    if args.pre_expand:
        shapes = [(base.F, base.H), (base.F, base.H), (base.H, base.F)]
        enc = [B.expand_tiled_weights(t, base.E_total, r, k, base.fmt) for t, (r, k) in zip(enc, shapes)]
        run_base = dataclasses.replace(base, fmt=(1, 1, 0))
        torch.cuda.synchronize()

    if args.copy_calibration:
        src = torch.ones((1 << 28,), dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1.0, out=dst)     # elementwise kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    head = run_point(run_base.with_tokens(tokens), enc, args.steps, args.warmup, B, synth, torch)
    cfg = base.with_tokens(tokens)
    rl = kernel_rooflines(cfg, head, args.config if not args.format else "-")
    roofline = rl["roofline"]
    roofline["flops"] = "executed on the kept half of the weights (dense-equivalent = 2x)"
    roofline["traffic_unit"] = "bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, copy-calibrated; profiles/)"
    roofline["combine_GBs"] = rl["combine_GBs"]

    sweep = []
    if not args.no_sweep:
        for T in (16, 256):
            pt = run_point(base.with_tokens(T), enc, args.steps, args.warmup, B, synth, torch)
            row = public(pt)
            row.update(kernel_rooflines(base.with_tokens(T), pt, args.config))
            sweep.append(row)

    cpu = None
    if not args.no_cpu:
        cpu = cpu_baseline(cfg, dense, head, torch, synth)
    del dense

    configs = []
    if not args.no_configs:
        del enc
        torch.cuda.empty_cache()
        for name, T in (("tiny", None), ("qwen", None), ("qwen", 64), ("deepseek", None), ("deepseek", 64),
                        ("mixtral75", None), ("mixtral75", 16)):
            c0 = synth.CONFIGS[name]
            if not configs or configs[-1]["config"] != name:
                d_, e_ = encode(c0)
                del d_
            c = c0.with_tokens(T if T is not None else c0.T)
            pt = run_point(c, e_, args.steps, args.warmup, B, synth, torch)
            row = {"config": name, "workload": WORKLOADS[name].format(T=c.T), "hidden": c.H, "ffn": c.F, "experts": c.E,
                   "shared_experts": c.S, "topk": c.topk, "format": list(c.fmt)}
            row.update(public(pt))
            row.update(kernel_rooflines(c, pt, name))
            configs.append(row)
            torch.cuda.empty_cache()

    out = {
        "metric": "dense-equiv TFLOP/s per MoE layer (route+bucket+SSMM gate/up+SiLU+SSMM down+combine)",
        "value": head["tflops_dense_equiv"], "unit": "TFLOP/s (dense-equivalent)", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": WORKLOADS[args.config].format(T=tokens), "tokens": tokens,
                   "hidden": cfg.H, "ffn": cfg.F, "experts": cfg.E, "topk": cfg.topk, "format": list(cfg.fmt),
                   "weights_resident_as": "plain 2:4 operands, expanded once from the pruning format" if args.pre_expand
                   else "the pruning format"},
        "tokens_per_s": head["tokens_per_s"], "kernel_ms": head["kernel_ms"],
        "route_bucket_ms": head["route_bucket_ms"],
        "mfma_frac_sparse_peak": head["mfma_frac_sparse_peak"],
        "mfma_frac_dense_peak": head["tflops_dense_equiv"] / MFMA_BF16_PEAK_TFLOPS,
        "hbm_GBs": head["hbm_GBs"], "hbm_frac": head["hbm_frac"],
        "roofline": roofline, "roofline_down": rl["roofline_down"], "cpu_baseline": cpu, "sweep": sweep, "configs": configs,
        "paper_context": "paper reports only speedups on an RTX 4070 Super (up to 1.99x kernel vs VENOM, "
                         "1.58x model-level); no absolute number for this metric",
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
