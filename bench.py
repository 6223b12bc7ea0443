#!/usr/bin/env python3
"""Benchmark of the Shamir-share hot path on one MI355X.

A step is one pass of the share arithmetic of the ResNet-152-shaped linear
stack (n=5, t=2, p=2^61-1, f=13, batch 1): for each of the 152 layers
    GEN of the layer input -> conv/dense on shares (int8-limb MFMA) ->
    degree reduction + re-randomisation -> truncation -> REC,
on inputs already resident in HBM (each layer's plaintext input was produced
by an untimed pass that applied ReLU/pooling between layers).  Weight shares
and their limb tiles are prepared once, before timing.

Prints ONE JSON line: throughput in field multiply-accumulates per second over
all parties, the roofline of the dominant kernel (the MFMA GEMM), the bulk
share/reconstruct roofline (2^28 elements, HBM-bound) and the CPU oracle timed
on a bounded sample of the same workload.

--legs selects what runs beside the headline step (default: everything), so
that a profiler run can cover one workload at a time:
  chain   the headline step                        shapes  product kernel per layer shape
  direct  step with the no-message shortcuts       secure  ReLU (and pooling) on shares
  batch8  the same stack at batch 8                p45     passes over the prime 2^45 - 55
  bulk    configs[1], 2^28 elements                conv    configs[2], one conv layer
  stream  reduction / ReLU at 2^24 elements        peaks   measured copy / MFMA ceilings
  cpu     the oracle on the host cores             copycal one 1 GiB device copy (counter scaling)
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

METRIC = "mod-p GEMM field-MAC/s over all parties + ResNet-152 linear-stack latency, n=5"
INT8_PEAK_TOPS = 5000.0      # MI355X dense int8, published
HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
OPS_PER_FIELD_MAC = 128      # 8 x 8 int8 limb products, multiply + add


def event_ms(fn, stream, reps=1):
    import torch
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record(stream)
    for _ in range(reps):
        fn()
    b.record(stream)
    b.synchronize()
    return a.elapsed_time(b) / reps


def bulk_share_reconstruct(log2_count, reps):
    """configs[1]: n=5, t=2, 2^28 uniform field elements: GEN, then REC from
    parties {1,2,3} and from {3,4,5}.  Returns per-kernel ms and GB/s on the
    algorithmic bytes (share: 1 read + n writes; reconstruct: m reads + 1 write)."""
    import torch
    from paper_2406_02629_amd import SSNet
    from ssnet_inputs import P61, uniform_below
    n, t, count = 5, 2, 1 << log2_count
    ss = SSNet(n, t, f=13, seed=2)
    stream = torch.cuda.current_stream()
    secret = torch.from_numpy(uniform_below(count, P61, 2).view("int64")).cuda()
    shares = torch.empty((n, count), dtype=torch.int64, device="cuda")
    rec = torch.empty(count, dtype=torch.int64, device="cuda")
    ss.share(secret, stream_id=0, out=shares)
    ss.reconstruct(shares, [1, 2, 3], out=rec)
    torch.cuda.synchronize()
    ok = bool(torch.equal(rec, secret))
    ss.reconstruct(shares, [3, 4, 5], out=rec)
    ok = ok and bool(torch.equal(rec, secret))
    t_share = event_ms(lambda: ss.share(secret, stream_id=0, out=shares), stream, reps)
    t_r1 = event_ms(lambda: ss.reconstruct(shares, [1, 2, 3], out=rec), stream, reps)
    t_r2 = event_ms(lambda: ss.reconstruct(shares, [3, 4, 5], out=rec), stream, reps)
    b_share, b_rec = (1 + n) * 8 * count, (3 + 1) * 8 * count
    total_ms = t_share + t_r1 + t_r2
    out = {
        "workload": f"bulk share/reconstruct n=5 t=2 2^{log2_count} elements (configs[1])",
        "roundtrip_ok": ok,
        "share": {"ms": t_share, "GB/s": b_share / t_share / 1e6},
        "reconstruct_123": {"ms": t_r1, "GB/s": b_rec / t_r1 / 1e6},
        "reconstruct_345": {"ms": t_r2, "GB/s": b_rec / t_r2 / 1e6},
        "bound": "hbm", "achieved": (b_share + 2 * b_rec) / total_ms / 1e6, "peak": HBM_PEAK_GBS, "unit": "GB/s",
    }
    out["frac"] = out["achieved"] / HBM_PEAK_GBS
    del secret, shares, rec
    torch.cuda.empty_cache()
    return out


def bulk_streaming_steps(log2_count, reps):
    """The other element-wise steps at a size where launch cost does not matter (n=5, t=2): reduction +
    truncation + opening in one launch, and ReLU on shares.  GB/s on the algorithmic bytes (a message is
    written once and read once; random coefficients cost nothing)."""
    import torch
    from paper_2406_02629_amd import SSNet
    from ssnet_inputs import uniform_below
    n, t, count = 5, 2, 1 << log2_count
    k, nr = t + 1, 2 * t + 1
    ss = SSNet(n, t, f=13, seed=4)
    stream = torch.cuda.current_stream()
    c = torch.from_numpy(uniform_below(n * count, 1 << 45, 3).view("int64")).cuda().view(n, count)
    out = torch.empty_like(c)
    rec = torch.empty(count, dtype=torch.int64, device="cuda")
    ids = list(range(1, k + 1))
    ss.degree_reduce_truncate_reconstruct(c, 1, ids, out=out, secret=rec)     # reserves the workspace
    torch.cuda.synchronize()
    t_red = event_ms(lambda: ss.degree_reduce_truncate_reconstruct(c, 1, ids, out=out, secret=rec), stream, reps)
    b_red = (n * (1 + k) + 2 * k * n + n * (k + 1) + 3 * k + 3 * n + k + 1) * 8 * count
    x = torch.from_numpy(uniform_below(n * count, 1 << 30, 5).view("int64")).cuda().view(n, count)
    b, bi = ss.nonlinear_masks(count, stream_id=2)
    ss.relu(x, b, bi, out=out)
    torch.cuda.synchronize()
    t_relu = event_ms(lambda: ss.relu(x, b, bi, out=out), stream, reps)
    b_relu = (3 * nr + nr + 1 + 3 * n) * 8 * count
    m_red = (n + (2 * t + 1) * k + k * n + k + n + n + 1) * 8 * count   # shares in, messages out once, shares + opened value out
    res = {"workload": f"n=5 t=2, 2^{log2_count} elements",
           "degree_reduce+truncate+reconstruct": {"ms": t_red, "GB/s": b_red / t_red / 1e6,
                                                  "bytes_per_element": b_red // count,
                                                  "moved_GB/s": m_red / t_red / 1e6,
                                                  "moved_bytes_per_element": m_red // count},
           "relu": {"ms": t_relu, "GB/s": b_relu / t_relu / 1e6, "bytes_per_element": b_relu // count},
           "bound": "hbm", "peak": HBM_PEAK_GBS, "unit": "GB/s"}
    del c, out, rec, x, b, bi
    torch.cuda.empty_cache()
    return res


def conv_layer_roofline(reps):
    """configs[2]: n=3, t=1, batch 8 x 64x56x56, 3x3 64->64: the modular GEMM on a shape with many tiles
    (M = 25088, K = 576, N = 64 per party), weights packed beforehand; kernel times from HIP events."""
    import torch
    from paper_2406_02629_amd import SSNet
    from ssnet_inputs import P61, uniform_below
    n, B, C, H, Co, k = 3, 8, 64, 56, 64, 3
    ss = SSNet(n, 1, f=13, seed=3)
    x = torch.from_numpy(uniform_below(n * B * C * H * H, P61, 3).view("int64")).cuda().view(n, B, C, H, H)
    w = torch.from_numpy(uniform_below(n * Co * C * k * k, P61, 4).view("int64")).cuda().view(n, Co, C, k, k)
    macs = n * B * H * H * C * k * k * Co
    # (i) input gathered from channel-innermost limb planes (the path the stack uses for k x k layers)
    wt = ss.pack_weights_conv_taps(w)
    planes = ss.split_planes(x)
    y = ss.conv_mod_planes(planes, wt, B, C, H, H, Co, k, k, 1, 1)
    torch.cuda.synchronize()
    ss.profile_begin(kernels=True)
    for _ in range(reps):
        ss.split_planes(x, planes=planes)
        ss.conv_mod_planes(planes, wt, B, C, H, H, Co, k, k, 1, 1, out=y)
    prof = ss.profile_end()
    gemm_ms = prof["gemm_kernel"][0] / reps   # the product kernel itself; class gemm also holds the pass that adds planes up
    achieved = macs * OPS_PER_FIELD_MAC / (gemm_ms * 1e-3) / 1e12
    # (ii) the same layer through a materialised im2col matrix
    wp = ss.pack_weights_conv(w)
    y2 = ss.conv_mod_packed(x, wp, Co, k, k, 1, 1)
    same = bool(torch.equal(y, y2))
    ss.profile_begin(kernels=True)
    for _ in range(reps):
        ss.conv_mod_packed(x, wp, Co, k, k, 1, 1, out=y2)
    prof2 = ss.profile_end()
    return {"workload": "conv 3x3 64->64 on 8x64x56x56, n=3 (configs[2]): M=25088 K=576 N=64 per party",
            "bound": "mfma", "kernel": "gemm_limb_kernel<true> (input gathered from limb planes)", "achieved": achieved,
            "peak": INT8_PEAK_TOPS, "unit": "TOP/s", "frac": achieved / INT8_PEAK_TOPS, "gemm_ms": gemm_ms,
            "split_planes_ms": prof["pack_x"][0] / reps, "field_macs": macs,
            "via_im2col_matrix": {"gemm_ms": prof2["gemm_kernel"][0] / reps, "pack_im2col_ms": prof2["pack_x"][0] / reps,
                                  "same_result": same}}


def cpu_baseline(nlayers):
    """The CPU oracle, as it stands, on the first `nlayers` layers of the same
    stack with uniform random shares as operands: GEN, conv, RED+RERAND,
    truncation, REC per layer.  Returns field-MAC/s over that sample."""
    import numpy as np
    import oracle as orc
    from ssnet_inputs import P61, resnet_chain, uniform_below
    n, t, f = 5, 2, 13
    layers = resnet_chain(152)[:nlayers]
    macs, secs = 0, 0.0
    for l, L in enumerate(layers):
        x = uniform_below(L.cin * L.hin * L.hin, 1 << 20, 10 + l).reshape(1, L.cin, L.hin, L.hin)
        w = uniform_below(n * L.cout * L.K, P61, 50 + l).reshape(n, L.cout, L.cin, L.ksize, L.ksize)
        t0 = time.perf_counter()
        xs = orc.share(x, n, t, P61, 1, l)
        y = orc.conv(xs, w, L.stride, L.pad, P61)
        yr = orc.degree_reduce(y.reshape(n, -1), n, t, P61, 1, l)
        yt = orc.truncate(yr, n, t, f, P61, 1, l)
        orc.reconstruct(yt, [1, 2, 3], P61)
        secs += time.perf_counter() - t0
        macs += n * L.macs
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return {"value": macs / secs, "unit": "field-MAC/s", "cores": threads, "kind": "oracle",
            "sample": f"first {nlayers} of 152 layers, all five steps per layer, {macs / 1e9:.2f} G field-MAC "
                      f"in {secs:.1f} s (OpenMP over output rows / elements)"}


TRAFFIC_SUMMARY = os.path.join("profiles", "resnet152_chain_pmc_traffic.txt")


def measured_traffic_bytes(kernel):
    """HBM bytes per launch of `kernel` (fetch + write, scaled) from the committed summary of the
    rocprofv3 --pmc runs of this benchmark's headline leg; None if the summary is not there."""
    try:
        for line in open(os.path.join(ROOT, TRAFFIC_SUMMARY)):
            parts = line.split()
            if parts and parts[0] == kernel and len(parts) >= 5:
                return float(parts[-1]) * 1024 * 1024
    except OSError:
        pass
    return None


def stats(xs):
    xs = sorted(xs)
    return {"median": xs[len(xs) // 2] if len(xs) % 2 else 0.5 * (xs[len(xs) // 2 - 1] + xs[len(xs) // 2]),
            "min": xs[0], "max": xs[-1], "n": len(xs)}


def timed_steps(step, steps, warmup):
    """EXACTLY `steps` passes of step() bracketed by synchronize -> (wall ms per step, per-step HIP-event ms)"""
    import torch
    stream = torch.cuda.current_stream()
    for _ in range(warmup):
        step()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev[0].record(stream)
    for i in range(steps):
        step()
        ev[i + 1].record(stream)
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3 / steps
    return wall, [ev[i].elapsed_time(ev[i + 1]) for i in range(steps)]


def profiled_passes(ss, step, passes=5, kernels=False):
    """per kernel class: median over `passes` passes of the summed HIP-event time of its launches (ms), and the
    launches per pass.  kernels: the passes also stamp every product kernel's own start and end (class
    gemm_kernel); their bracketed spans are then wider, so the two kinds of figures come from separate passes."""
    per = {}
    for _ in range(passes):
        ss.profile_begin(kernels)
        step()
        for k, v in ss.profile_end().items():
            if v[1]:
                per.setdefault(k, []).append(v)
    return {k: (stats([x[0] for x in v])["median"], int(v[0][1])) for k, v in per.items()}


def measured_peaks():
    """what this GPU reaches on a plain device copy, on the write pattern of GEN (one plane read, five written)
    and on a register-resident int8 MFMA loop: the ceilings the published peaks are to be read against"""
    from paper_2406_02629_amd import binding
    return {"copy_GBps": binding.probe_planes(1 << 30, 1), "gen_pattern_1_read_5_writes_GBps": binding.probe_planes(1 << 28, 5),
            "mfma_int8_TOPs_random_operands": binding.probe_mfma_int8(True),
            "mfma_int8_TOPs_constant_operands": binding.probe_mfma_int8(False),
            "kernels": "ssnet_probe_planes, ssnet_probe_mfma_int8 (csrc/probes.hip)"}


def secure_chain(chain, ss, steps, warmup, macs, out_elems, pool_on_shares=False):
    """The same stack with ReLU evaluated on the shares (SSS-NonLinear, Sec. VI-C): a layer's output
    shares feed the next layer, nothing is opened except at the two pooling points; with pool_on_shares
    those stay on shares too (mask equal inside a pooling kernel, the average's division inside the
    truncation) and only the logits are opened.  Reported beside the headline, not in it."""
    import torch
    chain.secure_prepare(pool_on_shares)
    torch.cuda.synchronize()
    ms, _ = timed_steps(chain.secure_timed, steps, warmup)
    prof = profiled_passes(ss, chain.secure_timed, 3)
    relu_elems = sum(L.cout * L.M for L in chain.layers if L.post == "relu")
    opened = "the logits" if pool_on_shares else "the max-pool, the global average and the logits"
    return {"workload": "same stack, Linear - Truncation - NonLinear per layer on shares; opened only at " + opened,
            "ms_per_step": ms, "field_MAC_per_s": macs / (ms * 1e-3),
            "kernel_ms_per_step": {k: {"ms": round(v[0], 4), "spans": v[1]} for k, v in prof.items()},
            # the ReLU of the plain layers runs inside the layer tail (class degree_reduce); class nonlinear
            # holds the two ReLU + pooling calls
            "relu_elements_per_step": relu_elems}


def p45_chain(layers, steps, warmup, batch=1):
    """The headline step over the paper's own prime p = 2^45 - 55 (Sec. VII-A), on the second library: the same
    shapes, scheme and steps; a field element has six int8 limbs, so a field multiply-add is 36 int8
    multiply-adds instead of 64.  Another field, so another workload: reported beside the headline."""
    import torch
    from paper_2406_02629_amd import P45, SSNet
    from paper_2406_02629_amd.chain import Chain
    ss = SSNet(5, 2, f=13, seed=20240602, p=P45)
    chain = Chain(ss, layers, batch=batch)
    chain.forward_prepare()
    torch.cuda.synchronize()
    ms, _ = timed_steps(chain.forward_timed, steps, warmup)
    prof = profiled_passes(ss, chain.forward_timed, 3)
    macs = chain.total_field_macs()
    ops = macs * 2 * 36
    gemm_ms, gemm_launches = prof["gemm_kernel"] = profiled_passes(ss, chain.forward_timed, 3, kernels=True)["gemm_kernel"]
    return {"workload": f"headline stack over p = 2^45 - 55 (libssnet_p45.so), n=5 t=2 f=13 batch {batch}",
            "ms_per_step": ms, "field_MAC_per_s": macs / (ms * 1e-3),
            "kernel_ms_per_step": {k: {"ms": round(v[0], 4), "spans": v[1]} for k, v in prof.items()},
            "roofline": {"bound": "mfma", "kernel": "gemm_limb_kernel (6 limbs)", "achieved": ops / (gemm_ms * 1e-3) / 1e12,
                         "peak": INT8_PEAK_TOPS, "unit": "TOP/s", "frac": ops / (gemm_ms * 1e-3) / 1e12 / INT8_PEAK_TOPS,
                         "launches": gemm_launches, "int8_ops_per_step": ops}}


def gemm_by_shape(chain, ss, reps=20):
    """The product kernel of every distinct layer shape of the stack on its own: launch time (HIP events inside
    the library), int8 rate, and the two bounds of a launch: MFMA time at the nominal rate, and the time to read
    the operands (weight and activation limb tiles of all parties) once from HBM at 8 TB/s.  For the 7x7 maps
    (49 output pixels) the weight read is within a small factor of the MFMA time."""
    import torch
    seen, rows = {}, []
    for l, L in enumerate(chain.layers):
        seen.setdefault((L.M * chain.batch, L.K, L.N, L.ksize), []).append(l)
    for (M, K, N, ksize), ls in seen.items():
        l = ls[0]
        chain.run_layer(l, chain.x_plain[l], "sgp")
        torch.cuda.synchronize()
        ss.profile_begin(kernels=True)
        for _ in range(reps):
            chain.run_layer(l, chain.x_plain[l], "sgp")
        prof = ss.profile_end()
        us = prof["gemm_kernel"][0] * 1e3 / prof["gemm_kernel"][1]
        ops = ss.n * M * K * N * OPS_PER_FIELD_MAC
        operand_bytes = ss.n * 8 * (N * K + chain.layers[l].hin ** 2 * chain.batch * chain.layers[l].cin
                                    if chain.layers[l].kind == "conv" and ksize > 1 and chain.on_planes[l]
                                    else N * K + M * K)
        rows.append({"M": M, "K": K, "N": N, "kernel": f"{ksize}x{ksize}", "layers": len(ls), "us": round(us, 2),
                     "TOP/s": round(ops / us / 1e6, 1), "frac": round(ops / us / 1e6 / INT8_PEAK_TOPS, 3),
                     "mfma_bound_us": round(ops / INT8_PEAK_TOPS / 1e6, 2),
                     "operand_read_bound_us": round(operand_bytes / 8e12 * 1e6, 2)})
    return rows


def paper_setting_3pc(steps, warmup):
    """The setting of the paper's main table: three parties ((2,3) scheme), its prime 2^45 - 55, batch 1, the whole
    inference on shares (Linear - Truncation - NonLinear per layer, pooling on shares, only the logits opened), for
    the ResNet-50 / 101 / 152 main-path stacks.  Compute
    of all three parties on this one GPU, no network."""
    import torch
    from paper_2406_02629_amd import P45, SSNet
    from paper_2406_02629_amd.chain import Chain
    from ssnet_inputs import resnet_chain
    out = {"workload": "n=3 t=1, p = 2^45 - 55, f=12, batch 1, ReLU and pooling on shares; ms per inference"}
    stacks = [("resnet50", resnet_chain(50)), ("resnet101", resnet_chain(101)), ("resnet152", resnet_chain(152))]
    for name, stack in stacks:
        ss = SSNet(3, 1, f=12, seed=20240602, p=P45)
        chain = Chain(ss, stack)
        chain.secure_prepare(True)
        torch.cuda.synchronize()
        out[f"{name}_ms"] = timed_steps(chain.secure_timed, steps, warmup)[0]
        del chain, ss
        torch.cuda.empty_cache()
    return out


def batch8_chain(chain, ss, layers, steps, warmup, secure=True):
    """The headline step at batch 8 (the paper also reports batched inference): eight images through the same
    prepared weights.  M grows eightfold, so a launch has enough tiles to amortise its fixed cost."""
    import torch
    from paper_2406_02629_amd.chain import Chain
    c8 = Chain(ss, layers, batch=8, weights_of=chain)
    c8.forward_prepare()
    torch.cuda.synchronize()
    ms, _ = timed_steps(c8.forward_timed, steps, warmup)
    prof = profiled_passes(ss, c8.forward_timed, 3)
    macs = c8.total_field_macs()
    prof["gemm_kernel"] = profiled_passes(ss, c8.forward_timed, 3, kernels=True)["gemm_kernel"]
    gemm_ms = prof["gemm_kernel"][0]
    res = {"workload": "same stack and weights, batch 8", "ms_per_step": ms, "field_MAC_per_s": macs / (ms * 1e-3),
           "gemm": {"ms": gemm_ms, "TOP/s": macs * OPS_PER_FIELD_MAC / (gemm_ms * 1e-3) / 1e12,
                    "frac": macs * OPS_PER_FIELD_MAC / (gemm_ms * 1e-3) / 1e12 / INT8_PEAK_TOPS},
           "kernel_ms_per_step": {k: {"ms": round(v[0], 4), "spans": v[1]} for k, v in prof.items()}}
    if secure:
        # the eight images with ReLU and pooling on shares, only the logits opened
        sec = secure_chain(c8, ss, steps, warmup, macs, 0, pool_on_shares=True)
        res["nonlinear_and_pooling_on_shares"] = {"ms_per_step": sec["ms_per_step"], "field_MAC_per_s": sec["field_MAC_per_s"],
                                                   "kernel_ms_per_step": sec["kernel_ms_per_step"]}
    del c8
    torch.cuda.empty_cache()
    return res


LEGS = ("chain", "direct", "secure", "shapes", "batch8", "p45", "bulk", "conv", "stream", "peaks", "cpu", "copycal")


def chain_stream_bytes(chain, ss):
    """Bytes of the two streaming passes of one headline step.  Algorithmic: GEN reads an element and writes n
    shares; reduction + re-randomisation + truncation + opening read the n product shares, exchange every
    message once each way and write the n shares and the opened value.  Moved: what the launches really read
    and write: GEN also leaves the limb tiles / planes for the product kernel; the reduction reads the product
    as the planes its kernel left (one per workgroup that had a part in a tile), writes every message once and
    reads none back (one thread plays every party of its element)."""
    n, k, t = ss.n, ss.k, ss.t
    share_alg = share_moved = red_alg = red_moved = 0
    for l, L in enumerate(chain.layers):
        cin = chain.batch * L.cin * (L.hin * L.hin if L.kind == "conv" else 1)
        cout = chain.batch * L.cout * L.M
        share_alg += (1 + n) * 8 * cin
        share_moved += (1 + 2 * n) * 8 * cin if (chain.pointwise[l] or chain.on_planes[l]) else (1 + n) * 8 * cin
        if L.kind == "conv":
            pb = ss.lib.ssnet_product_bytes_conv(ss._ctx, chain.batch, L.cin, L.hin, L.hin, L.cout, L.ksize, L.ksize,
                                                 L.stride, L.pad)
        else:
            pb = ss.lib.ssnet_product_bytes_linear(ss._ctx, chain.batch, L.cin, L.cout)
        planes = max(1, round(pb / (n * cout * 8)))
        per_elem = n * ((1 + k) + 2 * k + (k + 1)) + (3 * k + 3 * n) + (k + 1)
        red_alg += per_elem * 8 * cout
        # the launch keeps the messages in registers for its own use and writes each once for the receiver
        red_moved += (n * planes + (2 * t + 1) * k + k * n + k + n + n + 1) * 8 * cout
    return {"share": (share_alg, share_moved), "degree_reduce": (red_alg, red_moved)}


def cpu_baselines(nlayers):
    """the oracle on every host core this process may use, and on one (a third of the sample: it is ~cores times
    slower); the thread count is set through the OpenMP runtime the oracle's library already uses"""
    import ctypes
    res = cpu_baseline(nlayers)
    try:
        gomp = ctypes.CDLL("libgomp.so.1")
        gomp.omp_get_max_threads.restype = ctypes.c_int
        had = gomp.omp_get_max_threads()
        gomp.omp_set_num_threads(1)
        one = cpu_baseline(max(nlayers // 8, 4))
        gomp.omp_set_num_threads(had)
        res["cores"] = had
        one["cores"] = 1
        res["single_thread"] = one
    except OSError:
        pass
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--depth", type=int, default=152, help="ResNet depth of the stack (152 is the benchmark)")
    ap.add_argument("--bulk-log2", type=int, default=28)
    ap.add_argument("--legs", default="all", help="comma-separated subset of: " + ", ".join(LEGS) +
                    " (all = everything but copycal)")
    ap.add_argument("--cpu-layers", type=int, default=152)
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU (all parties are a batch dimension on it); "
                 "use --gpus 1")
    legs = set(LEGS) - {"copycal"} if args.legs == "all" else set(x for x in args.legs.split(",") if x)
    if legs - set(LEGS):
        sys.exit("bench.py: unknown leg(s) " + ", ".join(sorted(legs - set(LEGS))))

    import torch
    from paper_2406_02629_amd import SSNet
    from paper_2406_02629_amd.chain import Chain
    from ssnet_inputs import resnet_chain
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")

    n, t, f = 5, 2, 13
    ss = SSNet(n, t, f=f, seed=20240602)
    layers = resnet_chain(args.depth)
    chain = None
    result = {"metric": METRIC, "value": None, "unit": "field-MAC/s", "n_gpus": 1, "data": "synthetic",
              "note": "headline leg not selected: only the legs asked for ran"}
    if legs & {"chain", "direct", "secure", "shapes", "batch8"}:
        chain = Chain(ss, layers)
        chain.forward_prepare()
        torch.cuda.synchronize()
        ms_per_step, per_step = timed_steps(chain.forward_timed, args.steps, args.warmup)
        macs = chain.total_field_macs()

        # live per-class kernel time (HIP events on the library's stream): median over five more passes.  Class
        # gemm_kernel is the product kernels from their own start to their own end (events stamped by the launch
        # itself: what a profiler reports as the kernel's duration); class gemm brackets the same launches with
        # events recorded before and after, which adds the gap between two launches.
        prof = profiled_passes(ss, chain.forward_timed)
        gemm_ms, gemm_launches = profiled_passes(ss, chain.forward_timed, kernels=True)["gemm_kernel"]
        prof["gemm_kernel"] = (gemm_ms, gemm_launches)
        span_ms = prof["gemm"][0]
        achieved = macs * OPS_PER_FIELD_MAC / (gemm_ms * 1e-3) / 1e12
        breakdown = {k: {"ms": round(v[0], 4), "spans": v[1]} for k, v in prof.items()}
        traffic = measured_traffic_bytes("gemm_limb_kernel")
        sb = chain_stream_bytes(chain, ss)
        out_elems = sum(L.cout * L.M for L in chain.layers)
        result = {
            "metric": METRIC, "value": macs / (ms_per_step * 1e-3), "unit": "field-MAC/s", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": "u64 mod 2^61-1 (int8 limbs, int32 MFMA accumulate)",
            "data": "synthetic",
            "config": {"workload": f"resnet{args.depth}-shaped linear stack, n=5 t=2 f=13 batch 1 (configs[4])",
                       "layers": len(chain.layers), "field_macs_per_step": macs,
                       "steps_in_timed_region": "share (+limb split for dense/1x1 layers), conv/dense, "
                                                "degree_reduce+rerand+truncate+reconstruct (one launch)"},
            # ms_per_step is wall time over the K steps; these are the same K steps one by one (HIP events)
            "ms_per_step_events": {k: round(v, 4) if k != "n" else v for k, v in stats(per_step).items()},
            "roofline": {"bound": "mfma", "kernel": "gemm_limb_kernel (+ gemm_skinny_kernel on the 7x7 maps)",
                         "achieved": achieved, "peak": INT8_PEAK_TOPS,
                         "unit": "TOP/s", "frac": achieved / INT8_PEAK_TOPS,
                         "traffic": traffic, "traffic_unit": "bytes per launch (HBM)",
                         "traffic_source": TRAFFIC_SUMMARY if traffic is not None else None,
                         "launches": gemm_launches, "avg_launch_us": gemm_ms * 1e3 / max(gemm_launches, 1),
                         "int8_ops_per_step": macs * OPS_PER_FIELD_MAC,
                         "timing": "median over 5 passes of the summed durations of the 152 product kernels, each from "
                                   "the HIP events its launch stamps with the kernel's own start and end",
                         # the same launches bracketed by events recorded before and after each (launch gap included)
                         "bracketed": {"avg_launch_us": span_ms * 1e3 / max(gemm_launches, 1),
                                       "achieved": macs * OPS_PER_FIELD_MAC / (span_ms * 1e-3) / 1e12,
                                       "frac": macs * OPS_PER_FIELD_MAC / (span_ms * 1e-3) / 1e12 / INT8_PEAK_TOPS}},
            "kernel_ms_per_step": breakdown,
            # algorithmic: the bytes the protocol steps need; moved: with the limb tiles / planes and the product's
            # planes the launches really read and write
            "stream_GBps_in_chain": {
                k: {"ms": round(prof[k][0], 4), "algorithmic_GBps": round(a / (prof[k][0] * 1e-3) / 1e9, 1),
                    "moved_GBps": round(m / (prof[k][0] * 1e-3) / 1e9, 1), "algorithmic_bytes": a, "moved_bytes": m}
                for k, (a, m) in sb.items() if k in prof},
        }
    if "peaks" in legs:
        result["peak_measured"] = measured_peaks()
    if chain is None:
        legs -= {"direct", "secure", "shapes", "batch8"}
    if "direct" in legs:
        # same step with the outputs of reduction + truncation + opening taken without the protocol's messages
        ms_direct, _ = timed_steps(lambda: chain.forward_timed("sgD"), args.steps, args.warmup)
        result["cross_party_single_pass"] = {
            "workload": "headline step with ssnet_reduce_truncate_direct in place of the protocol kernels "
                        "(bit-identical outputs, no messages: a simulation shortcut, not the protocol's work)",
            "ms_per_step": ms_direct, "field_MAC_per_s": macs / (ms_direct * 1e-3)}
    if "secure" in legs:
        result["nonlinear_on_shares"] = secure_chain(chain, ss, args.steps, args.warmup, macs, out_elems)
        result["nonlinear_and_pooling_on_shares"] = secure_chain(chain, ss, args.steps, args.warmup, macs, out_elems,
                                                                 pool_on_shares=True)
        if "direct" in legs:
            ms_sd, _ = timed_steps(lambda: chain.secure_timed(direct=True), args.steps, args.warmup)
            result["nonlinear_and_pooling_on_shares"]["layer_tails_single_pass"] = {
                "workload": "the same, every reduce + truncate + ReLU tail by ssnet_reduce_truncate_relu_direct "
                            "(same shares and limb planes, no messages: a simulation shortcut)",
                "ms_per_step": ms_sd, "field_MAC_per_s": macs / (ms_sd * 1e-3)}
    if "shapes" in legs:
        result["gemm_by_shape"] = gemm_by_shape(chain, ss)
    if "batch8" in legs:
        result["batch8"] = batch8_chain(chain, ss, layers, max(args.steps // 4, 2), 1, secure="secure" in legs)
    if "p45" in legs:
        if "secure" in legs:
            result["paper_setting_3pc_p45"] = paper_setting_3pc(max(args.steps // 2, 2), 2)
        result["paper_prime_p45"] = p45_chain(layers, args.steps, args.warmup)
        if "batch8" in legs:
            result["paper_prime_p45_batch8"] = p45_chain(layers, max(args.steps // 4, 2), 1, batch=8)
    del chain
    torch.cuda.empty_cache()
    if "copycal" in legs:
        src = torch.zeros(1 << 27, dtype=torch.int64, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if "bulk" in legs:
        result["roofline_hbm"] = bulk_share_reconstruct(args.bulk_log2, reps=5)
    if "conv" in legs:
        result["roofline_conv_layer"] = conv_layer_roofline(reps=10)
    if "stream" in legs:
        result["roofline_hbm_other_steps"] = bulk_streaming_steps(24, reps=5)
    if "cpu" in legs:
        result["cpu_baseline"] = cpu_baselines(args.cpu_layers)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
