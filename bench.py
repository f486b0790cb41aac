#!/usr/bin/env python3
"""Benchmark of the CHOCO-SGD iteration (local SGD step + CHOCO-Gossip step) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--all] [--only]

One "step" is one pass of the whole hot path over all n workers: choco_sgd_step followed by
choco_gossip_step (difference, statistic/select, encode, public-copy update, neighbour sums,
mix).  Inputs are synthetic, seeded, generated on the device, and resident in HBM before the
timed region.  Prints ONE JSON line.

The headline workload is the large-model shape (n = 8 ring, d = 28,000,000, top-k 0.1 %),
the largest single-GPU configuration and the one where the HBM roofline is meaningful.  The
same line also carries, in "alternatives", that workload in the other supported formulations
(Algorithm 1 in its printed order; the other form of the mix) and, in "configs", a compact
record of every other benchmark shape (d = 270,000 with n = 8 sign and n = 64 ring / torus x
top-k / random-k; d = 28,000,000 with gsgd) and, in "layer_wise", of the operators applied
layer by layer on the 65 layers of the 0.27 M-parameter model.  --all adds the layer-wise
workloads at the language-model sizes ("other_workloads") and the time of the message encoder
and decoder ("wire"); --only runs the one workload and nothing else (the form the rocprofv3
runs use).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth
# Row stride of the state arrays in floats: rows that start on 256-byte boundaries (ld a multiple
# of 64) keep every 1 KiB tile on whole cache lines; with d = 31.8 M and ld = d rounded to 4 the
# dense passes measured 15 % slower.  The three BASELINE sizes are aligned either way.
LD_ALIGN = int(os.environ.get("CHOCO_BENCH_LD_ALIGN", "64"))

WORKLOADS = {
    # name: shape and hyper-parameters of the synthetic stand-ins for the paper's workloads
    "large_topk": dict(desc="large-model shape: n=8 ring, d=28,000,000 fp32, top-k 0.1% (k=28000), "
                            "gamma=0.01, lr=0.05, gradients ~ N(0,0.01^2)",
                       n=8, d=28_000_000, topo="ring", comp="topk", k=28_000, gamma=0.01, lr=0.05,
                       bias_std=0.0),
    "large_qsgd": dict(desc="large-model shape: n=8 ring, d=28,000,000 fp32, QSGD s=16 (biased), "
                            "gamma=0.01, lr=0.05, gradients ~ N(0,0.01^2)",
                       n=8, d=28_000_000, topo="ring", comp="qsgd", levels=16, gamma=0.01, lr=0.05,
                       bias_std=0.0),
    "dc_sign": dict(desc="datacenter shape: n=8 ring, d=270,000 fp32, scaled sign, gamma=0.4, lr=0.1, "
                         "non-IID gradients",
                    n=8, d=270_000, topo="ring", comp="sign", gamma=0.4, lr=0.1, bias_std=0.001),
    "p2p_ring_topk": dict(desc="peer-to-peer shape: n=64 ring, d=270,000 fp32, top-k 1% (k=2700), "
                               "gamma=0.02, lr=0.1",
                          n=64, d=270_000, topo="ring", comp="topk", k=2700, gamma=0.02, lr=0.1,
                          bias_std=0.001),
    "p2p_torus_topk": dict(desc="peer-to-peer shape: n=64 8x8 torus, d=270,000 fp32, top-k 1%, "
                                "gamma=0.02, lr=0.1",
                           n=64, d=270_000, topo="torus", comp="topk", k=2700, gamma=0.02, lr=0.1,
                           bias_std=0.001),
    "p2p_ring_randk": dict(desc="peer-to-peer shape: n=64 ring, d=270,000 fp32, random-k 1%, "
                                "gamma=0.02, lr=0.1",
                           n=64, d=270_000, topo="ring", comp="randk", k=2700, gamma=0.02, lr=0.1,
                           bias_std=0.001),
    "p2p_torus_randk": dict(desc="peer-to-peer shape: n=64 8x8 torus, d=270,000 fp32, random-k 1%, "
                                 "gamma=0.02, lr=0.1",
                            n=64, d=270_000, topo="torus", comp="randk", k=2700, gamma=0.02, lr=0.1,
                            bias_std=0.001),
    # layer-wise compression (Section 5: the operator is applied to every layer on its own):
    # the 65 layer sizes of the 0.27 M-parameter image model, d = 272,474
    "dc_sign_layers": dict(desc="datacenter shape, per layer: n=8 ring, 65 layers (d=272,474), scaled sign "
                                "per layer, gamma=0.4, lr=0.1",
                           n=8, layers="resnet20", topo="ring", comp="sign", gamma=0.4, lr=0.1, bias_std=0.001),
    "p2p_ring_sign_layers": dict(desc="peer-to-peer shape, per layer: n=64 ring, 65 layers (d=272,474), "
                                      "scaled sign per layer, gamma=0.4, lr=0.1",
                                 n=64, layers="resnet20", topo="ring", comp="sign", gamma=0.4, lr=0.1,
                                 bias_std=0.001),
    "p2p_ring_topk_layers": dict(desc="peer-to-peer shape, per layer: n=64 ring, 65 layers (d=272,474), "
                                      "top-k 1% of every layer (at least 1), gamma=0.02, lr=0.1",
                                 n=64, layers="resnet20", fraction=0.01, topo="ring", comp="topk", gamma=0.02,
                                 lr=0.1, bias_std=0.001),
    "p2p_ring_randk_layers": dict(desc="peer-to-peer shape, per layer: n=64 ring, 65 layers (d=272,474), "
                                       "random-k 1% of every layer (at least 1), gamma=0.02, lr=0.1",
                                  n=64, layers="resnet20", fraction=0.01, topo="ring", comp="randk", gamma=0.02,
                                  lr=0.1, bias_std=0.001),
    # the language model's mix of layer sizes (one 21.6 M-entry embedding, 1.69 M-entry matrices, biases)
    "large_sign_layers": dict(desc="large-model shape, per layer: n=8 ring, 14 layers of a 3-layer LSTM language "
                                   "model (d=31,819,578), scaled sign per layer, gamma=0.01, lr=0.05",
                              n=8, layers="lstm", topo="ring", comp="sign", gamma=0.01, lr=0.05, bias_std=0.0),
    # the same layers, sparsified: the seven long layers take the guessed-threshold select one
    # after the other, the biases the layer kernel
    "large_topk_layers": dict(desc="large-model shape, per layer: n=8 ring, 14 layers of a 3-layer LSTM language "
                                   "model (d=31,819,578), top-k 0.1% of every layer, gamma=0.01, lr=0.05",
                              n=8, layers="lstm", fraction=0.001, topo="ring", comp="topk", gamma=0.01, lr=0.05,
                              bias_std=0.0),
    "large_randk_layers": dict(desc="large-model shape, per layer: n=8 ring, 14 layers of a 3-layer LSTM language "
                                    "model (d=31,819,578), random-k 0.1% of every layer, gamma=0.01, lr=0.05",
                               n=8, layers="lstm", fraction=0.001, topo="ring", comp="randk", gamma=0.01, lr=0.05,
                               bias_std=0.0),
}


def layer_table_of(w):
    """(start, length, k) of a layered workload, or None."""
    if "layers" not in w:
        return None
    from paper_1907_09356_amd import synth
    lengths = {"resnet20": synth.resnet20_like_lengths, "lstm": synth.lstm_like_lengths}[w["layers"]]()
    return synth.layer_table(lengths, fraction=w.get("fraction", 0.01))


for _w in WORKLOADS.values():
    if "layers" in _w:
        _t = layer_table_of(_w)
        _w["d"] = int(_t[0][-1] + _t[1][-1])
        if _w["comp"] in ("topk", "randk"):
            _w["k"] = int(_t[2].sum())

# Algorithmic bytes each kernel must move per (worker, coordinate): every array it needs is
# streamed once (reads + writes, fp32), xhat rows shared across neighbours through LDS.
KERNEL_BYTES_PER_ELEM = {
    "k_sgd": 12,              # read x, g; write x
    "k_sel_compact": 8,       # read x, xhat (top-k); random-k reads nothing
    "k_mix_incremental": 16,  # read x, s, xhat; write x
    "k_dense_stat": 8,        # read x, xhat
    "k_dense_apply_mix": 16,  # read x, xhat; write x, xhat
    "k_tile_mix": 12,         # read x, xhat; write x
    "k_dense_apply": 12,      # read x, xhat; write xhat
    "k_mix_direct_global": 12,
    # first pass of a fused choco_step: also reads g and writes x
    "k_dense_stat_sgd": 16,       # read x, g, xhat; write x
    "k_sel_compact_sgd": 16,      # read x, g, xhat; write x
    "k_tile_mix_sgd": 16,         # read x, g, xhat; write x
    "k_mix_incremental_sgd": 20,  # read x, g, s, xhat; write x
    # layer-wise sign / gsgd: the norm pass over (layer, group) work items
    "k_layer_stat": 8,            # read x, xhat
    "k_layer_stat_sgd": 16,       # read x, g, xhat; write x
}


def profile_traffic(workload, kernel, mix, order, launched):
    """HBM bytes per launch of `kernel` as the committed rocprofv3 counter summary of this
    workload states them (profiles/<workload>_hbm_counters.txt: FETCH_SIZE and WRITE_SIZE per
    dispatch, each scaled by what the counter read for the calibration copy).  The summary
    names the formulation and the kernels of the run it was taken from; if this run's differ,
    the figure would describe other code, and None is returned with the reason."""
    path = os.path.join(ROOT, "profiles", "%s_hbm_counters.txt" % workload)
    rel = os.path.relpath(path, ROOT)
    if not os.path.exists(path):
        return None, "no counter summary %s" % rel
    traffic, kernels, form = {}, None, {}
    for line in open(path):
        parts = line.split()
        if line.startswith("traffic:"):
            kv = dict(p.split("=", 1) for p in parts[1:])
            traffic[kv["kernel"]] = int(kv["bytes"])
        elif line.startswith("kernels:"):
            kernels = set(parts[1:])
        elif line.startswith("formulation:"):
            form = dict(p.split("=", 1) for p in parts[1:])
    if form.get("mix") != mix or form.get("order") != order:
        return None, "%s was taken with mix=%s order=%s, this run is mix=%s order=%s" % (
            rel, form.get("mix"), form.get("order"), mix, order)
    if kernels is None or kernels != set(launched):
        return None, "%s lists kernels %s, this run launched %s" % (
            rel, sorted(kernels or []), sorted(launched))
    if kernel not in traffic:
        return None, "%s has no traffic line for %s" % (rel, kernel)
    return traffic[kernel], rel


def message_bits_per_entry(w):
    """Bits per entry that the encoding pass of a dense operator writes as the message
    (Appendix C: 1 for sign, b = 1 + log2(s) for gsgd with s = 2^(b-1) levels)."""
    if w["comp"] == "sign":
        return 1
    if w["comp"] == "qsgd":
        return 1 + max(1, (w["levels"] - 1).bit_length())
    return 0


def make_topology(w):
    from paper_1907_09356_amd import synth
    if w["topo"] == "ring":
        return synth.ring_csr(w["n"])
    side = int(round(w["n"] ** 0.5))
    return synth.torus_csr(side, side)


def comp_kwargs(w, B):
    comp = {"topk": B.Q_TOPK, "randk": B.Q_RANDK, "sign": B.Q_SIGN, "qsgd": B.Q_QSGD}[w["comp"]]
    kw = dict(compressor=comp)
    if "k" in w:
        kw["k"] = w["k"]
    if "levels" in w:
        kw["levels"] = w["levels"]
    layers = layer_table_of(w)
    if layers is not None:
        kw["layers"] = layers
    return kw


def device_inputs(w, torch, seed=20190709):
    """x0 ~ N(0, 0.05^2) shared by all workers; a pool of two gradient buffers
    g = b_i + eps, eps ~ N(0, 0.01^2), b_i ~ N(0, bias_std^2) fixed per worker."""
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    n, d = w["n"], w["d"]
    ld = (d + LD_ALIGN - 1) // LD_ALIGN * LD_ALIGN
    row = torch.randn(ld, generator=gen, device=dev, dtype=torch.float32) * 0.05
    X = row.repeat(n, 1).contiguous()
    pool = []
    bias = None
    if w["bias_std"] > 0:
        bias = torch.randn((n, ld), generator=gen, device=dev, dtype=torch.float32) * w["bias_std"]
    for _ in range(2):
        g = torch.randn((n, ld), generator=gen, device=dev, dtype=torch.float32) * 0.01
        if bias is not None:
            g += bias
        pool.append(g.contiguous())
    return X, pool


def calibration_copy(torch, nbytes=896_000_000, reps=10):
    """A plain device copy of known size (reads nbytes, writes nbytes), run before the
    timed region so that a `rocprofv3 --pmc FETCH_SIZE` / `WRITE_SIZE` pass over this same
    command line also records what those counters read for a known amount of traffic."""
    a = torch.empty(nbytes // 4, dtype=torch.float32, device="cuda:0").normal_()
    b = torch.empty_like(a)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        b.copy_(a)
    torch.cuda.synchronize()
    el = (time.perf_counter() - t0) / reps
    # the same arrays through a library triad c = a + 2 b (reads 2 x nbytes, writes nbytes): with the
    # copy above, the practical ceiling that the streaming kernels' GB/s can be held against
    c = torch.empty_like(a)
    torch.add(a, b, alpha=2.0, out=c)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        torch.add(a, b, alpha=2.0, out=c)
    torch.cuda.synchronize()
    el3 = (time.perf_counter() - t0) / reps
    # and a library 3-read / 1-write stream e = a + b * c (the access pattern of the mix pass)
    e = torch.empty_like(a)
    torch.addcmul(a, b, c, out=e)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        torch.addcmul(a, b, c, out=e)
    torch.cuda.synchronize()
    el4 = (time.perf_counter() - t0) / reps
    del a, b, c, e
    torch.cuda.empty_cache()
    return dict(bytes_read=nbytes, bytes_written=nbytes, ms=1e3 * el, GBps=2 * nbytes / el / 1e9,
                triad_ms=1e3 * el3, triad_GBps=3 * nbytes / el3 / 1e9,
                stream_3r1w_ms=1e3 * el4, stream_3r1w_GBps=4 * nbytes / el4 / 1e9)


def run_gpu(w, steps, warmup, profile=True, fused=True, mix_form=None, order=None, momentum=False):
    import torch
    from paper_1907_09356_amd import binding as B
    X, pool = device_inputs(w, torch)
    kw = comp_kwargs(w, B)
    if mix_form is not None:
        kw["mix_form"] = mix_form
    if order is not None:
        kw["order"] = order
    ctx = B.Choco(X, w["d"], *make_topology(w), w["gamma"], seed=7, **kw)
    M = torch.zeros_like(X) if momentum else None   # momentum memory of Algorithm 2

    def one_step(t):
        if momentum:
            # Algorithm 2 (momentum 0.9, weight decay 1e-4) + gossip step, fused
            ctx.step_momentum(pool[t & 1], M, w["lr"], 0.9, 1e-4)
        elif fused:
            ctx.step(pool[t & 1], w["lr"])      # choco_step = sgd step + gossip step in one call
        else:
            ctx.sgd_step(pool[t & 1], w["lr"])
            ctx.gossip_step()

    for t in range(warmup):
        one_step(t)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(steps):
        one_step(warmup + t)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    out = dict(ms_per_step=1e3 * elapsed / steps, steps_per_s=steps / elapsed)

    if profile:
        # the same K steps again with every kernel bracketed by HIP events on its stream
        ctx.set_profiling(True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for t in range(steps):
            one_step(warmup + steps + t)
        torch.cuda.synchronize()
        out["ms_per_step_profiled"] = 1e3 * (time.perf_counter() - t0) / steps
        rep = ctx.profile_report()
        ctx.set_profiling(False)
        kernels = {}
        elems = w["n"] * w["d"]
        for name, (count, total_ms) in rep.items():
            avg_ms = total_ms / count
            entry = dict(launches_per_step=count / steps, avg_ms=avg_ms,
                         ms_per_step=total_ms / steps)
            bpe = KERNEL_BYTES_PER_ELEM.get(name)
            if name.startswith("k_layer_compress"):
                # top-k: read x, xhat; random-k reads nothing; a pass that carries the local update
                # also reads g and writes x
                bpe = {"topk": 8, "randk": 0}[w["comp"]]
                if name.endswith("_sgd"):
                    bpe += 8
                bpe = bpe or None
            if (bpe is not None and name.startswith("k_sel_compact") and w["comp"] == "topk"
                    and order == B.ORDER_MIX_THEN_COMPRESS and mix_form != B.MIX_DIRECT):
                bpe += 4 if name.endswith("_sgd") else 8   # the mix rides on this pass: + read s (+ write x)
            if bpe is not None and momentum and name.endswith("_sgd"):
                bpe += 8                                   # + read and write the momentum memory
            if bpe is not None and name in ("k_dense_apply_mix", "k_dense_apply"):
                # + the message itself: one sign bit per entry (sign), b bits per entry (gsgd)
                bpe += message_bits_per_entry(w) / 8.0
            if bpe is not None and not (w["comp"] == "randk" and name == "k_sel_compact"):
                per_launch = bpe * elems
                if "layers" in w and (name.startswith("k_layer_compress") or name.startswith("k_sel_compact")):
                    # layers above 10,240 entries go through k_sel_compact, the others through
                    # k_layer_compress; the launches of each share its part of one pass over the rows
                    lengths = layer_table_of(w)[1]
                    long_part = float(lengths[lengths > 10240].sum()) / float(lengths.sum())
                    per_launch *= long_part if name.startswith("k_sel_compact") else 1.0 - long_part
                    per_launch /= entry["launches_per_step"]
                entry["alg_bytes_per_launch"] = per_launch
                entry["alg_GBps"] = per_launch / (avg_ms * 1e-3) / 1e9
            kernels[name] = entry
        out["kernels"] = kernels
    if w["comp"] in ("topk", "randk") and "layers" not in w:
        sc = ctx.last_scalars()
        out["select"] = dict(fallback_steps=int(sc[:, 4].max()), last_mode=int(sc[:, 3].max()),
                             candidates_per_worker=float(sc[:, 5].mean()), k=w["k"])
    if w["comp"] in ("topk", "randk") and "layers" in w:
        sc = ctx.layer_scalars()
        lengths = layer_table_of(w)[1]
        out["select"] = dict(k=w["k"], layers=int(len(lengths)),
                             bracket_hit_fraction=float(sc[:, :, 3].mean()),
                             bracket_hit_fraction_large_layers=float(sc[:, lengths > 10240, 3].mean()))
    out["mix"] = {B.MIX_INCREMENTAL_S: "incremental", B.MIX_DIRECT: "direct"}[ctx.mix_form()]
    m = ctx.metrics()
    out["consensus_error"] = m["consensus"]
    out["mean_norm"] = m["mean_norm"]
    ctx.close()
    del ctx, X, pool
    torch.cuda.empty_cache()
    return out


def wire_bench(w, reps=20):
    """Time of encoding and decoding the messages of one gossip step (not part of `value`)."""
    import torch
    from paper_1907_09356_amd import binding as B
    X, pool = device_inputs(w, torch)
    kw = comp_kwargs(w, B)
    ctx = B.Choco(X, w["d"], *make_topology(w), w["gamma"], seed=7, **kw)
    if w["comp"] in ("sign", "qsgd"):
        codes = torch.zeros_like(X, dtype=torch.int32)
        ctx.set_capture(codes)
    for t in range(3):
        ctx.step(pool[t & 1], w["lr"])
    msgs = ctx.pack_messages()
    ctx.unpack_messages(msgs)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        msgs = ctx.pack_messages()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(reps):
        ctx.unpack_messages(msgs)
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    out = dict(message_bytes_per_worker=ctx.message_bytes(),
               paper_bits_per_message=B.paper_message_bits(kw["compressor"], w["d"], kw.get("k", 1),
                                                           kw.get("levels", 1)),
               dense_bytes_per_worker=4 * w["d"],
               pack_us=1e6 * (t1 - t0) / reps, unpack_us=1e6 * (t2 - t1) / reps)
    ctx.close()
    return out


def step_bytes_per_elem(w, kernels):
    """Algorithmic bytes of one whole step per (worker, coordinate)."""
    total = 0.0
    for name, e in kernels.items():
        if "alg_bytes_per_launch" in e:
            total += e["alg_bytes_per_launch"] * e["launches_per_step"]
    return total / (w["n"] * w["d"])


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def host_inputs(w, seed=20190709):
    """The workload's inputs in host memory at full size (float32, made row by row): x0 shared
    by all workers, two gradient buffers g = b_i + eps."""
    import numpy as np
    n, d = w["n"], w["d"]
    rng = np.random.default_rng(seed)
    row = rng.standard_normal(d, dtype=np.float32) * np.float32(0.05)
    X0 = np.repeat(row[None, :], n, axis=0)
    bias = None
    if w["bias_std"] > 0:
        bias = rng.standard_normal((n, d), dtype=np.float32) * np.float32(w["bias_std"])
    G = []
    for _ in range(2):
        g = np.empty((n, d), dtype=np.float32)
        for i in range(n):
            g[i] = rng.standard_normal(d, dtype=np.float32) * np.float32(0.01)
        if bias is not None:
            g += bias
        G.append(g)
    return X0, G


def cpu_baseline(w, mix, order, steps=3):
    """The oracle as it stands on the SAME workload at full size: `steps` iterations of
    sgd_step + gossip_step after one warm-up iteration, one thread (the oracle is
    single-threaded).  Second figure: min(n, host cores) threads, each stepping ONE worker's
    row at full d through the same oracle (a one-node graph: that worker's difference,
    statistic / select, encode, public-copy update and mix; the neighbours' terms of the mix
    are left out), which is what one core per simulated worker would give.  The threads
    run in the oracle's compiled code (ctypes releases the interpreter lock)."""
    import threading
    import numpy as np
    from oracle import choco_ref as ref
    n, d = w["n"], w["d"]
    comp = {"topk": ref.TOPK, "randk": ref.RANDK, "sign": ref.SIGN, "qsgd": ref.QSGD}[w["comp"]]
    kw = dict(compressor=comp, mix_form={"incremental": ref.INCREMENTAL_S, "direct": ref.DIRECT}[mix],
              order={"compress_then_mix": ref.COMPRESS_THEN_MIX, "mix_then_compress": ref.MIX_THEN_COMPRESS}[order])
    if "k" in w:
        kw["k"] = w["k"]
    if "levels" in w:
        kw["levels"] = w["levels"]
    layers = layer_table_of(w)
    if layers is not None:
        kw["layers"] = layers
    t0 = time.perf_counter()
    X0, G = host_inputs(w)
    gen_s = time.perf_counter() - t0
    st = ref.RefState(X0, *make_topology(w), gamma=w["gamma"], seed=7, **kw)
    st.sgd_step(G[0], w["lr"])   # warm-up iteration (pages in the state, first touch)
    st.gossip_step()
    t0 = time.perf_counter()
    for t in range(steps):
        st.sgd_step(G[(t + 1) & 1], w["lr"])
        st.gossip_step()
    el = time.perf_counter() - t0
    del st
    # one core per simulated worker
    try:
        avail = len(os.sched_getaffinity(0))
    except AttributeError:
        avail = os.cpu_count() or 1
    cores = max(1, min(n, avail, 16))
    one = (np.array([0, 1], dtype=np.int32), np.array([0], dtype=np.int32), np.array([1.0], dtype=np.float32))
    states = [ref.RefState(X0[i:i + 1], *one, gamma=w["gamma"], seed=7, **kw) for i in range(n)]

    def work(rank, first, count):
        for i in range(rank, n, cores):
            for t in range(first, first + count):
                states[i].sgd_step(G[t & 1][i:i + 1], w["lr"])
                states[i].gossip_step()

    def run_threads(first, count):
        th = [threading.Thread(target=work, args=(r, first, count)) for r in range(cores)]
        for x in th:
            x.start()
        for x in th:
            x.join()

    run_threads(0, 1)             # warm-up
    t0 = time.perf_counter()
    run_threads(1, steps)
    elp = time.perf_counter() - t0
    return dict(value=steps / el, unit="steps/s", cores=1, kind="oracle",
                element_updates_per_s=steps * n * d / el, seconds_per_step=el / steps,
                cpu_model=cpu_model(), host_cores_available=avail,
                sample="the full workload: n=%d, d=%d, %s, mix=%s, order=%s; %d iterations of sgd_step + gossip_step "
                       "after 1 warm-up iteration, %.1f s; inputs generated on the host in %.1f s (not timed)"
                       % (n, d, w["comp"], mix, order, steps, el, gen_s),
                workers_in_parallel=dict(
                    value=steps / elp, unit="steps/s", cores=cores, seconds_per_step=elp / steps,
                    element_updates_per_s=steps * n * d / elp,
                    what="%d threads, each stepping one worker's row at full d through the same oracle "
                         "(one-node graph: the neighbours' terms of the mix are left out); %d iterations after "
                         "1 warm-up" % (cores, steps)))


def compact_record(name, w, r, steps):
    """One line per workload for the "configs" array: time, rate and algorithmic bandwidth."""
    elems = w["n"] * w["d"]
    bpe = step_bytes_per_elem(w, r["kernels"])
    gbps = bpe * elems * r["steps_per_s"] / 1e9
    timed = {k: v for k, v in r["kernels"].items() if "alg_GBps" in v}
    rec = dict(name=name, workload=w["desc"], n=w["n"], d=w["d"], mix=r["mix"], steps=steps,
               ms_per_step=r["ms_per_step"], steps_per_s=r["steps_per_s"],
               element_updates_per_s=r["steps_per_s"] * elems,
               alg_bytes_per_elem=bpe, alg_GBps=gbps, frac_of_hbm_peak=gbps / HBM_PEAK_GBS,
               kernels_us={k: round(1e3 * v["ms_per_step"], 2) for k, v in r["kernels"].items()})
    if timed:
        dom = max(timed, key=lambda k: timed[k]["ms_per_step"])
        rec["dominant_kernel"] = dict(kernel=dom, avg_us=round(1e3 * timed[dom]["avg_ms"], 2),
                                      alg_GBps=round(timed[dom]["alg_GBps"], 1),
                                      frac_of_hbm_peak=round(timed[dom]["alg_GBps"] / HBM_PEAK_GBS, 4))
    if "select" in r:
        rec["select"] = r["select"]
    return rec


CONFIG_WORKLOADS = ["dc_sign", "p2p_ring_topk", "p2p_torus_topk", "p2p_ring_randk", "p2p_torus_randk",
                    "large_qsgd"]
LAYER_WORKLOADS = ["dc_sign_layers", "p2p_ring_sign_layers", "p2p_ring_topk_layers", "p2p_ring_randk_layers"]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="large_topk", choices=sorted(WORKLOADS))
    ap.add_argument("--all", action="store_true",
                    help="also time the layer-wise workloads and the message encoder / decoder")
    ap.add_argument("--only", action="store_true",
                    help="the one workload and nothing else: no alternatives, no other configs, no CPU baseline")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--mix", choices=["auto", "incremental", "direct"], default="auto",
                    help="evaluation of the mix: auto = the library's choice (direct, LDS-tiled, no S array, "
                         "wherever the tile of all rows fits; else incremental neighbour sums)")
    ap.add_argument("--order", choices=["compress_then_mix", "mix_then_compress"],
                    default="compress_then_mix",
                    help="order of the two halves of the gossip step (the second is Algorithm 1 as printed)")
    ap.add_argument("--momentum", action="store_true",
                    help="local update = Algorithm 2 (momentum 0.9, weight decay 1e-4) via choco_step_momentum")
    ap.add_argument("--unfused", action="store_true",
                    help="call choco_sgd_step + choco_gossip_step instead of the fused choco_step")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build runs on ONE GPU (all n workers live in one n x d array); "
                 "--gpus N with N > 1 is not supported")
    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")

    w = WORKLOADS[args.workload]
    copy_ref = calibration_copy(torch)
    from paper_1907_09356_amd import binding as B
    mix_form = {"auto": None, "incremental": B.MIX_INCREMENTAL_S, "direct": B.MIX_DIRECT}[args.mix]
    if w["comp"] in ("sign", "qsgd"):
        mix_form = None   # dense operators always use the direct form
    order = (B.ORDER_MIX_THEN_COMPRESS if args.order == "mix_then_compress"
             else B.ORDER_COMPRESS_THEN_MIX)
    res = run_gpu(w, args.steps, args.warmup, fused=not args.unfused, mix_form=mix_form, order=order,
                  momentum=args.momentum)
    elems = w["n"] * w["d"]
    kernels = res["kernels"]
    timed = {k: v for k, v in kernels.items() if "alg_GBps" in v}
    dominant = max(timed, key=lambda k: timed[k]["ms_per_step"])
    dk = timed[dominant]
    traffic, traffic_source = None, "not a default run (unfused or momentum)"
    if not args.unfused and not args.momentum:
        traffic, traffic_source = profile_traffic(args.workload, dominant, res["mix"], args.order, kernels.keys())
    roofline = dict(bound="hbm", kernel=dominant, achieved=dk["alg_GBps"], peak=HBM_PEAK_GBS,
                    unit="GB/s", frac=dk["alg_GBps"] / HBM_PEAK_GBS,
                    alg_bytes_per_launch=dk["alg_bytes_per_launch"], avg_launch_ms=dk["avg_ms"],
                    traffic=traffic, traffic_source=traffic_source)
    bpe = step_bytes_per_elem(w, kernels)
    line = {
        "metric": "choco_gossip_steps_per_s",
        "value": res["steps_per_s"],
        "unit": "steps/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": w["desc"], "name": args.workload, "n": w["n"], "d": w["d"],
                   "step": ("choco_sgd_step + choco_gossip_step" if args.unfused else
                            "choco_step (= choco_sgd_step + choco_gossip_step, local update fused "
                            "into the first pass)"),
                   "order": args.order, "mix": res["mix"], "mix_requested": args.mix,
                   "local_update": "momentum 0.9, weight decay 1e-4 (Algorithm 2)" if args.momentum else "sgd"},
        "element_updates_per_s": res["steps_per_s"] * elems,
        "step_alg_bytes_per_elem": bpe,
        "step_alg_GBps": bpe * elems * res["steps_per_s"] / 1e9,
        "step_frac_of_hbm_peak": bpe * elems * res["steps_per_s"] / 1e9 / HBM_PEAK_GBS,
        "roofline": roofline,
        "kernels": {k: {kk: (round(vv, 6) if isinstance(vv, float) else vv) for kk, vv in v.items()}
                    for k, v in kernels.items()},
        "ms_per_step_profiled": res["ms_per_step_profiled"],
        "consensus_error": res["consensus_error"],
        "device_copy_reference": copy_ref,
    }
    if "select" in res:
        line["select"] = res["select"]
    if not args.only:
        # the same workload in the other supported formulations (each has its own form of the
        # oracle): the other evaluation of the mix, and Algorithm 1's printed order
        alts = []
        variants = []
        if w["comp"] in ("topk", "randk") and "layers" not in w:
            other = B.MIX_INCREMENTAL_S if res["mix"] == "direct" else B.MIX_DIRECT
            variants.append(dict(order=order, mix_form=other))
            variants.append(dict(order=B.ORDER_MIX_THEN_COMPRESS, mix_form=B.MIX_INCREMENTAL_S))
            variants.append(dict(order=B.ORDER_MIX_THEN_COMPRESS, mix_form=B.MIX_DIRECT))
        elif "layers" not in w:
            variants.append(dict(order=B.ORDER_MIX_THEN_COMPRESS, mix_form=None))
        for kw in variants:
            k = min(args.steps, 50)
            r = run_gpu(w, k, min(args.warmup, 10), fused=not args.unfused, momentum=args.momentum, **kw)
            rec = compact_record(args.workload, w, r, k)
            rec["order"] = ("mix_then_compress" if kw["order"] == B.ORDER_MIX_THEN_COMPRESS
                            else "compress_then_mix")
            del rec["workload"]
            alts.append(rec)
        line["alternatives"] = alts
        # every other benchmark shape, briefly (the library's default formulation)
        confs = []
        for name in CONFIG_WORKLOADS:
            if name == args.workload:
                continue
            ow = WORKLOADS[name]
            # the d = 270 k shapes take 20-100 us per step: 100 steps after 10 warm-up steps whatever
            # --steps says, so that the figure is not the first launches' (their own count is recorded)
            small = ow["n"] * ow["d"] < 100_000_000
            k = 100 if small else min(args.steps, 100)
            r = run_gpu(ow, k, 10 if small else min(args.warmup, 10), fused=not args.unfused, mix_form=None,
                        order=order, momentum=args.momentum)
            confs.append(compact_record(name, ow, r, k))
        line["configs"] = confs
        # the operator applied layer by layer (Section 5 set-up), on the 65 layers of the 0.27 M model
        line["layer_wise"] = []
        for name in LAYER_WORKLOADS:
            ow = WORKLOADS[name]
            r = run_gpu(ow, 100, 10, fused=not args.unfused, mix_form=None, order=order, momentum=args.momentum)
            line["layer_wise"].append(compact_record(name, ow, r, 100))
    if not args.only and not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(w, res["mix"], args.order)
    if args.all and not args.only:
        # encoder / decoder of the messages (Appendix C sizes) for the shapes they cover
        line["wire"] = [dict(name=name, **wire_bench(WORKLOADS[name]))
                        for name in ("dc_sign", "large_qsgd", "p2p_ring_topk", "p2p_ring_randk", "large_topk")]
        others = []
        for name, ow in WORKLOADS.items():
            if name == args.workload or name in CONFIG_WORKLOADS or name in LAYER_WORKLOADS:
                continue
            k = min(args.steps, 100)
            r = run_gpu(ow, k, min(args.warmup, 10), fused=not args.unfused, mix_form=None, order=order,
                        momentum=args.momentum)
            others.append(compact_record(name, ow, r, k))
        line["other_workloads"] = others
    print(json.dumps(line))


if __name__ == "__main__":
    main()
