#!/usr/bin/env python3
"""Benchmark of the compressed-MoE hot path on one MI355X.

A step is one pass of the whole path -- dispatch, first fused decode+product
(+ReLU, bf16 hidden), second fused decode+product -- over one batch of routed
tokens of a synthetic SwitchTransformer-shaped layer.  Weights, activations and
routing are resident in HBM before the timed region starts.

Prints one JSON line: compressed-weight GB/s (headline), ms per layer, the
roofline of the dominant kernel, the same layer on uncompressed bf16 weights,
and the CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E bandwidth


def log(msg):
    print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


def build_layer(w, dd, gpu, workers, interchange_order=False, minmax=False, lanes_for_tokens=0, copies=1):
    """Generate and encode every expert (host threads), upload `copies` separate copies of the layer (a
    list; more than one for a cold-cache measurement of a layer that would otherwise stay in the
    last-level cache).  minmax: rows on the asymmetric grid (a bf16 (w_min, w_max) pair per row in place
    of the binary16 scale)."""
    import paper_2310_16795_amd as q
    from paper_2310_16795_amd import device as dev

    layers = [dev.DeviceLayer(w.n_experts, w.d_model, w.d_ff, gpu, minmax=minmax) for _ in range(copies)]
    q.qmoe_set_tuning("host_threads", 1)  # parallelism is across experts here

    def one(e):
        out = []
        for which, tern, scale in (("wi", w.wi_ternary(e), w.wi_minmax(e) if minmax else w.wi_scale(e)),
                                   ("wo", w.wo_ternary(e), w.wo_minmax(e) if minmax else w.wo_scale(e))):
            codes, row_off = q.qmoe_encode_host(dd.handle, tern)
            out.append((which, codes, row_off, scale))
        return e, out

    t0 = time.time()
    done = 0
    with ThreadPoolExecutor(max_workers=workers) as pool:
        for e, parts in pool.map(one, range(w.n_experts)):
            for which, codes, row_off, scale in parts:
                for layer in layers:
                    layer.set_expert(e, which, codes, row_off, scale)
            done += 1
            if done % 256 == 0:
                log(f"encoded {done}/{w.n_experts} experts ({time.time() - t0:.0f} s)")
    q.qmoe_set_tuning("host_threads", 0)
    for layer in layers:
        layer.finalize(device_order_of=None if interchange_order else dd, lanes_for_tokens=lanes_for_tokens)
    return layers


def dense_bf16_experts(layer, dd, active, gpu, stats=None):
    """Uncompressed bf16 copies (scale folded in) of the experts that receive tokens, made by
    the library's decompression kernel, one launch per projection; `stats` receives its rate."""
    import torch
    import paper_2310_16795_amd as q

    ptrs, keep, out = {}, [], {}
    for which in ("wi", "wo"):
        rows = layer.d_ff if which == "wi" else layer.d_model
        cols = layer.d_model if which == "wi" else layer.d_ff
        p = np.zeros(layer.n_experts, dtype=np.int64)
        for e in active:
            dense = torch.empty((rows, cols), dtype=torch.bfloat16, device=gpu)
            keep.append(dense)
            p[e] = dense.data_ptr()
        ptrs[which] = torch.from_numpy(p).to(gpu)
        out[which] = (rows, cols)
    def run():
        for which in ("wi", "wo"):
            q.qmoe_decompress(dd.handle, layer.desc_dev[which], layer.format, layer.n_experts, out[which][0],
                              out[which][1], 1, ptrs[which])
    ms, _ = time_steps(run, 3, 1)
    if stats is not None:
        written = 2 * len(active) * 2 * layer.d_model * layer.d_ff
        stats.update({"experts": len(active), "ms": ms, "bf16_bytes_written": written,
                      "GBps_written": written / (ms * 1e-3) / 1e9,
                      "compressed_GBps_read": layer_bytes_of(layer, active) / (ms * 1e-3) / 1e9,
                      "kind": "qmoe_decompress to bf16, both projections of every expert with tokens, two launches"})
    return ptrs["wi"], ptrs["wo"], keep


def single_matvec(w, dd, gpu, expert, minmax=False):
    """The paper's per-matrix benchmark: one compressed expert matrix (rows back to back, device
    numbering) times one token (`qmoe_decode_matvec`) next to torch.matmul on the same matrix in bf16,
    back-to-back launches, microseconds per call."""
    import torch
    import paper_2310_16795_amd as q
    from paper_2310_16795_amd import device as dev

    out = {}
    for which in ("wi", "wo"):
        tern = w.wi_ternary(expert) if which == "wi" else w.wo_ternary(expert)
        rows, cols = tern.shape
        codes, row_off = q.qmoe_encode_host(dd.handle, tern)
        scale = None if minmax else (w.wi_scale(expert) if which == "wi" else w.wo_scale(expert))
        pairs = (w.wi_minmax(expert) if which == "wi" else w.wo_minmax(expert)) if minmax else None
        M = dev.DeviceMatrix(codes, row_off, scale, rows, cols, device=gpu, device_order_of=dd, minmax_bf16=pairs)
        x = torch.randn(1, cols, device=gpu).to(torch.bfloat16)
        y = torch.empty(1, rows, dtype=torch.float32, device=gpu)
        dense = torch.empty((rows, cols), dtype=torch.bfloat16, device=gpu)
        desc_dev = torch.from_numpy(np.frombuffer(bytes(M.desc), dtype=np.uint8).copy()).to(gpu)
        fmt = q.FORMAT_DEVICE_ORDER | (q.FORMAT_GRID_MINMAX if minmax else 0)
        q.qmoe_decompress(dd.handle, desc_dev, fmt, 1, rows, cols, 1,
                          torch.tensor([dense.data_ptr()], dtype=torch.int64, device=gpu))
        t_c, _ = time_steps(lambda: q.qmoe_decode_matvec(dd.handle, M.desc, x.view(torch.int16), y), 200, 20)
        t_b, _ = time_steps(lambda: torch.matmul(x, dense.T), 200, 20)
        ref = torch.matmul(x.float(), dense.float().T)
        out[which] = {"rows": rows, "cols": cols, "compressed_us": t_c * 1e3, "bf16_torch_matmul_us": t_b * 1e3,
                      "ratio": t_c / t_b, "max_abs_diff_vs_dense": float((y - ref).abs().max())}
    return out


def layer_bytes_of(layer, experts):
    """Bytes of the experts' matrices as the device holds them: codewords (in the lane-interleaved layout the
    padding counts), per row a 4-byte offset and the 2-byte scale (4-byte pair on the asymmetric grid), and in
    the lane-interleaved layout a 4-byte offset per group of 64 lanes."""
    return int(sum(2 * (layer.n_codes["wi"][e] + layer.n_codes["wo"][e]) + layer.matrix_meta["wi"] + layer.matrix_meta["wo"]
                   for e in experts))


def time_steps(fn, steps, warmup, spread=None):
    """Mean ms per step over exactly `steps` steps (HIP events on the current stream around
    the whole run, device idle before and after) and the wall-clock figure; with `spread`
    (a dict) also the median, 10th and 90th percentile of the single steps."""
    import torch

    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(steps):
        fn()
        marks[i + 1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    if spread is not None:
        each = np.array([marks[i].elapsed_time(marks[i + 1]) for i in range(steps)])
        spread.update({"median": float(np.median(each)), "p10": float(np.percentile(each, 10)),
                       "p90": float(np.percentile(each, 90))})
    return marks[0].elapsed_time(marks[steps]) / steps, wall / steps * 1e3


PHASES = (("dispatch", 1), ("first_product_mfma", 8), ("first_product_scalar", 2),
          ("second_product_mfma", 16), ("second_product_scalar", 4))


def time_phases(fn, steps):
    """Per-kernel durations: the kernels of a step enqueued one by one, in the order a
    step runs them, with HIP events between them on the stream they run on."""
    import torch
    import paper_2310_16795_amd as q

    n = len(PHASES)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(n + 1)] for _ in range(steps)]
    for s in range(steps):
        ev[s][0].record()
        for i, (_, mask) in enumerate(PHASES):
            q.qmoe_hook_set("phases", mask)
            fn()
            ev[s][i + 1].record()
    q.qmoe_hook_set("phases", 0)
    torch.cuda.synchronize()
    return {name: float(np.mean([ev[s][i].elapsed_time(ev[s][i + 1]) for s in range(steps)]))
            for i, (name, _) in enumerate(PHASES)}


def cpu_baseline(w, idx, x_bits, active, budget_s=7.0, minmax=False):
    """The oracle, as it stands, on a bounded sample of the workload (expert after expert: decode both
    matrices, push the expert's tokens through in fp64), timed three ways: one thread; every host core
    this job may use, one expert per thread at a time (the C routines release the interpreter lock);
    and, on one thread, the products alone on matrices that are already decoded (the decode-free dense
    int8 leg).  Rates are bytes of the sample's compressed matrices (2 per codeword + row metadata) per
    second, so that they compare with the GPU line."""
    import oracle

    od = oracle.Dictionary()
    cores = max(1, min(16, os.cpu_count() or 1))  # a job's share of the machine's cores

    def prepare(e):
        wi, wo = w.wi_ternary(e), w.wo_ternary(e)
        ci, ri = oracle.encode(od, wi)
        co, ro = oracle.encode(od, wo)
        meta = (8 if minmax else 6) * (wi.shape[0] + wo.shape[0])
        return {"e": e, "wi": (ci, ri, wi.shape), "wo": (co, ro, wo.shape), "bytes": 2 * (ci.size + co.size) + meta,
                "scales": (None, None) if minmax else (w.wi_scale(e), w.wo_scale(e)),
                "pairs": (w.wi_minmax(e), w.wo_minmax(e)) if minmax else (None, None),
                "toks": np.nonzero(idx == e)[0]}

    def decode(p):
        return (oracle.decode(od.words, p["wi"][0], p["wi"][1], *p["wi"][2]),
                oracle.decode(od.words, p["wo"][0], p["wo"][1], *p["wo"][2]))

    def products(p, di, do):
        for t in p["toks"]:
            oracle.ffn_token(di, p["scales"][0], do, p["scales"][1], x_bits[t], 1.0, p["pairs"][0], p["pairs"][1])

    # one thread, and the decode-free leg on the same experts
    t_one = t_dense = 0.0
    sample = []
    for e in active:
        p = prepare(e)
        t0 = time.perf_counter()
        di, do = decode(p)
        t1 = time.perf_counter()
        products(p, di, do)
        t2 = time.perf_counter()
        t_one += t2 - t0
        t_dense += t2 - t1
        sample.append(p)
        if t_one > budget_s:
            break
    b_one = sum(p["bytes"] for p in sample)
    n_tok = int(sum(p["toks"].size for p in sample))
    # every core: about the same wall time, `cores` times the experts
    more = [e for e in active if e not in {p["e"] for p in sample}][: len(sample) * (cores - 1)]
    with ThreadPoolExecutor(max_workers=cores) as pool:
        batch = sample + list(pool.map(prepare, more))
        t0 = time.perf_counter()
        list(pool.map(lambda p: products(p, *decode(p)), batch))
        t_all = time.perf_counter() - t0
    b_all = sum(p["bytes"] for p in batch)
    return {"value": b_all / t_all / 1e9, "unit": "GB/s", "cores": cores, "kind": "oracle",
            "sample": f"{len(batch)} active experts of the workload with their {int(sum(p['toks'].size for p in batch))} "
                      f"tokens (decode both matrices + fp64 products), one expert per thread, {t_all:.1f} s",
            "one_thread": {"value": b_one / t_one / 1e9, "unit": "GB/s", "cores": 1,
                           "sample": f"first {len(sample)} active experts, {n_tok} tokens, {t_one:.1f} s"},
            "decode_free_dense_int8_one_thread": {
                "value": b_one / max(t_dense, 1e-9) / 1e9, "unit": "GB/s (bytes of the compressed form; the matrices are "
                "already decoded int8, only the fp64 products are timed)", "cores": 1,
                "sample": f"the same {len(sample)} experts, {t_dense:.1f} s"}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c2048")
    ap.add_argument("--no-bf16", action="store_true", help="skip the uncompressed comparator")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--tune", action="append", default=[], help="key=value for qmoe_set_tuning")
    ap.add_argument("--dict-entries", type=int, default=65536,
                    help="dictionary size (the paper's is 65536; smaller tables trade bits per parameter for LDS)")
    ap.add_argument("--dict-max-pairs", type=int, default=14, help="longest dictionary entry in pairs (the paper's is 14)")
    ap.add_argument("--interchange-order", action="store_true",
                    help="leave the codeword streams as encoded instead of renumbering them at load time")
    ap.add_argument("--copies", type=int, default=0,
                    help="resident copies of the layer that the timed steps rotate through, so that every step reads its "
                         "weights from HBM; 0 = as many as make the rotation at least four times the last-level cache "
                         "plus L2 (one for the c2048 workloads, whose single step already is)")
    ap.add_argument("--layout", choices=("lanes", "rows"), default="lanes",
                    help="codeword streams re-packed at load time into the lane-interleaved layout (a wavefront's 64 loads "
                         "are consecutive; its padding counts as compressed bytes), or rows back to back as encoded")
    ap.add_argument("--grid", choices=("scale", "minmax"), default="scale",
                    help="per-row grid: {-s,0,+s} with one binary16 scale (the headline format) or the paper's "
                         "{w_min,0,w_max} with a bf16 pair")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (--gpus 1); no multi-GPU path exists", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2310_16795_amd as q
    from paper_2310_16795_amd import device as dev
    from paper_2310_16795_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no fallback", file=sys.stderr)
        sys.exit(2)
    gpu = "cuda:0"
    w = synth.WORKLOADS[args.workload]
    for kv in args.tune:
        k, v = kv.split("=")
        q.qmoe_set_tuning(k, int(v))

    idx, x_bits = w.expert_idx(), w.tokens()
    T = idx.size
    counts = np.bincount(idx, minlength=w.n_experts)
    active = np.nonzero(counts)[0].tolist()
    log(f"workload {w.name}: {w.n_experts} experts {w.d_model}x{w.d_ff}, {T} tokens, {len(active)} experts with tokens, "
        f"max {counts.max()} tokens on one expert")

    custom_dict = (args.dict_entries, args.dict_max_pairs) != (65536, 14)
    dd = dev.DeviceDict(q.qmoe_dict_create(0.885, args.dict_max_pairs, args.dict_entries) if custom_dict else None,
                        device=gpu)
    workers = min(16, os.cpu_count() or 1)
    t0 = time.time()
    minmax = args.grid == "minmax"
    lanes_layout = args.layout == "lanes" and not args.interchange_order
    # cold protocol: a step must not find its weights in the 256 MB last-level cache or the 8 x 4 MB of L2
    est_touched = 2 * 2 * w.d_model * w.d_ff * len(active) * 0.09  # ~0.71 bits per weight
    copies = args.copies if args.copies > 0 else int(min(32, max(1, np.ceil(4 * 288e6 / est_touched))))
    layers = build_layer(w, dd, gpu, workers, args.interchange_order, minmax, lanes_for_tokens=T if lanes_layout else 0,
                         copies=copies)
    layer = layers[0]
    log(f"layer resident: {layer.compressed_bytes / 1e9:.3f} GB compressed x {copies} copies, built in {time.time() - t0:.0f} s")

    x = torch.from_numpy(x_bits.view(np.int16).copy()).to(gpu)
    d_idx = torch.from_numpy(idx).to(gpu)
    y = torch.empty((T, w.d_model), dtype=torch.float32, device=gpu)
    ws = layer.workspace(T)

    turn = [0]

    def step():
        layers[turn[0] % copies].forward(dd, x, d_idx, y, ws)
        turn[0] += 1

    def step_warm():
        layer.forward(dd, x, d_idx, y, ws)

    spread = {}
    ms, wall_ms = time_steps(step, args.steps, args.warmup, spread)
    warm_ms = ms if copies == 1 else time_steps(step_warm, args.steps, args.warmup)[0]
    kernel_ms = time_phases(step, min(args.steps, 30))

    # which experts went to the matrix-core kernels (tiles of up to 64 tokens), which to the scalar ones
    torch.cuda.synchronize()
    wsout = dev.read_workspace(ws, w.n_experts, w.d_model, w.d_ff, T)
    crowded = sorted({int(e) for e, _, _, _ in wsout["items_mm"][: wsout["counters"][7]]})
    few = [e for e in active if e not in set(crowded)]

    # algorithmic bytes: what the method itself has to move once per step -- every active
    # expert's compressed matrix (codewords + 6 bytes of row metadata) once, activations in, results out
    n_params = 2 * w.d_model * w.d_ff
    def mat_bytes(which, rows, experts):
        return int(sum(2 * layer.n_codes[which][e] + layer.matrix_meta[which] for e in experts))
    weight_bytes = mat_bytes("wi", w.d_ff, active) + mat_bytes("wo", w.d_model, active)
    n_codewords = int(sum(layer.n_codes["wi"][e] + layer.n_codes["wo"][e] for e in active))
    def kernel_bytes(which, experts):
        toks = int(sum(counts[e] for e in experts))
        if which == "wi":
            return mat_bytes("wi", w.d_ff, experts) + toks * w.d_model * 2 + toks * w.d_ff * 2
        return mat_bytes("wo", w.d_model, experts) + toks * w.d_ff * 2 + toks * w.d_model * 4
    dict_mode = "0|1" if args.interchange_order else "3"  # template argument: where the table is read from
    g = 1 if minmax else 0                                # template argument: the grid
    kernels = {
        "first_product_scalar": (f"k_product<{dict_mode}, 1, {g}> (first product, experts with few tokens)", kernel_bytes("wi", few)),
        "second_product_scalar": (f"k_product<{dict_mode}, 0, {g}> (second product, experts with few tokens)", kernel_bytes("wo", few)),
        "first_product_mfma": (f"k_product_mm<1, {g}> (first product, crowded experts)", kernel_bytes("wi", crowded)),
        "second_product_mfma": (f"k_product_mm<0, {g}> (second product, crowded experts)", kernel_bytes("wo", crowded)),
    }
    dom_key = max(kernels, key=lambda k: kernel_ms[k])
    dom = (kernels[dom_key][0], kernel_ms[dom_key], kernels[dom_key][1])
    achieved = dom[2] / (dom[1] * 1e-3) / 1e9

    # plain copy kernel: what pure streaming reaches here
    src = torch.empty(1 << 30, dtype=torch.uint8, device=gpu)
    dst = torch.empty_like(src)
    copy_ms, _ = time_steps(lambda: q.qmoe_stream_copy(dst, src), 10, 3)
    copy_gbps = 2 * src.numel() / (copy_ms * 1e-3) / 1e9
    del src, dst

    # HBM bytes per launch of the dominant kernel: not measured by this run (counters need the profiler) but
    # read from the committed rocprofv3 --pmc summary (FETCH_SIZE + WRITE_SIZE, each scaled by what the same
    # counter reads for k_stream_copy) -- and only if that summary was taken from the kernel sources present
    from paper_2310_16795_amd import build as lib_build
    traffic, traffic_source = None, "none"
    tpath = os.path.join(ROOT, "profiles", f"traffic_{w.name}.json")
    if os.path.exists(tpath):
        with open(tpath) as f:
            tj = json.load(f)
        same = tj.get("kernel_sources") == lib_build.kernel_sources_hash()
        fits = tj.get("layout") == args.layout and not minmax and not custom_dict and not args.interchange_order and not args.tune
        if same and fits:
            traffic = tj["bytes_per_launch"].get(dom_key)
            traffic_source = f"profiles/traffic_{w.name}.json: {tj.get('command', 'rocprofv3 --pmc')}"
        else:
            traffic_source = (f"none: profiles/traffic_{w.name}.json was measured for " +
                              ("other kernel sources" if not same else "another configuration"))

    result = {
        "metric": "compressed_weight_GBps", "value": weight_bytes / (ms * 1e-3) / 1e9, "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "n_experts": w.n_experts, "d_model": w.d_model, "d_ff": w.d_ff,
                   "tokens": T, "experts_with_tokens": len(active), "routing": w.routing,
                   "zero_fraction": "0.80-0.97 per row" if w.p0_spread else w.p0,
                   "code_order": "interchange" if args.interchange_order else "device",
                   "stream_layout": (f"lane-interleaved ({layer.lanes['wi']} / {layer.lanes['wo']} lanes per matrix)"
                                     if lanes_layout else "rows back to back"),
                   "grid": "{w_min,0,w_max}, bf16 pair per row" if minmax else "{-s,0,+s}, binary16 scale per row",
                   "dict_entries": args.dict_entries, "dict_max_pairs": args.dict_max_pairs},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic, "traffic_source": traffic_source, "kernel": dom[0],
                     "kernel_ms": dom[1], "algorithmic_bytes": dom[2]},
        "hbm_frac_whole_step": weight_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "ms_per_step_spread": spread,
        "frac_of_stream_copy_rate": weight_bytes / (ms * 1e-3) / 1e9 / copy_gbps,
        # decode rate of the whole step: codewords per clock per compute unit at 2.4 GHz, 256 units
        "codewords_per_clk_per_cu": n_codewords / (ms * 1e-3) / (256 * 2.4e9),
        "cache_state": ("cold by construction: a step touches %.2f GB of codewords, more than four times the 256 MB "
                        "last-level cache plus L2" % (weight_bytes / 1e9)) if copies == 1 else
                       ("cold by rotation: the timed steps go round %d resident copies of the layer (%.2f GB together, at "
                        "least four times the 256 MB last-level cache plus L2)" % (copies, copies * weight_bytes / 1e9)),
        "ms_per_step_warm": warm_ms,
        "kernel_ms": kernel_ms,
        "kernels": {k: {"name": v[0], "algorithmic_bytes": v[1],
                        "GBps": (v[1] / (kernel_ms[k] * 1e-3) / 1e9) if kernel_ms[k] > 0 else None}
                    for k, v in kernels.items()},
        "experts_on_matrix_cores": len(crowded),
        "tokens_on_matrix_cores": int(sum(counts[e] for e in crowded)),
        "wall_ms_per_step": wall_ms,
        "compressed_bytes_touched": weight_bytes,
        "compressed_bytes_resident": layer.compressed_bytes,
        "bits_per_param": 8.0 * layer.compressed_bytes / (w.n_experts * n_params),
        "stream_copy_GBps": copy_gbps,
    }

    if not args.interchange_order:
        result["single_matvec_batch1"] = single_matvec(w, dd, gpu, active[0], minmax)

    if not args.no_bf16:
        t0 = time.time()
        if args.interchange_order:
            raise SystemExit("bench.py: the bf16 comparator needs device-order streams (drop --interchange-order "
                             "or add --no-bf16)")
        dstats = {}
        wi_p, wo_p, keep = dense_bf16_experts(layer, dd, active, gpu, dstats)
        result["decompress"] = dstats
        log(f"bf16 copies of {len(active)} experts: {sum(k.numel() for k in keep) * 2 / 1e9:.1f} GB "
            f"({time.time() - t0:.0f} s), decompressed at {dstats['GBps_written']:.0f} GB/s written")
        y2 = torch.empty_like(y)

        def step_bf16():
            q.qmoe_bf16_layer_forward(wi_p, wo_p, w.n_experts, w.d_model, w.d_ff, x, d_idx, None, y2, ws)

        bf_ms, _ = time_steps(step_bf16, max(3, args.steps // 3), 2)
        step()
        torch.cuda.synchronize()
        rel = float((y - y2).norm() / y.norm())
        bf_bytes = len(active) * n_params * 2
        result["bf16"] = {"ms_per_step": bf_ms, "GBps": bf_bytes / (bf_ms * 1e-3) / 1e9,
                          "bytes_touched": bf_bytes, "rel_diff_of_outputs": rel,
                          "kind": "hand-written grouped bf16 kernel, same dispatch, one launch per projection"}
        # the paper's own baseline style: one library matmul per expert (PyTorch / hipBLASLt)
        xb = x.view(torch.bfloat16)
        tok_of = {e: torch.from_numpy(np.nonzero(idx == e)[0]).to(gpu) for e in active}
        dense = {e: (keep[i], keep[len(active) + i]) for i, e in enumerate(active)}
        y3 = torch.empty_like(y)

        def step_torch():
            for e in active:
                t = tok_of[e]
                h = torch.relu(xb[t] @ dense[e][0].T)
                y3[t] = (h @ dense[e][1].T).float()

        tl_ms, _ = time_steps(step_torch, 3, 1)
        result["bf16"]["torch_loop_ms_per_step"] = tl_ms
        result["bf16"]["ideal_ms_at_stream_copy_rate"] = bf_bytes / (copy_gbps * 1e9) * 1e3
        result["time_vs_bf16"] = ms / min(bf_ms, tl_ms)
        del keep, dense

    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(w, idx, x_bits, active, minmax=minmax)
        result["cpu_baseline"]["host_cores_visible"] = os.cpu_count()

    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
