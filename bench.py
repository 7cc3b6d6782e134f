#!/usr/bin/env python3
"""Benchmark of the decode hot path on one MI355X.

A step is one pass of the hot path over the largest single-GPU workload: the full 32-layer
Llama-7B-shaped weight set (224 matrices from per-layer seeds, per-row absmax INT8, |q| <= 1 pruned;
6 476 005 376 int8 weights), cut in 64 KiB chunks of 256 sub-streams, all chunks Huffman coded: one
dc_decompress_chunks launch that decodes every chunk into one buffer in HBM.  All inputs are resident
in HBM before the timed region.

Prints one JSON line: decoded GB/s (value), the HBM roofline of the decode kernel, the CPU oracle timed
on the host cores, and under extras.configs every other workload (one matrix at 32 and 256 sub-streams,
one compression-aware layer, the speed-adaptive sweep, the fused paths on a 13B-shaped layer), each with
its compression ratio, decoded rate, share of the HBM roofline and whether the output was exact.

Host-only modes (no GPU): --alpha-sweep (compression ratio against the exponent of the per-channel
rescale and the pruning sparsity), --pair-stats (how often two codes fit one 11-bit table look-up).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
# Vector-ALU peak in lane-operations per second: 256 compute units x 4 SIMDs x 64 lanes of a wavefront instruction every
# `cycles` cycles at 2.4 GHz.  A SIMD issues plain 32-bit logic, add, subtract, right shift, move and fp32 add / multiply
# every 2 cycles and every other instruction the kernels use every 4 (bench.py --issue-rates); a kernel's peak follows
# from the mix of its main loop (profiles/counters.json, valu_cycles_per_instruction), 4 where no mix is recorded.
def alu_peak_lane_ops(cycles_per_instruction=4.0):
    return 256 * 4 * 64 * 2.4e9 / cycles_per_instruction


COUNTERS_FILE = os.path.join(ROOT, "profiles", "counters.json")


def load_counters(dc):
    """Per-kernel counter readings kept under profiles/ (rocprofv3 --pmc runs of this file), for the stored
    format this library writes; {} when the file is of another format id."""
    try:
        with open(COUNTERS_FILE) as f:
            doc = json.load(f)
    except (OSError, ValueError):
        return {}
    if doc.get("format_id") != dc.FORMAT_ID:
        return {}
    return doc.get("kernels", {})


def issue_rates(counters, key, raw_bytes, ms):
    """What keeps the decode launch below the HBM roofline: vector-ALU instructions (SQ_INSTS_VALU x 64 lanes, from the
    tracked counter run) over this run's duration against the rate the chip issues them at its nominal clock, and the
    share of LDS cycles lost to bank conflicts.  None where no counter run of this kernel and workload is tracked."""
    c = (counters or {}).get(key)
    if not c or "valu_insts" not in c:
        return None
    lane_ops = c["valu_insts"] * 64
    cpi = c.get("valu_cycles_per_instruction", 4.0)
    peak = alu_peak_lane_ops(cpi)
    out = {"bound": "alu", "achieved": round(lane_ops / (ms * 1e-3) / 1e12, 2), "peak": round(peak / 1e12, 2),
           "unit": "T lane-ops/s", "frac": round(lane_ops / (ms * 1e-3) / peak, 4),
           "lane_ops_per_decoded_byte": round(lane_ops / raw_bytes, 2),
           "peak_is": f"256 CUs x 4 SIMDs x 64 lanes / {cpi} cycles an instruction (this kernel's mix of 2- and 4-cycle "
                      "instructions) x 2.4 GHz; under this load the clock reads 2.0 GHz",
           "source": f"profiles/counters.json [{key}]"}
    if "lds_idx_active" in c and "lds_bank_conflict" in c:
        out["lds_cycles_lost_to_bank_conflicts"] = round(c["lds_bank_conflict"] / c["lds_idx_active"], 3)
    return out


def measured_traffic(counters, key):
    """HBM bytes per launch from the FETCH_SIZE / WRITE_SIZE readings of `key`, scaled by what the same
    counters read for the plain copy kernel; None when profiles/ has no reading for this kernel and workload."""
    c = counters.get(key)
    if not c or "fetch_kib" not in c or "write_kib" not in c:
        return None
    return int((c["fetch_kib"] * c.get("fetch_scale", 2.0) + c["write_kib"] * c.get("write_scale", 1.0)) * 1024)


_QUANTISED = {}


def quantise_layer(kind: str, layer: int, rescale: bool, dc, synth):
    """Generate and quantise (library) every matrix of a decoder layer once; cached."""
    key = (kind, layer, rescale)
    if key not in _QUANTISED:
        mats = []
        for m in synth.layer_specs(kind):
            seed = synth.matrix_seed(layer, m.index)
            w = synth.gen_weight(m.rows, m.cols, seed)
            a = synth.gen_act_absmax(m.cols, seed) if rescale else None
            q, row_scale, _ = dc.quantize_rows(w, a, 0.5, 1)
            del w
            mats.append((m, seed, q, row_scale))
        _QUANTISED[key] = mats
    return _QUANTISED[key]


def build_layer(kind: str, layer: int, rescale: bool, params, dc, synth):
    """Compress every matrix of a decoder layer with the library.  Returns a dict with the concatenated
    blob/table, per-matrix slices and the int8 bytes (for the parity check)."""
    blobs, tables, qs, scales, slices = [], [], [], [], []
    off = 0
    k0 = 0
    for m, seed, q, row_scale in quantise_layer(kind, layer, rescale, dc, synth):
        blob, table = dc.compress_chunks(q, params)
        table = table.copy()
        table["off"] += off
        slices.append(dict(name=m.name, rows=m.rows, cols=m.cols, k0=k0, n_chunks=len(table), seed=seed))
        off += blob.size
        k0 += len(table)
        blobs.append(blob)
        tables.append(table)
        qs.append(q.reshape(-1))
        scales.append(row_scale)
    return dict(blob=np.concatenate(blobs), table=np.concatenate(tables), q=np.concatenate(qs).view(np.uint8),
                scales=scales, slices=slices)


def model_weights(n_layers: int, dc, synth):
    """The int8 bytes of n_layers Llama-7B-shaped layers (per-layer seeds, per-row INT8 without the rescale,
    |q| <= 1 pruned), matrix after matrix in one array.  Matrices are drawn and quantised on a few threads."""
    jobs = [(layer, m) for layer in range(n_layers) for m in synth.layer_specs("llama7b")]
    sizes = [m.rows * m.cols for _, m in jobs]
    offs = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    flat = np.empty(int(offs[-1]), dtype=np.uint8)

    def one(i):
        layer, m = jobs[i]
        q, _, _ = dc.quantize_rows(synth.gen_weight(m.rows, m.cols, synth.matrix_seed(layer, m.index)), None, 0.5, 1)
        flat[offs[i]:offs[i + 1]] = q.reshape(-1).view(np.uint8)

    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
        list(pool.map(one, range(len(jobs))))
    return flat


def time_launches(torch, fn, steps, warmup):
    """Average duration (ms) of fn() launches on torch's current stream, by HIP events."""
    for i in range(warmup):
        fn(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for i in range(steps):
        fn(warmup + i)
    e1.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3
    return e0.elapsed_time(e1) / steps, wall / steps


def time_each_launch(torch, fn, n, first=0):
    """Durations (ms) of n launches of fn(), each between its own pair of HIP events, in launch order."""
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
    torch.cuda.synchronize()
    for i, (e0, e1) in enumerate(pairs):
        e0.record()
        fn(first + i)
        e1.record()
    torch.cuda.synchronize()
    return [e0.elapsed_time(e1) for e0, e1 in pairs]


def up(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.uint8).reshape(-1)).cuda()


def hbm_frac(raw_bytes, blob_bytes, table_bytes, ms, written_per_byte=1):
    """Algorithmic bytes of a launch (blob and table read, decoded bytes written) per second over the HBM peak."""
    return (written_per_byte * raw_bytes + blob_bytes + table_bytes) / ms / 1e6 / HBM_PEAK_GBPS


def compress_on_device(torch, dc, src_d, raw_bytes, params, stream):
    """dc_compress_chunks_dev into buffers of exactly the size used.  Its blob and table are byte for byte the
    host compressor's and the oracle's (tests/test_gpu_compress.py), so the compression ratio is theirs."""
    cap, nc = dc.compress_bound(raw_bytes, params)
    big = torch.empty(cap, dtype=torch.uint8, device="cuda")
    table_d = torch.empty(nc * 16, dtype=torch.uint8, device="cuda")
    ws_n = dc.compress_chunks_dev_workspace(raw_bytes, params)
    ws = torch.empty(ws_n, dtype=torch.uint8, device="cuda")
    res = torch.zeros(2, dtype=torch.int64, device="cuda")
    ms = None
    for _ in range(2):  # the second call is the one timed: the first loads the compression kernels
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        dc.compress_chunks_dev(src_d, raw_bytes, params, big, cap, table_d, nc, ws, ws_n, res, stream)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3
    used, status = (int(v) for v in res.cpu())
    if status != 0:
        raise RuntimeError("dc_compress_chunks_dev: blob buffer too small")
    blob_d = big[:used].clone()
    del big, ws
    return blob_d, used, table_d, nc, ms


# ---------------------------------------------------------------------------------------------- config 3


def run_config3(torch, dc, synth, args, counters):
    """The whole model in one launch: headline figures, cold and steady launches, the chunk-size sweep."""
    stream = torch.cuda.current_stream().cuda_stream
    t0 = time.perf_counter()
    flat = model_weights(args.layers, dc, synth)
    gen_s = time.perf_counter() - t0
    raw_bytes = flat.size
    src_d = torch.from_numpy(flat).cuda()
    dst = torch.empty(raw_bytes, dtype=torch.uint8, device="cuda")
    C, S = args.chunk, args.streams
    codec = dc.CODEC_TANS if args.codec == "tans" else dc.CODEC_HUFFMAN
    params = dc.Params(C, S, codec=codec)
    blob_d, blob_bytes, table_d, n_chunks, comp_ms = compress_on_device(torch, dc, src_d, raw_bytes, params, stream)

    def decode(i):
        dc.decompress_chunks(blob_d, blob_bytes, table_d, n_chunks, params, dst, raw_bytes, stream)

    cold = time_each_launch(torch, decode, 21)  # launches 0..20 of this kernel in this process
    ms, wall_ms = time_launches(torch, decode, args.steps, args.warmup)
    exact = bool(torch.equal(dst, src_d))
    alone = sorted(time_each_launch(torch, decode, 20)) if not args.no_side else None
    table_bytes = 16 * n_chunks
    ratio = raw_bytes / (blob_bytes + table_bytes)
    algo_bytes = raw_bytes + blob_bytes + table_bytes
    achieved = algo_bytes / ms / 1e6
    kernel = f"dc_decode_kernel<{S},int8" + (",tANS>" if args.codec == "tans" else ">")
    whole = args.layers == 32
    workload = (f"config 3: {'full ' if whole else 'SUBSET of '}{args.layers}-layer Llama-7B-shaped weight set from per-layer "
                f"seeds (per-row absmax INT8, |q|<=1 pruned), every chunk decoded into one HBM buffer by one launch, "
                f"{C // 1024} KiB chunks, {S} sub-streams, all chunks " + ("Huffman" if args.codec == "huffman" else "tANS") + " coded")
    tag = f"{kernel}|config3_{args.layers}layers_{C // 1024}KiB"
    traffic = measured_traffic(counters, tag)
    out = {
        "value": round(raw_bytes / ms / 1e6, 2),
        "ms_per_step": round(ms, 5),
        "config": {"workload": workload, "raw_bytes": raw_bytes, "chunk_bytes": C, "n_streams": S, "n_chunks": n_chunks,
                   "blob_bytes": blob_bytes, "compression_ratio": round(ratio, 5), "exact": exact,
                   "buffers_rotated": 1,
                   "note": "one launch moves 12 GB, 48 times the 256 MB memory-side cache: no rotation of buffers needed"},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
                     "traffic_source": f"profiles/counters.json [{tag}]" if traffic else None,
                     "kernel": kernel, "algorithmic_bytes_per_launch": int(algo_bytes), "avg_launch_ms": round(ms, 5)},
        "issue_rates": issue_rates(counters, tag, raw_bytes, ms),
        "wall_ms_per_step": round(wall_ms, 5),
        "roofline_limited_decoded_gbps": round(HBM_PEAK_GBPS / (1 + 1 / ratio), 1),
        "launch_index_against_duration": {
            "cold_launches_0_to_20_ms": [round(t, 4) for t in cold],
            "cold_mean_ms": round(float(np.mean(cold)), 4),
            "cold_decoded_GBps": round(raw_bytes / float(np.mean(cold)) / 1e6, 1),
            "steady_ms": round(ms, 5),
            "note": "cold: the first 21 launches of the kernel in this process, each between its own events; "
                    "steady: mean of the timed launches issued back to back after the warm-ups"},
        "generate_and_quantise_s": round(gen_s, 1),
        "compress_on_gpu_ms": round(comp_ms, 2),
    }
    if alone:
        out["launch_ms_each_timed_alone"] = {"median": round(alone[len(alone) // 2], 5), "min": round(alone[0], 5), "n": len(alone)}
    sample = None
    if not args.no_cpu:
        # the front of the blob for the CPU oracle, closed as a blob of its own
        n_sample = min(n_chunks, 4096)
        t = table_d[:16 * n_sample].cpu().numpy().view(dc.CHUNK_DTYPE)
        end = int(t["off"][-1]) + int(t["comp_bytes"][-1])
        sample = dict(blob=np.concatenate([blob_d[:end].cpu().numpy(), blob_d[blob_bytes - 64:blob_bytes].cpu().numpy()]),
                      table=t, q=flat[:min(raw_bytes, n_sample * C)], C=C, S=S, codec=codec)
    sweep = []
    if not args.no_extras:
        for c2, s2 in ((16384, 64), (16384, 256), (65536, 64), (65536, 256), (262144, 64), (262144, 256)):
            if (c2, s2) == (C, S) and args.codec == "huffman":
                sweep.append({"chunk_bytes": c2, "n_streams": s2, "n_chunks": n_chunks, "compression_ratio": round(ratio, 5),
                              "ms": round(ms, 4), "decoded_GBps": out["value"], "hbm_frac": out["roofline"]["frac"], "exact": exact})
                continue
            p2 = dc.Params(c2, s2)
            b2, nb2, t2, nc2, _ = compress_on_device(torch, dc, src_d, raw_bytes, p2, stream)
            dst.zero_()
            ms2, _ = time_launches(torch, lambda i: dc.decompress_chunks(b2, nb2, t2, nc2, p2, dst, raw_bytes, stream), 10, 3)
            sweep.append({"chunk_bytes": c2, "n_streams": s2, "n_chunks": nc2,
                          "compression_ratio": round(raw_bytes / (nb2 + 16 * nc2), 5), "ms": round(ms2, 4),
                          "decoded_GBps": round(raw_bytes / ms2 / 1e6, 1),
                          "hbm_frac": round(hbm_frac(raw_bytes, nb2, 16 * nc2, ms2), 4),
                          "exact": bool(torch.equal(dst, src_d))})
            del b2, t2
    # plain copy kernel at the same size: the achievable-bandwidth line
    cms, _ = time_launches(torch, lambda i: dc.device_copy(src_d, dst, raw_bytes, stream), 10, 3)
    out["copy_kernel_GBps_read_plus_write"] = round(2 * raw_bytes / cms / 1e6, 1)
    out["decode_frac_of_copy_bandwidth"] = round(achieved / (2 * raw_bytes / cms / 1e6), 4)
    del src_d, dst, blob_d, table_d
    torch.cuda.empty_cache()
    return out, sweep, sample, flat


# ---------------------------------------------------------------------------------------------- configs 1, 2, 4


def timed_decode(torch, dc, blob, table, params, q, steps=200, warmup=20, rotate=True):
    """Decode a host blob on the device, buffers rotated through more than 640 MB unless told otherwise.
    Returns ms per launch and whether every decoded byte equals q."""
    stream = torch.cuda.current_stream().cuda_stream
    raw = q.size
    nbuf = max(2, int(np.ceil(640e6 / (raw + blob.size)))) if rotate else 1
    blobs = [up(torch, blob) for _ in range(nbuf)]
    table_d = up(torch, table)
    dsts = [torch.zeros(raw, dtype=torch.uint8, device="cuda") for _ in range(nbuf)]
    n = len(table)

    def decode(i):
        dc.decompress_chunks(blobs[i % nbuf], blob.size, table_d, n, params, dsts[i % nbuf], raw, stream)

    warmup = max(warmup, nbuf)  # every destination is written at least once
    ms, _ = time_launches(torch, decode, steps, warmup)
    want = up(torch, q)
    exact = all(bool(torch.equal(d, want)) for d in dsts)
    return ms, exact, nbuf


def decode_row(torch, dc, blob, table, params, q, **kw):
    ms, exact, nbuf = timed_decode(torch, dc, blob, table, params, q, **kw)
    return {"n_streams": params.n_streams, "chunk_bytes": params.chunk_bytes, "n_chunks": len(table),
            "compression_ratio": round(q.size / (blob.size + table.nbytes), 5), "ms": round(ms, 5),
            "decoded_GBps": round(q.size / ms / 1e6, 1),
            "hbm_frac": round(hbm_frac(q.size, blob.size, table.nbytes, ms), 4), "exact": exact, "buffers_rotated": nbuf}


def run_config1(torch, dc, q1):
    """One 4096 x 4096 matrix, 256 chunks of 64 KiB, all Huffman coded: at the 32 sub-streams the workload
    names, and at 64 and 256; with the buffers rotated (HBM) and not (memory-side cache)."""
    rows = []
    for S in (32, 64, 256):
        p = dc.Params(65536, S)
        blob, table = dc.compress_chunks(q1, p)
        r = decode_row(torch, dc, blob, table, p, q1)
        ms_c, _, _ = timed_decode(torch, dc, blob, table, p, q1, rotate=False)
        r["cache_resident_ms"] = round(ms_c, 5)
        r["cache_resident_decoded_GBps"] = round(q1.size / ms_c / 1e6, 1)
        rows.append(r)
    return {"workload": "config 1: one 4096x4096 matrix (per-row INT8, |q|<=1 pruned), 64 KiB chunks, all Huffman coded; "
                        "256 chunks are one workgroup per compute unit, so the launch is bound by the latency of one "
                        "chunk's chain of dependent table look-ups, not by bandwidth",
            "raw_bytes": int(q1.size), "by_n_streams": rows}


def run_config4(torch, dc, q, S, label):
    """Speed-adaptive partial compression: fraction f of the chunks stored raw, lowest Huffman gain first."""
    sweep = []
    for f in (0.0, 0.25, 0.5, 0.75, 1.0):
        pf = dc.Params(65536, S, dc.POLICY_RAW_FRACTION, f)
        blob, table = dc.compress_chunks(q, pf)
        r = decode_row(torch, dc, blob, table, pf, q, steps=100, warmup=10)
        r["raw_fraction"] = f
        r["raw_chunks"] = int(((table["raw_bytes_flags"] >> 31) & 1).sum())
        sweep.append(r)
    # Section 3.3's throughput reasoning for a mix: time per byte = (1-f)/D_coded + f/D_raw
    d0, d1 = sweep[0]["decoded_GBps"], sweep[-1]["decoded_GBps"]
    for r in sweep:
        r["model_GBps"] = round(1.0 / ((1 - r["raw_fraction"]) / d0 + r["raw_fraction"] / d1), 1)
    return {"workload": label, "n_streams": S, "sweep": sweep}


def run_config2(torch, dc, synth, args):
    """One compression-aware Llama-7B-shaped layer (3088 chunks): sub-stream sweep, the second coder, the paper's
    positional rule against the gain-ranked one, the compressors."""
    stream = torch.cuda.current_stream().cuda_stream
    C = 65536
    out = {"workload": "config 2: one Llama-7B-shaped decoder layer, 7 matrices, compression-aware INT8 (s=a^0.5, "
                       "a~LogNormal(0,1)), 64 KiB chunks, all chunks coded, one launch; 3088 chunks are 1.5 rounds of "
                       "the 2048 workgroups the GPU holds at 256 sub-streams"}
    rows = []
    layer = None
    for S in (32, 64, 128, 256):
        p = dc.Params(C, S)
        l2 = build_layer("llama7b", 0, True, p, dc, synth)
        rows.append(decode_row(torch, dc, l2["blob"], l2["table"], p, l2["q"]))
        if S == 256:
            layer = l2
    out["raw_bytes"] = int(layer["q"].size)
    out["by_n_streams"] = rows
    q = layer["q"]
    # the container's second coder (tANS, 2048 states; the paper settles on ANS in Section 4.2)
    tans_rows = []
    for c2, s2 in ((C, 256), (262144, 64), (262144, 256)):
        row = {"chunk_bytes": c2, "n_streams": s2}
        for name, codec in (("huffman", dc.CODEC_HUFFMAN), ("tans", dc.CODEC_TANS)):
            p2 = dc.Params(c2, s2, codec=codec)
            l2 = build_layer("llama7b", 0, True, p2, dc, synth)
            r = decode_row(torch, dc, l2["blob"], l2["table"], p2, l2["q"])
            row[name] = {k: r[k] for k in ("decoded_GBps", "compression_ratio", "hbm_frac", "exact")}
        tans_rows.append(row)
    out["tans_against_huffman"] = tans_rows
    # The paper's own rule (Section 3.3: of every block of N chunks only the last is compressed) beside the
    # gain-ranked rule at the same share of raw chunks, 1 - 1/N
    pareto = []
    for n_block in (2, 4, 5):
        row = {"block_chunks": n_block, "raw_fraction": round(1 - 1 / n_block, 4)}
        for name, pf in (("positional", dc.Params(C, 256, dc.POLICY_BLOCK_LAST, 0.0, n_block)),
                         ("gain_ranked", dc.Params(C, 256, dc.POLICY_RAW_FRACTION, 1 - 1 / n_block))):
            lf = build_layer("llama7b", 0, True, pf, dc, synth)
            r = decode_row(torch, dc, lf["blob"], lf["table"], pf, lf["q"], steps=100, warmup=10)
            row[name] = {k: r[k] for k in ("decoded_GBps", "compression_ratio", "hbm_frac", "exact")}
            row[name]["raw_chunks"] = int(((lf["table"]["raw_bytes_flags"] >> 31) & 1).sum())
        pareto.append(row)
    out["positional_rule_against_gain_ranked"] = pareto
    # compression of the same layer on the GPU (Section 4.2 reports compression speed as well), and on the host
    q_d = up(torch, q)
    for name, codec in (("compress_on_gpu", dc.CODEC_HUFFMAN), ("compress_on_gpu_tans", dc.CODEC_TANS)):
        pc = dc.Params(C, 256, codec=codec)
        cap_c, nc_c = dc.compress_bound(q.size, pc)
        blob_c = torch.empty(cap_c, dtype=torch.uint8, device="cuda")
        table_c = torch.empty(nc_c * 16, dtype=torch.uint8, device="cuda")
        ws_n = dc.compress_chunks_dev_workspace(q.size, pc)
        ws_c = torch.empty(ws_n, dtype=torch.uint8, device="cuda")
        res_c = torch.zeros(2, dtype=torch.int64, device="cuda")
        cms, _ = time_launches(
            torch, lambda i: dc.compress_chunks_dev(q_d, q.size, pc, blob_c, cap_c, table_c, nc_c, ws_c, ws_n, res_c, stream),
            20, 3)
        out[name] = {"GBps": round(q.size / cms / 1e6, 1), "ms": round(cms, 4), "blob_bytes": int(res_c.cpu()[0]),
                     "workspace_bytes": ws_n}
        del blob_c, table_c, ws_c
    t0 = time.perf_counter()
    dc.compress_chunks(q, dc.Params(C, 256))
    out["compress_on_host"] = {"GBps": round(q.size / (time.perf_counter() - t0) / 1e9, 3), "threads": os.cpu_count()}
    return out, layer


# ---------------------------------------------------------------------------------------------- config 5


def run_config5(torch, dc, synth, counters):
    """Fused paths on the Llama-13B-shaped layer (hidden 5120, FFN 13824, quantised without rescale): decode
    fused with the dequantisation to bf16, and with the batch-1 product; matrix by matrix and as one launch
    over the layer.  The outputs are checked here against plain PyTorch on the device (the tests hold them to
    the CPU oracle): bf16 bits must be equal, the product within 1e-2 of an fp64 product."""
    stream = torch.cuda.current_stream().cuda_stream
    C, S = 65536, 256
    params = dc.Params(C, S)
    l13 = build_layer("llama13b", 0, False, params, dc, synth)
    b13 = [up(torch, l13["blob"]) for _ in range(2)]
    t13 = up(torch, l13["table"])
    raw13, blob13, nc13 = l13["q"].size, l13["blob"].size, len(l13["table"])
    scales_d = [torch.from_numpy(s).cuda() for s in l13["scales"]]
    offs13 = np.cumsum([0] + [sl["rows"] * sl["cols"] for sl in l13["slices"]])
    layer16 = [torch.empty(raw13, dtype=torch.int16, device="cuda") for _ in range(2)]
    xs = [torch.from_numpy(synth.gen_activation_bf16(sl["cols"], sl["seed"]).view(np.int16)).cuda() for sl in l13["slices"]]
    ys = [torch.empty(sl["rows"], dtype=torch.float32, device="cuda") for sl in l13["slices"]]
    ws_bytes = dc.decompress_gemv_workspace(nc13)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")

    def dequant(i):
        for j, sl in enumerate(l13["slices"]):
            dc.decompress_dequant_bf16(b13[i % 2], blob13, t13.data_ptr() + 16 * sl["k0"], sl["n_chunks"], params,
                                       scales_d[j], sl["rows"], sl["cols"], layer16[i % 2].data_ptr() + 2 * int(offs13[j]),
                                       sl["rows"] * sl["cols"], stream)

    def gemv(i):
        for j, sl in enumerate(l13["slices"]):
            dc.decompress_gemv(b13[i % 2], blob13, t13.data_ptr() + 16 * sl["k0"], sl["n_chunks"], params,
                               scales_d[j], sl["rows"], sl["cols"], xs[j], ys[j], None, ws, ws_bytes, stream)

    mats_b = [dc.Matrix(sl["k0"], sl["rows"], sl["cols"], scales_d[j], dst_bf16_dev=None, dst_cap_elems=sl["rows"] * sl["cols"])
              for j, sl in enumerate(l13["slices"])]
    mats_g = [dc.Matrix(sl["k0"], sl["rows"], sl["cols"], scales_d[j], x_bf16_dev=xs[j], y_accum_dev=ys[j])
              for j, sl in enumerate(l13["slices"])]

    def dequant_layer(i):
        for j, m in enumerate(mats_b):
            m.dst_bf16_dev = layer16[i % 2].data_ptr() + 2 * int(offs13[j])
        dc.decompress_dequant_bf16_layer(b13[i % 2], blob13, t13, nc13, params, mats_b, stream)

    def gemv_layer(i):
        dc.decompress_gemv_layer(b13[i % 2], blob13, t13, nc13, params, mats_g, ws, ws_bytes, stream)

    def matrix_on_device(j, sl):
        return torch.from_numpy(l13["q"][offs13[j]:offs13[j + 1]].view(np.int8)).cuda().view(sl["rows"], sl["cols"])

    def check_dequant():
        ok = True
        for j, sl in enumerate(l13["slices"]):
            want = (matrix_on_device(j, sl).float() * scales_d[j][:, None]).to(torch.bfloat16).view(torch.int16).reshape(-1)
            for buf in layer16:
                ok = ok and bool(torch.equal(buf[offs13[j]:offs13[j + 1]], want))
        return ok

    def check_gemv():
        ok, worst = True, 0.0
        for j, sl in enumerate(l13["slices"]):
            x64 = (xs[j].to(torch.int32) << 16).view(torch.float32).double()
            ref = (matrix_on_device(j, sl).double() @ x64) * scales_d[j].double()
            err = (ys[j].double() - ref).abs()
            rms = ref.pow(2).mean().sqrt()
            ok = ok and bool((err <= 1e-2 * ref.abs() + 1e-2 * rms).all())
            worst = max(worst, float(err.max() / ref.abs().max()))
        return ok, worst

    res = {}
    for name, fn, kind in (("per_matrix_calls", (dequant, gemv), "7 calls a pass"),
                           ("whole_layer_call", (dequant_layer, gemv_layer), "1 call a pass")):
        for b in layer16:
            b.zero_()
        dms, _ = time_launches(torch, fn[0], 30, 3)
        d_ok = check_dequant()
        for y in ys:
            y.zero_()
        gms, _ = time_launches(torch, fn[1], 30, 3)
        g_ok, g_err = check_gemv()
        res[name] = {"calls": kind,
                     "dequant_bf16": {"ms": round(dms, 4), "int8_GBps": round(raw13 / dms / 1e6, 1),
                                      "hbm_frac": round((blob13 + 16 * nc13 + 2 * raw13) / dms / 1e6 / HBM_PEAK_GBPS, 4),
                                      "bf16_bits_equal_torch": d_ok},
                     "gemv": {"ms": round(gms, 4), "weights_GBps": round(raw13 / gms / 1e6, 1),
                              "hbm_frac": round((blob13 + 16 * nc13) / gms / 1e6 / HBM_PEAK_GBPS, 4),
                              "within_1e-2_of_fp64": g_ok, "max_normwise_error": float(f"{g_err:.3e}")}}
    # the product is bound by the vector ALU, not by HBM: lane-operations issued (counter reading kept under
    # profiles/) over the chip's lane-operations per second
    g = res["whole_layer_call"]["gemv"]
    g["roofline_alu"] = issue_rates(counters, "dc_decode_kernel<256,gemv>|config5_layer", raw13, g["ms"])
    if g["roofline_alu"]:
        g["roofline_alu"]["lane_ops_per_weight"] = g["roofline_alu"].pop("lane_ops_per_decoded_byte")
    g["gemv_alu_frac"] = g["roofline_alu"]["frac"] if g["roofline_alu"] else None
    d = res["whole_layer_call"]["dequant_bf16"]
    d["issue_rates"] = issue_rates(counters, "dc_decode_kernel<256,bf16>|config5_layer", raw13, d["ms"])
    return {"workload": "config 5: fused paths on one Llama-13B-shaped layer (4 x 5120x5120, 2 x 13824x5120, 5120x13824; per-row "
                        "INT8, |q|<=1 pruned), 64 KiB chunks, 256 sub-streams, bf16 activations ~N(0,1)",
            "raw_bytes": int(raw13), "n_chunks": nc13, "compression_ratio": round(raw13 / (blob13 + 16 * nc13), 5), **res}


# ---------------------------------------------------------------------------------------------- layer streaming


def layer_streaming(torch, dc, synth, params, layer, n_layers=8, reps=10):
    """The paper's runtime loop (Section 3.3, case (b): everything in GPU memory) on the Llama-7B-shaped
    layer: per-layer latency of batch-1 inference (seven matrix-vector products a layer) with the
    weights (i) resident uncompressed, (ii) decoded into the decompression buffer and then used, on one
    stream, (iii) the same with the decode of layer l+1 on a second stream while layer l computes
    (two buffers), (iv) through the fused decode+product call.  Every layer uses the same weights (distinct
    buffers); times are wall-clock per layer of launches recorded once into a HIP graph and replayed."""
    lay = layer
    raw_bytes = lay["q"].size
    side = torch.cuda.Stream()
    scales = [torch.from_numpy(s).cuda() for s in lay["scales"]]
    xs = [torch.from_numpy(synth.gen_activation_bf16(sl["cols"], sl["seed"]).view(np.int16)).cuda() for sl in lay["slices"]]
    ys = [torch.empty(sl["rows"], dtype=torch.float32, device="cuda") for sl in lay["slices"]]
    bufs = [torch.empty(raw_bytes, dtype=torch.uint8, device="cuda") for _ in range(2)]
    offs = np.cumsum([0] + [sl["rows"] * sl["cols"] for sl in lay["slices"]])
    blobs = [up(torch, lay["blob"]) for _ in range(2)]
    table = up(torch, lay["table"])
    nb, nc = lay["blob"].size, len(lay["table"])
    not_replayed = []

    def compute(buf, st):
        for j, sl in enumerate(lay["slices"]):
            dc.gemv_i8(buf.data_ptr() + int(offs[j]), scales[j], sl["rows"], sl["cols"], xs[j], ys[j], None, st.cuda_stream)

    def wall(name, fn):
        """ms per layer of fn(stream), which enqueues n_layers layers, replayed from a HIP graph so that the
        host's launch cost stays out of the per-layer time; a leg that could not be captured is timed with
        eager launches and named in `legs_not_replayed_from_a_graph`."""
        cap = torch.cuda.Stream()
        cap.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(cap):
            fn(cap)
        torch.cuda.synchronize()
        try:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=cap):
                fn(cap)
            g.replay()
            torch.cuda.synchronize()
            run = g.replay
        except RuntimeError as e:
            torch.cuda.synchronize()
            not_replayed.append(f"{name}: {type(e).__name__}")
            run = lambda: fn(torch.cuda.current_stream())  # noqa: E731
        t0 = time.perf_counter()
        for _ in range(reps):
            run()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / (reps * n_layers)

    def decode(i, st):
        dc.decompress_chunks(blobs[i % 2], nb, table, nc, params, bufs[i % 2], raw_bytes, st.cuda_stream)

    def decode_only(main):
        for i in range(n_layers):
            decode(i, main)

    def serial(main):
        for i in range(n_layers):
            decode(i, main)
            compute(bufs[i % 2], main)

    def overlapped(main):
        side.wait_stream(main)
        done = [None, None]  # compute that last read each buffer
        for i in range(n_layers):
            if done[i % 2] is not None:
                side.wait_event(done[i % 2])
            decode(i, side)
            ready = torch.cuda.Event()
            ready.record(side)
            main.wait_event(ready)
            compute(bufs[i % 2], main)
            done[i % 2] = torch.cuda.Event()
            done[i % 2].record(main)
        main.wait_stream(side)

    d_ms, ser_ms, ovl_ms = wall("decode", decode_only), wall("one_stream", serial), wall("second_stream", overlapped)
    i_ms = wall("resident", lambda main: [compute(bufs[i % 2], main) for i in range(n_layers)])
    y_resident = [y.clone() for y in ys]
    mats = [dc.Matrix(sl["k0"], sl["rows"], sl["cols"], scales[j], x_bf16_dev=xs[j], y_accum_dev=ys[j])
            for j, sl in enumerate(lay["slices"])]
    ws_bytes = dc.decompress_gemv_workspace(nc)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")

    def fused(main):
        for i in range(n_layers):
            dc.decompress_gemv_layer(blobs[i % 2], nb, table, nc, params, mats, ws, ws_bytes, main.cuda_stream)

    f_ms = wall("fused", fused)
    torch.cuda.synchronize()
    ok = bool(torch.equal(bufs[1], up(torch, lay["q"])))
    for yf, y in zip(ys, y_resident):
        ok = ok and bool(torch.allclose(yf, y, rtol=1e-3, atol=1e-3 * float(y.abs().max())))
    return {"n_layers": n_layers, "n_streams": params.n_streams,
            "decoded_buffer_exact_and_products_agree": ok,
            "ms_per_layer": {"resident_compute_I": round(i_ms, 4), "decode_D": round(d_ms, 4),
                             "decode_then_compute_one_stream": round(ser_ms, 4),
                             "decode_next_layer_on_second_stream": round(ovl_ms, 4), "fused_decode_product": round(f_ms, 4)},
            "model_ms_per_layer": {"one_stream_D_plus_I": round(d_ms + i_ms, 4), "overlapped_max_D_I": round(max(d_ms, i_ms), 4)},
            "overhead_vs_resident": {"one_stream": round(ser_ms / i_ms - 1, 3), "second_stream": round(ovl_ms / i_ms - 1, 3),
                                     "fused": round(f_ms / i_ms - 1, 3)},
            "legs_not_replayed_from_a_graph": not_replayed}


# ---------------------------------------------------------------------------------------------- CPU oracle


def cpu_baseline(sample):
    """The plain-C oracle on the host cores, on the front of the blob the GPU decoded."""
    import oracle.codec as oc

    blob, table, q, C, S, codec = (sample[k] for k in ("blob", "table", "q", "C", "S", "codec"))
    threads = min(os.cpu_count() or 1, 16)
    raw = q.size
    t0 = time.perf_counter()
    reps = 0
    while True:
        ref = oc.decompress(blob, table, C, S, raw, threads=threads, codec=codec)
        reps += 1
        if time.perf_counter() - t0 > 1.5 and reps >= 2:
            break
    dt = (time.perf_counter() - t0) / reps
    assert np.array_equal(ref, q)
    n_small = min(128, len(table))
    small_raw = min(raw, n_small * C)
    t0 = time.perf_counter()
    oc.decompress(blob, table[:n_small], C, S, small_raw, threads=1, codec=codec)
    one_thread = small_raw / (time.perf_counter() - t0) / 1e9
    t0 = time.perf_counter()
    enc = oc.compress(q[:small_raw], C, S, threads=threads, codec=codec)
    encode = small_raw / (time.perf_counter() - t0) / 1e9
    # the oracle's own blob of these chunks is the front of the blob the GPU decoded: same compression ratio
    same = np.array_equal(enc.blob[:-64], blob[:int(table["off"][n_small - 1]) + int(table["comp_bytes"][n_small - 1])])
    return {"value": round(raw / dt / 1e9, 3), "unit": "GB/s", "cores": threads, "kind": "oracle",
            "sample": f"first {len(table)} chunks ({raw} decoded bytes) of the blob the GPU decoded, {reps} passes, "
                      f"bit-serial C oracle, chunk range split over {threads} threads",
            "one_thread_GBps": round(one_thread, 4), "encode_GBps": round(encode, 4),
            "encode_sample": f"first {n_small} chunks compressed by the oracle on {threads} threads",
            "oracle_blob_equals_decoded_blob": bool(same)}


# ---------------------------------------------------------------------------------------------- host-only modes


def alpha_sweep_table(dc, synth, rows, cols, alphas, sparsities, chunk_bytes=65536, n_streams=64):
    """[(sparsity, [compression ratio per alpha])]: the paper's per-tensor quantisation (dc_quantize_tensor: one
    scale for the tensor, rescale s = a^alpha of Eq. 2, score pruning of Eq. 5), chunks that do not shrink raw."""
    seed = synth.matrix_seed(0, 0)
    w = synth.gen_weight(rows, cols, seed)
    a = synth.gen_act_absmax(cols, seed)
    p = dc.Params(chunk_bytes, n_streams, dc.POLICY_AUTO)
    out = []
    for sparsity in sparsities:
        crs = []
        for alpha in alphas:
            q, _, _ = dc.quantize_tensor(w, a, alpha, sparsity)
            blob, t = dc.compress_chunks(q, p)
            crs.append(q.size / (blob.size + t.nbytes))
        out.append((sparsity, crs))
    return out


def alpha_sweep(dc, synth, rows=4096, cols=4096):
    """Compression ratio against the exponent alpha of the per-channel rescale and the sparsity of the score
    pruning on the config-1 tensor: the shape of the paper's ablation on alpha (Section 4.4).  Host only."""
    alphas = [i / 10 for i in range(11)]
    table = alpha_sweep_table(dc, synth, rows, cols, alphas, (0.0, 0.2, 0.4))
    print(json.dumps({"workload": f"{rows}x{cols} synthetic weights (1% of rows x8), a~LogNormal(0,1), per-tensor INT8, "
                                  "64 KiB chunks, 64 sub-streams, chunks that do not shrink stored raw",
                      "rows": [{"sparsity": s, "compression_ratio_by_alpha": {f"{a:.1f}": round(c, 4) for a, c in zip(alphas, crs)}}
                               for s, crs in table]}))
    return 0


def pair_stats(dc, synth):
    """How often would a decode table that holds two symbols per entry deliver two?  For chunks of configs 1/3
    (no rescale) and 2 (rescale): the share of adjacent code pairs of a sub-stream that fit the 11-bit window, and
    what a wavefront gains, whose 64 lanes move in step through half groups of 8 symbols (the stored format
    places blocks by that step): the look-ups of a half group are those of its slowest lane.  Host only."""
    out = []
    for name, rescale in (("configs 1 and 3 (per-row INT8, no rescale)", False), ("config 2 (rescale s=a^0.5)", True)):
        seed = synth.matrix_seed(0, 0)
        w = synth.gen_weight(4096, 4096, seed)
        q, _, _ = dc.quantize_rows(w, synth.gen_act_absmax(4096, seed) if rescale else None, 0.5, 1)
        data = q.reshape(-1).view(np.uint8)[:16 * 65536]
        S = 256
        blob, table = dc.compress_chunks(data, dc.Params(65536, S))
        fits, pairs, lane_lookups, wave_lookups, halves, bits, syms = 0, 0, 0.0, 0.0, 0, 0, 0
        for k in range(len(table)):
            o = int(table["off"][k])
            nib = blob[o:o + 128]
            lens = np.empty(256, dtype=np.int64)
            lens[0::2], lens[1::2] = nib & 15, nib >> 4
            chunk = data[k * 65536:(k + 1) * 65536]
            bits += int(lens[chunk].sum())
            syms += chunk.size
            ln = lens[chunk].reshape(-1, S, 16)  # [round][stream][symbol of the group]
            ln = ln.transpose(1, 0, 2).reshape(S, -1, 8)  # [stream][half group][symbol]
            two = (ln[:, :, :-1] + ln[:, :, 1:]) <= 11
            fits += int(two.sum())
            pairs += two.size
            # greedy pairing inside a half group: look-ups a lane needs for its 8 symbols
            need = np.zeros(ln.shape[:2], dtype=np.int64)
            i = np.zeros(ln.shape[:2], dtype=np.int64)
            for _ in range(8):
                live = i < 8
                cur = np.take_along_axis(ln, np.minimum(i, 7)[..., None], 2)[..., 0]
                nxt = np.take_along_axis(ln, np.minimum(i + 1, 7)[..., None], 2)[..., 0]
                pair = live & (i < 7) & (cur + nxt <= 11)
                need += live
                i += np.where(live, np.where(pair, 2, 1), 0)
            lane_lookups += float(need.mean()) * need.shape[1]
            wave = need.reshape(S // 64, 64, -1).max(axis=1)  # a wavefront waits for its slowest lane
            wave_lookups += float(wave.mean()) * need.shape[1]
            halves += need.shape[1]
        out.append({"data": name, "mean_code_bits": round(bits / syms, 3),
                    "adjacent_pairs_that_fit_11_bits": round(fits / pairs, 4),
                    "lookups_per_half_group_a_lane_alone": round(lane_lookups / halves, 3),
                    "lookups_per_half_group_a_wavefront_in_step": round(wave_lookups / halves, 3),
                    "lookups_per_half_group_now": 8})
    print(json.dumps({"two_symbol_table_entries": out}))
    return 0


def mix_sweep(torch, dc, synth):
    """Raw and coded chunks in one launch (Section 3.3's speed-adaptive storage), on the config-2 layer and on a
    four-layer weight set: the share f of raw chunks by gain and the positional rule with blocks of N, and, on the
    layer at f = 0.5, the same chunks with the table (and the expected bytes) put into other orders: runs of c coded
    then r raw chunks.  One JSON line."""
    p0 = dc.Params(65536, 256)
    layer_q = build_layer("llama7b", 0, True, p0, dc, synth)["q"]
    model_q = model_weights(4, dc, synth)
    out = {"n_streams": 256, "chunk_bytes": 65536}

    def rate(q, p, table_order=None, **kw):
        blob, table = dc.compress_chunks(q, p)
        if table_order is not None:  # chunk k of the launch is chunk table_order[k] of the blob
            order = table_order(table)
            table = table[order]
            q = q.reshape(len(order), -1)[order].reshape(-1)
        r = decode_row(torch, dc, blob, table, p, q, **kw)
        return {"decoded_GBps": r["decoded_GBps"], "compression_ratio": r["compression_ratio"], "exact": r["exact"],
                "raw_chunks": int(((table["raw_bytes_flags"] >> 31) & 1).sum()), "n_chunks": len(table)}

    for name, q, kw in (("config2_layer", layer_q, dict(steps=300, warmup=30)), ("four_layers", model_q, dict(steps=40, warmup=5))):
        rows = []
        for f in (0.0, 0.1, 0.25, 0.5, 0.75, 0.9, 1.0):
            rows.append(dict(raw_fraction=f, **rate(q, dc.Params(65536, 256, dc.POLICY_RAW_FRACTION, f), **kw)))
        out[name + "_by_gain"] = rows
    rows = []
    for n in (2, 3, 4, 5, 6, 7, 8, 9, 16):
        rows.append(dict(block_chunks=n, **rate(layer_q, dc.Params(65536, 256, dc.POLICY_BLOCK_LAST, 0.0, n), steps=300, warmup=30)))
    out["config2_layer_positional"] = rows

    def runs(c, r, raw_first=False):
        def order(table):
            is_raw = ((table["raw_bytes_flags"] >> 31) & 1).astype(bool)
            raw, coded, o = list(np.nonzero(is_raw)[0]), list(np.nonzero(~is_raw)[0]), []
            while raw or coded:
                for src, cnt in (((raw, r), (coded, c)) if raw_first else ((coded, c), (raw, r))):
                    o += src[:cnt]
                    del src[:cnt]
            return np.array(o)
        return order

    rows = []
    half = dc.Params(65536, 256, dc.POLICY_RAW_FRACTION, 0.5)
    for label, order in (("as stored", None), ("1 coded, 1 raw", runs(1, 1)), ("1 raw, 1 coded", runs(1, 1, True)),
                         ("8, 8", runs(8, 8)), ("32, 32", runs(32, 32)), ("256, 256", runs(256, 256)),
                         ("all coded, then all raw", runs(1 << 30, 1 << 30)), ("all raw, then all coded", runs(1 << 30, 1 << 30, True))):
        rows.append(dict(order=label, **rate(layer_q, half, order, steps=300, warmup=30)))
    out["config2_layer_half_raw_by_order"] = rows
    # the same share chosen by place and not by gain, the decoded bytes in their own order: the back half of the layer raw
    n = (layer_q.size + 65535) // 65536
    mask = np.zeros(n, dtype=np.uint8)
    mask[n - n // 2:] = 1
    out["config2_layer_back_half_raw"] = [dict(rule="DC_POLICY_RAW_MASK, the last half of the chunks",
                                               **rate(layer_q, dc.Params(65536, 256, dc.POLICY_RAW_MASK, 0.0, 0, mask), steps=300, warmup=30))]
    ok = all(r["exact"] for k in out if isinstance(out[k], list) for r in out[k])
    print(json.dumps({"mix_sweep": out, "exact": ok}))
    return 0 if ok else 1


def compress_only(torch, dc, synth, args):
    """dc_compress_chunks_dev alone (for a profiler): the config-2 layer and a four-layer weight set, both coders,
    --steps calls each after 3 untimed ones.  One JSON line."""
    stream = torch.cuda.current_stream().cuda_stream
    sets = (("config2_layer", build_layer("llama7b", 0, True, dc.Params(65536, 256), dc, synth)["q"]),
            ("four_layers", model_weights(4, dc, synth)))
    rows = []
    for name, q in sets:
        q_d = up(torch, q)
        for codec_name, codec in (("huffman", dc.CODEC_HUFFMAN), ("tans", dc.CODEC_TANS)):
            p = dc.Params(args.chunk, args.streams, codec=codec)
            cap, nc = dc.compress_bound(q.size, p)
            blob = torch.empty(cap, dtype=torch.uint8, device="cuda")
            table = torch.empty(nc * 16, dtype=torch.uint8, device="cuda")
            ws_n = dc.compress_chunks_dev_workspace(q.size, p)
            ws = torch.empty(ws_n, dtype=torch.uint8, device="cuda")
            res = torch.zeros(2, dtype=torch.int64, device="cuda")
            ms, _ = time_launches(
                torch, lambda i: dc.compress_chunks_dev(q_d, q.size, p, blob, cap, table, nc, ws, ws_n, res, stream), args.steps, 3)
            blob_bytes = int(res.cpu()[0])
            rows.append({"input": name, "codec": codec_name, "raw_bytes": int(q.size), "ms": round(ms, 4),
                         "GBps": round(q.size / ms / 1e6, 1), "compression_ratio": round(q.size / (blob_bytes + nc * 16), 5),
                         "hbm_frac": round((q.size * 2 + blob_bytes) / ms / 1e6 / HBM_PEAK_GBPS, 4),
                         "bytes_moved": "the input is read twice (statistics, then coding) and the blob written once"})
            del blob, table, ws
    print(json.dumps({"compress_on_gpu": rows, "n_streams": args.streams, "chunk_bytes": args.chunk, "steps": args.steps}))
    return 0


def issue_rates_table(torch, dc):
    """dc_issue_rate for every instruction the library knows: time from one wavefront instruction to the next on a
    SIMD (eight wavefronts resident), and the class it falls into, the fastest instruction's time taken as two
    cycles.  The LDS reads (names beginning with ds_) share one LDS among a compute unit's four SIMDs: their cycles
    divided by four are LDS cycles a read.  One JSON line."""
    sink = torch.zeros(1024, dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    names = dc.issue_rate_names()
    ns = [min(dc.issue_rate(i, sink, 1024, stream) for _ in range(3)) for i in range(len(names))]
    fastest = min(ns)
    rows = []
    for n, t in zip(names, ns):
        row = {"instruction": n, "ns": round(t, 3), "cycles_if_the_fastest_takes_two": round(2 * t / fastest, 2)}
        if n.startswith("ds_"):
            row["lds_cycles_a_read"] = round(2 * t / fastest / 4, 2)
        rows.append(row)
    print(json.dumps({"instruction_issue": rows, "implied_clock_GHz": round(2 / fastest, 2),
                      "how": "32 copies of the instruction per loop turn on registers only, 1000 turns, 8 wavefronts per SIMD, "
                             "best of 3 timed launches"}))
    return 0


def workgroup_timeline(torch, dc, synth):
    """One traced launch (dc_decompress_chunks_traced) of the config-2 layer per storage rule, after 60 launches without
    the record: when the workgroups of coded and of raw chunks began, how long they took, how many were resident at
    once and how the coded ones were spread over the compute units.  Times in microseconds from the launch's first
    workgroup.  One JSON line."""
    p0 = dc.Params(65536, 256)
    q = build_layer("llama7b", 0, True, p0, dc, synth)["q"]
    n = (q.size + 65535) // 65536
    back_half = np.zeros(n, dtype=np.uint8)
    back_half[n - n // 2:] = 1
    cases = (("all coded", p0),
             ("half raw, lowest gain", dc.Params(65536, 256, dc.POLICY_RAW_FRACTION, 0.5)),
             ("half raw, the back half", dc.Params(65536, 256, dc.POLICY_RAW_MASK, 0.0, 0, back_half)),
             ("blocks of 2, last coded", dc.Params(65536, 256, dc.POLICY_BLOCK_LAST, 0.0, 2)),
             ("blocks of 3, last coded", dc.Params(65536, 256, dc.POLICY_BLOCK_LAST, 0.0, 3)),
             ("all raw", dc.Params(65536, 256, dc.POLICY_RAW_FRACTION, 1.0)))
    stream = torch.cuda.current_stream().cuda_stream
    want = up(torch, q)
    rows, ok = [], True

    def pct(x, *ps):
        return [round(float(np.percentile(x, p_)), 1) for p_ in ps]

    for label, p in cases:
        blob, table = dc.compress_chunks(q, p)
        blob_d, table_d = up(torch, blob), up(torch, table)
        dst = torch.zeros(q.size, dtype=torch.uint8, device="cuda")
        trace = torch.zeros(4 * n, dtype=torch.int64, device="cuda")
        for _ in range(60):
            dc.decompress_chunks(blob_d, blob.size, table_d, n, p, dst, q.size, stream)
        dst.zero_()
        for _ in range(3):
            dc.decompress_chunks_traced(blob_d, blob.size, table_d, n, p, dst, q.size, trace, stream)
        torch.cuda.synchronize()
        exact = bool(torch.equal(dst, want))
        ok = ok and exact
        t = trace.cpu().numpy().reshape(n, 4)
        t0 = t[:, 0].min()
        began, ended = (t[:, 0] - t0) / 100.0, (t[:, 1] - t0) / 100.0
        hw, xcd = t[:, 2] & 0xFFFFFFFF, (t[:, 2] >> 32) & 0xF
        unit = xcd * 256 + ((hw >> 13) & 7) * 16 + ((hw >> 8) & 0xF)  # compute unit: XCD, shader engine, unit
        row = {"stored": label, "exact": exact, "span_us": round(float(ended.max()), 1),
               "resident_at_once": int((began < 2.0).sum()), "compute_units_seen": int(len(np.unique(unit))),
               "xcd_is_workgroup_mod_8": bool(np.all(xcd == np.arange(n) % 8))}
        for name, kind in (("coded", dc.TRACE_DECODED), ("raw", dc.TRACE_COPIED)):
            m = t[:, 3] == kind
            if not m.any():
                continue
            dur = ended[m] - began[m]
            d = {"workgroups": int(m.sum()), "began_p50_p90_max": pct(began[m], 50, 90, 100),
                 "took_p10_p50_p90": pct(dur, 10, 50, 90), "last_ended": round(float(ended[m].max()), 1)}
            late = m & (began >= 2.0)
            if late.any():
                d["took_p50_when_begun_later"] = pct(ended[late] - began[late], 50)[0]
            if kind == dc.TRACE_DECODED:
                per_unit = np.bincount(unit[m], minlength=int(unit.max()) + 1)[np.unique(unit)]
                d["per_compute_unit_min_mean_max"] = [int(per_unit.min()), round(float(per_unit.mean()), 1), int(per_unit.max())]
            row[name] = d
        rows.append(row)
    print(json.dumps({"workgroup_timeline": {"workload": "config-2 layer, 3088 chunks of 64 KiB, 256 sub-streams; launch 63 of its run",
                                             "clock": "wall_clock64, 100 MHz", "launches": rows}, "exact": ok}))
    return 0 if ok else 1


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", choices=("config3", "config2"), default="config3",
                    help="what the timed steps decode: the whole model (the headline) or one compression-aware layer")
    ap.add_argument("--layers", type=int, default=32, help="config3: layers of the weight set (32 = the whole model)")
    ap.add_argument("--streams", type=int, default=256, help="sub-streams per chunk of the timed workload (32, 64, 128 or 256)")
    ap.add_argument("--chunk", type=int, default=65536, help="chunk size of the timed workload")
    ap.add_argument("--codec", choices=("huffman", "tans"), default="huffman",
                    help="coder of the timed launches (the headline is Huffman)")
    ap.add_argument("--tile", type=int, default=1, help="config2: decode this many copies of the layer in one launch")
    ap.add_argument("--first-chunks", type=int, default=0, metavar="K",
                    help="config2: decode only the first K chunks of the (tiled) layer in the timed launch")
    ap.add_argument("--fused", choices=("none", "dequant", "gemv"), default="none",
                    help="time only the whole-layer fused call of config 5 (for a profiler) and exit")
    ap.add_argument("--streaming-only", action="store_true",
                    help="only the layer-streaming loop on the config-2 layer (for a kernel trace) and exit")
    ap.add_argument("--mix-sweep", action="store_true",
                    help="only launches that mix raw and coded chunks: by share, by rule and by order, and exit")
    ap.add_argument("--compress-only", action="store_true",
                    help="only the compression on the GPU, both coders (for a profiler), and exit")
    ap.add_argument("--issue-rates", action="store_true",
                    help="only the issue rate of single vector-ALU instructions (dc_issue_rate), and exit")
    ap.add_argument("--wg-trace", action="store_true",
                    help="only one traced launch of the config-2 layer per storage rule: when its workgroups ran and where, and exit")
    ap.add_argument("--no-extras", action="store_true", help="skip the other workloads (extras.configs)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-side", action="store_true", help="skip the side timings of the headline launch")
    ap.add_argument("--alpha-sweep", action="store_true", help="host only: compression ratio against alpha and sparsity")
    ap.add_argument("--pair-stats", action="store_true", help="host only: two codes in one 11-bit look-up, how often")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build targets one GPU; decode shards by chunk range with no exchange step, "
              "but no multi-GPU path is built. Run with --gpus 1.", file=sys.stderr)
        return 2

    import paper_2502_15443_amd as dc
    import synth

    if args.alpha_sweep:
        return alpha_sweep(dc, synth)
    if args.pair_stats:
        return pair_stats(dc, synth)

    import torch

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    counters = load_counters(dc)

    if args.fused != "none":
        return fused_only(torch, dc, synth, args)
    if args.mix_sweep:
        return mix_sweep(torch, dc, synth)
    if args.wg_trace:
        return workgroup_timeline(torch, dc, synth)
    if args.issue_rates:
        return issue_rates_table(torch, dc)
    if args.compress_only:
        return compress_only(torch, dc, synth, args)
    if args.streaming_only:
        p2 = dc.Params(65536, 256)
        print(json.dumps(layer_streaming(torch, dc, synth, p2, build_layer("llama7b", 0, True, p2, dc, synth))))
        return 0

    out = {"metric": "decoded weight GB/s on 1 MI355X (and % HBM roofline); compression ratio", "value": None,
           "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": None,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic"}
    extras = {}
    if args.workload == "config3":
        head, sweep, sample, flat = run_config3(torch, dc, synth, args, counters)
        out.update(head)
        if sweep:
            extras["config3_chunk_size_sweep"] = sweep
        q1 = flat[:4096 * 4096].copy()  # layer 0, matrix 0: the config-1 matrix
        del flat
    else:
        head, sample, q1 = run_config2_headline(torch, dc, synth, args, counters)
        out.update(head)
    if not out["config"]["exact"]:
        print("bench.py: decoded bytes differ from the quantised input", file=sys.stderr)
        return 1

    if not args.no_extras:
        configs = {"config1": run_config1(torch, dc, q1)}
        c2, layer2 = run_config2(torch, dc, synth, args)
        configs["config2"] = c2
        configs["config4"] = {
            "on_the_config1_matrix": run_config4(torch, dc, q1, 32, "config 4 on the config-1 matrix (256 chunks, 32 sub-streams)"),
            "on_the_config2_layer": run_config4(torch, dc, layer2["q"], 256,
                                                "config 4 on the config-2 layer (3088 chunks, 256 sub-streams)")}
        configs["config5"] = run_config5(torch, dc, synth, counters)
        extras["configs"] = configs
        extras["layer_streaming"] = layer_streaming(torch, dc, synth, dc.Params(65536, 256), layer2)
        below = [f"config1 S={r['n_streams']}: {r['hbm_frac']}" for r in configs["config1"]["by_n_streams"] if r["hbm_frac"] < 0.5]
        below += [f"config2 S={r['n_streams']}: {r['hbm_frac']}" for r in configs["config2"]["by_n_streams"] if r["hbm_frac"] < 0.5]
        extras["below_half_of_the_hbm_roofline"] = below
    if extras:
        out["extras"] = extras
    if sample is not None and not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(sample)
    print(json.dumps(out))
    return 0


def run_config2_headline(torch, dc, synth, args, counters):
    """--workload config2: the timed steps decode one compression-aware layer (or --tile copies of it in one launch),
    buffers rotated through more than 640 MB.  For profiler runs and for the launch-shape measurements."""
    stream = torch.cuda.current_stream().cuda_stream
    S, C = args.streams, args.chunk
    codec = dc.CODEC_TANS if args.codec == "tans" else dc.CODEC_HUFFMAN
    params = dc.Params(C, S, codec=codec)
    layer = build_layer("llama7b", 0, True, params, dc, synth)
    blob, table, q = layer["blob"], layer["table"], layer["q"]
    if args.tile > 1:
        tables = []
        for i in range(args.tile):
            t = table.copy()
            t["off"] += i * blob.size
            tables.append(t)
        blob, table, q = np.tile(blob, args.tile), np.concatenate(tables), np.tile(q, args.tile)
    if args.first_chunks:
        # only the first K chunks of the (tiled) layer: the launch-shape measurements (how long K workgroups take)
        k = min(args.first_chunks, len(table))
        table, q = table[:k], q[:k * C]
    raw_bytes, n_chunks = q.size, len(table)
    ratio = raw_bytes / (blob.size + table.nbytes)
    nbuf = max(2, int(np.ceil(640e6 / (raw_bytes + blob.size))))
    blobs_d = [up(torch, blob) for _ in range(nbuf)]
    table_d = up(torch, table)
    dsts = [torch.empty(raw_bytes, dtype=torch.uint8, device="cuda") for _ in range(nbuf)]

    def decode(i):
        b = i % nbuf
        dc.decompress_chunks(blobs_d[b], blob.size, table_d, n_chunks, params, dsts[b], raw_bytes, stream)

    cold = time_each_launch(torch, decode, 21)
    ms, wall_ms = time_launches(torch, decode, args.steps, max(args.warmup, nbuf))
    want = up(torch, q)
    exact = all(bool(torch.equal(d, want)) for d in dsts)
    algo_bytes = raw_bytes + blob.size + table.nbytes
    achieved = algo_bytes / ms / 1e6
    kernel = f"dc_decode_kernel<{S},int8" + (",tANS>" if args.codec == "tans" else ">")
    tag = f"{kernel}|config2_layer_x{args.tile}_{C // 1024}KiB" + (f"_first{n_chunks}" if args.first_chunks else "")
    head = {
        "value": round(raw_bytes / ms / 1e6, 2), "ms_per_step": round(ms, 5),
        "config": {"workload": "config 2" + (f" x {args.tile} in one launch" if args.tile > 1 else "") +
                               ": Llama-7B-shaped decoder layer, 7 matrices, compression-aware INT8 (s=a^0.5), "
                               f"{C // 1024} KiB chunks, {S} sub-streams, all chunks {args.codec} coded (NOT the headline workload)",
                   "raw_bytes": raw_bytes, "chunk_bytes": C, "n_streams": S, "n_chunks": n_chunks, "blob_bytes": int(blob.size),
                   "compression_ratio": round(ratio, 5), "exact": exact, "buffers_rotated": nbuf},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": measured_traffic(counters, tag),
                     "kernel": kernel, "algorithmic_bytes_per_launch": int(algo_bytes), "avg_launch_ms": round(ms, 5)},
        "wall_ms_per_step": round(wall_ms, 5),
        "launch_index_against_duration": {"cold_launches_0_to_20_ms": [round(t, 4) for t in cold],
                                          "cold_mean_ms": round(float(np.mean(cold)), 4), "steady_ms": round(ms, 5)},
    }
    n_sample = min(n_chunks, 1024, layer["slices"][0]["n_chunks"])
    end = int(table["off"][n_sample - 1]) + int(table["comp_bytes"][n_sample - 1])
    sample = dict(blob=np.concatenate([blob[:end], blob[-64:]]), table=table[:n_sample], q=q[:n_sample * C].view(np.uint8),
                  C=C, S=S, codec=codec)
    q1, _, _ = dc.quantize_rows(synth.gen_weight(4096, 4096, synth.matrix_seed(0, 0)), None, 0.5, 1)
    return head, sample, q1.reshape(-1).view(np.uint8)


def fused_only(torch, dc, synth, args):
    """Only the whole-layer fused call of config 5, for a profiler: --fused dequant | gemv."""
    stream = torch.cuda.current_stream().cuda_stream
    params = dc.Params(65536, 256)
    l13 = build_layer("llama13b", 0, False, params, dc, synth)
    b = up(torch, l13["blob"])
    t = up(torch, l13["table"])
    raw, nb, nc = l13["q"].size, l13["blob"].size, len(l13["table"])
    scales = [torch.from_numpy(s).cuda() for s in l13["scales"]]
    offs = np.cumsum([0] + [sl["rows"] * sl["cols"] for sl in l13["slices"]])
    if args.fused == "dequant":
        out16 = torch.empty(raw, dtype=torch.int16, device="cuda")
        mats = [dc.Matrix(sl["k0"], sl["rows"], sl["cols"], scales[j], dst_bf16_dev=out16.data_ptr() + 2 * int(offs[j]),
                          dst_cap_elems=sl["rows"] * sl["cols"]) for j, sl in enumerate(l13["slices"])]
        fn = lambda i: dc.decompress_dequant_bf16_layer(b, nb, t, nc, params, mats, stream)  # noqa: E731
    else:
        xs = [torch.from_numpy(synth.gen_activation_bf16(sl["cols"], sl["seed"]).view(np.int16)).cuda() for sl in l13["slices"]]
        ys = [torch.empty(sl["rows"], dtype=torch.float32, device="cuda") for sl in l13["slices"]]
        ws_bytes = dc.decompress_gemv_workspace(nc)
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
        mats = [dc.Matrix(sl["k0"], sl["rows"], sl["cols"], scales[j], x_bf16_dev=xs[j], y_accum_dev=ys[j])
                for j, sl in enumerate(l13["slices"])]
        fn = lambda i: dc.decompress_gemv_layer(b, nb, t, nc, params, mats, ws, ws_bytes, stream)  # noqa: E731
    ms, _ = time_launches(torch, fn, args.steps, args.warmup)
    print(json.dumps({"fused": args.fused, "workload": "config 5 layer, one whole-layer call", "raw_bytes": int(raw),
                      "blob_bytes": int(nb), "n_chunks": nc, "ms": round(ms, 5), "weights_GBps": round(raw / ms / 1e6, 1)}))
    return 0


if __name__ == "__main__":
    sys.exit(main())
