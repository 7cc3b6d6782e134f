#!/usr/bin/env python3
"""Benchmark of the decode hot path on one MI355X.

A step is one pass of the hot path over one Llama-7B-shaped decoder layer (q/k/v/o 4096x4096,
gate/up 11008x4096, down 4096x11008; 202 375 168 int8 weights), compression-aware quantised
(per-input-channel rescale with s = a^0.5, a ~ LogNormal(0,1); per-row absmax INT8; |q| <= 1 pruned),
cut in 64 KiB chunks: one dc_decompress_chunks launch that decodes every chunk of the layer into one
buffer in HBM.  All inputs are resident in HBM before the timed region; buffers rotate through
distinct copies so that the 256 MiB last-level cache cannot serve them.

Prints one JSON line: decoded GB/s (value), the HBM roofline of the decode kernel, the CPU oracle
timed on the host cores, and extra rates (fused bf16 dequantisation, fused GEMV, raw-fraction sweep,
plain copy kernel) measured in the same run.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0

# HBM bytes per launch of the decode kernel on the headline workload, from the rocprofv3 counter runs
# summarised under profiles/ (FETCH_SIZE and WRITE_SIZE in KiB per dispatch, each scaled by what the
# same counter reads for the plain copy kernel: FETCH_SIZE x 2.000, WRITE_SIZE x 1.000).
MEASURED_TRAFFIC_KIB = {256: (74467.8, 197632.0), 128: (73533.3, 197632.0), 64: (73076.4, 197632.0)}


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
    return dict(blob=np.concatenate(blobs), table=np.concatenate(tables), q=np.concatenate(qs),
                scales=scales, slices=slices)


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


def time_each_launch(torch, fn, n, first):
    """Median and minimum duration (ms) of n launches of fn(), each between its own pair of HIP events."""
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
    torch.cuda.synchronize()
    for i, (e0, e1) in enumerate(pairs):
        e0.record()
        fn(first + i)
        e1.record()
    torch.cuda.synchronize()
    t = sorted(e0.elapsed_time(e1) for e0, e1 in pairs)
    return t[len(t) // 2], t[0]


def headline_side_timings(torch, dc, decode, blobs_d, blob, table_d, n_chunks, params, dsts, raw_bytes, first):
    """The headline launch seen three other ways; none of them is the headline."""
    med_ms, min_ms = time_each_launch(torch, decode, 30, first)
    # the same launch on one blob and one destination every time (no rotation through distinct copies)
    same_ms, _ = time_launches(torch, lambda i: decode(0), 30, 3)
    # launches issued alternately on two streams (each stream keeps its own blob and destination): the start of
    # one launch fills the compute units that the end of the other leaves idle
    side = torch.cuda.Stream()
    streams = [torch.cuda.current_stream(), side]

    def decode_on(i):
        b = i % 2
        dc.decompress_chunks(blobs_d[b], blob.size, table_d, n_chunks, params, dsts[b], raw_bytes, streams[b].cuda_stream)

    side.wait_stream(streams[0])
    for i in range(6):
        decode_on(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(100):
        decode_on(i)
    torch.cuda.synchronize()
    two_ms = (time.perf_counter() - t0) * 1e3 / 100
    return {
        "launch_ms_each_timed_alone": {"median": round(med_ms, 5), "min": round(min_ms, 5), "n": 30},
        "same_buffers_every_launch": {"ms": round(same_ms, 5), "decoded_GBps": round(raw_bytes / same_ms / 1e6, 1),
                                      "note": "no rotation: blob and destination may partly stay in the 256 MB "
                                              "memory-side cache; not the headline"},
        "two_streams_alternating": {"ms": round(two_ms, 5), "decoded_GBps": round(raw_bytes / two_ms / 1e6, 1),
                                    "note": "wall clock per launch with launches on two streams in turn; not the headline"},
    }


def layer_streaming(torch, dc, synth, params, n_layers=8, reps=10):
    """The paper's runtime loop (Section 3.3, case (b): everything in GPU memory) on the Llama-7B-shaped
    layer: per-layer latency of batch-1 inference (seven matrix-vector products a layer) with the
    weights (i) resident uncompressed, (ii) decoded into the decompression buffer and then used, on one
    stream, (iii) the same with the decode of layer l+1 on a second stream while layer l computes
    (two buffers), (iv) through the fused decode+product call, and (iii) again with part of the chunks
    stored raw.  Every layer uses the same weights (distinct buffers); times are wall-clock per layer."""
    S, C = params.n_streams, params.chunk_bytes

    def up(a):
        return torch.from_numpy(np.ascontiguousarray(a).view(np.uint8).reshape(-1)).cuda()

    side = torch.cuda.Stream()
    out = {"n_layers": n_layers, "n_streams": S}
    lay = build_layer("llama7b", 0, True, params, dc, synth)
    raw_bytes = lay["q"].size
    scales = [torch.from_numpy(s).cuda() for s in lay["scales"]]
    xs = [torch.from_numpy(synth.gen_activation_bf16(sl["cols"], sl["seed"]).view(np.int16)).cuda() for sl in lay["slices"]]
    ys = [torch.empty(sl["rows"], dtype=torch.float32, device="cuda") for sl in lay["slices"]]
    bufs = [torch.empty(raw_bytes, dtype=torch.uint8, device="cuda") for _ in range(2)]
    offs = np.cumsum([0] + [sl["rows"] * sl["cols"] for sl in lay["slices"]])
    graphs_used = []

    def compute(buf, st):
        for j, sl in enumerate(lay["slices"]):
            dc.gemv_i8(buf.data_ptr() + int(offs[j]), scales[j], sl["rows"], sl["cols"], xs[j], ys[j], None, st.cuda_stream)

    def wall(fn):
        """ms per layer of fn(stream), which enqueues n_layers layers.  The launches are recorded once into
        a HIP graph and replayed, so that the host's launch cost stays out of the per-layer time."""
        cap = torch.cuda.Stream()
        cap.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(cap):
            fn(cap)
        torch.cuda.synchronize()
        run = None
        try:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=cap):
                fn(cap)
            g.replay()
            torch.cuda.synchronize()
            run = g.replay
            graphs_used.append(True)
        except Exception:
            torch.cuda.synchronize()
            graphs_used.append(False)
            run = lambda: fn(torch.cuda.current_stream())
        t0 = time.perf_counter()
        for _ in range(reps):
            run()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / (reps * n_layers)

    def variant(l):
        blobs = [up(l["blob"]) for _ in range(2)]
        table = up(l["table"])
        nb, nc = l["blob"].size, len(l["table"])

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

        return blobs, table, wall(decode_only), wall(serial), wall(overlapped)

    blobs, table, d_ms, ser_ms, ovl_ms = variant(lay)
    # decoded weights are now in bufs: the resident case
    i_ms = wall(lambda main: [compute(bufs[i % 2], main) for i in range(n_layers)])

    mats = [dc.Matrix(sl["k0"], sl["rows"], sl["cols"], scales[j], x_bf16_dev=xs[j], y_accum_dev=ys[j])
            for j, sl in enumerate(lay["slices"])]

    ws_bytes = dc.decompress_gemv_workspace(len(lay["table"]))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")

    def fused(main):
        for i in range(n_layers):
            dc.decompress_gemv_layer(blobs[i % 2], lay["blob"].size, table, len(lay["table"]), params, mats,
                                     ws, ws_bytes, main.cuda_stream)

    f_ms = wall(fused)
    # the replayed launches must have produced what the eager calls produce
    y_fused = [y.clone() for y in ys]
    compute(bufs[1], torch.cuda.current_stream())
    torch.cuda.synchronize()
    ok = bool(torch.equal(bufs[1].cpu(), torch.from_numpy(lay["q"].view(np.uint8))))
    for yf, y in zip(y_fused, ys):
        ok = ok and bool(torch.allclose(yf, y, rtol=1e-3, atol=1e-3 * float(y.abs().max())))
    out["replayed_results_match_eager"] = ok
    out["ms_per_layer"] = {"resident_compute_I": round(i_ms, 4), "decode_D": round(d_ms, 4),
                           "decode_then_compute_one_stream": round(ser_ms, 4),
                           "decode_next_layer_on_second_stream": round(ovl_ms, 4), "fused_decode_product": round(f_ms, 4)}
    out["model_ms_per_layer"] = {"one_stream_D_plus_I": round(d_ms + i_ms, 4), "overlapped_max_D_I": round(max(d_ms, i_ms), 4)}
    out["overhead_vs_resident"] = {"one_stream": round(ser_ms / i_ms - 1, 3), "second_stream": round(ovl_ms / i_ms - 1, 3),
                                   "fused": round(f_ms / i_ms - 1, 3)}
    out["compression_ratio"] = round(raw_bytes / (lay["blob"].size + lay["table"].nbytes), 5)

    # The same loop in the paper's own arithmetic (Eq. 4: weights and activations both INT8): the product on
    # resident weights, and the fused decode + product.  Integer sums: the two must agree bit for bit.
    xq = []
    for sl in lay["slices"]:
        v, sc = dc.quantize_vector(np.random.default_rng(sl["seed"] & 0xFFFFFFFF).standard_normal(sl["cols"]).astype(np.float32))
        xq.append((torch.from_numpy(v).cuda(), sc))
    yw = [torch.empty(sl["rows"], dtype=torch.float32, device="cuda") for sl in lay["slices"]]

    def compute_w8a8(buf, st):
        for j, sl in enumerate(lay["slices"]):
            dc.gemv_w8a8(buf.data_ptr() + int(offs[j]), scales[j], sl["rows"], sl["cols"], xq[j][0], xq[j][1], yw[j], None,
                         st.cuda_stream)

    mats_w = [dc.Matrix(sl["k0"], sl["rows"], sl["cols"], scales[j], y_accum_dev=ys[j], x_i8_dev=xq[j][0], x_scale=xq[j][1])
              for j, sl in enumerate(lay["slices"])]

    def fused_w8a8(main):
        for i in range(n_layers):
            dc.decompress_gemv_w8a8_layer(blobs[i % 2], lay["blob"].size, table, len(lay["table"]), params, mats_w,
                                          main.cuda_stream)

    iw_ms = wall(lambda main: [compute_w8a8(bufs[i % 2], main) for i in range(n_layers)])
    fw_ms = wall(fused_w8a8)
    same = all(bool(torch.equal(a, b)) for a, b in zip(ys, yw))
    out["w8a8"] = {"ms_per_layer": {"resident_compute_I": round(iw_ms, 4), "fused_decode_product": round(fw_ms, 4)},
                   "overhead_vs_resident_fused": round(fw_ms / iw_ms - 1, 3),
                   "fused_weights_GBps": round(raw_bytes / fw_ms / 1e6, 1),
                   "fused_equals_resident_bit_for_bit": same}
    del blobs, table
    partial = []
    for f in (0.5, 0.8):
        pf = dc.Params(C, S, dc.POLICY_RAW_FRACTION, f)
        lf = build_layer("llama7b", 0, True, pf, dc, synth)
        _, _, dm, sm, om = variant(lf)
        partial.append({"raw_fraction": f, "compression_ratio": round(raw_bytes / (lf["blob"].size + lf["table"].nbytes), 5),
                        "decode_D": round(dm, 4), "one_stream": round(sm, 4), "second_stream": round(om, 4),
                        "overhead_vs_resident_second_stream": round(om / i_ms - 1, 3)})
    out["speed_adaptive"] = partial
    out["hip_graph_replay"] = all(graphs_used)
    return out


def full_model(torch, dc, synth, n_layers, sweep):
    """The 32-layer Llama-7B-shaped weight set (per-layer seeds, quantised without the rescale), every chunk
    decoded into one buffer by one launch, for each (chunk_bytes, n_streams) of `sweep`.  One JSON line.
    Not the headline: the weights take minutes to generate."""
    stream = torch.cuda.current_stream().cuda_stream
    t0 = time.perf_counter()
    qs = []
    for layer in range(n_layers):
        for m in synth.layer_specs("llama7b"):
            seed = synth.matrix_seed(layer, m.index)
            q, _, _ = dc.quantize_rows(synth.gen_weight(m.rows, m.cols, seed), None, 0.5, 1)
            qs.append(q.reshape(-1))
    gen_s = time.perf_counter() - t0
    raw_bytes = int(sum(q.size for q in qs))
    flat = torch.from_numpy(np.concatenate(qs).view(np.uint8))
    dst = torch.empty(raw_bytes, dtype=torch.uint8, device="cuda")
    rows = []
    for C, S in sweep:
        p = dc.Params(C, S)
        blobs, tables, off = [], [], 0
        t0 = time.perf_counter()
        for q in qs:
            b, t = dc.compress_chunks(q, p)
            t = t.copy()
            t["off"] += off
            off += b.size
            blobs.append(b)
            tables.append(t)
        comp_s = time.perf_counter() - t0
        blob, table = np.concatenate(blobs), np.concatenate(tables)
        del blobs, tables
        blob_d = torch.from_numpy(blob).cuda()
        table_d = torch.from_numpy(table.view(np.uint8)).cuda()
        ms, _ = time_launches(
            torch, lambda i: dc.decompress_chunks(blob_d, blob.size, table_d, len(table), p, dst, raw_bytes, stream), 10, 2)
        exact = bool(torch.equal(dst.cpu(), flat))
        rows.append({"chunk_bytes": C, "n_streams": S, "n_chunks": len(table),
                     "compression_ratio": round(raw_bytes / (blob.size + table.nbytes), 5), "ms": round(ms, 4),
                     "decoded_GBps": round(raw_bytes / ms / 1e6, 1),
                     "hbm_frac": round((raw_bytes + blob.size + table.nbytes) / ms / 1e6 / HBM_PEAK_GBPS, 4),
                     "exact": exact, "host_compress_s": round(comp_s, 1)})
        del blob_d, table_d, blob, table
    print(json.dumps({"workload": f"{n_layers} Llama-7B-shaped layers, distinct per-layer seeds, per-row INT8 without "
                                  "rescale, one launch into one buffer", "raw_bytes": raw_bytes,
                      "generate_and_quantise_s": round(gen_s, 1), "sweep": rows}))
    return 0 if all(r["exact"] for r in rows) else 1


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--streams", type=int, default=int(os.environ.get("DC_BENCH_STREAMS", "256")),
                    help="sub-streams per chunk (32, 64, 128 or 256)")
    ap.add_argument("--chunk", type=int, default=65536)
    ap.add_argument("--codec", choices=("huffman", "tans"), default="huffman",
                    help="coder of the timed launches (the headline is Huffman; tans times the second coder instead)")
    ap.add_argument("--tile", type=int, default=1,
                    help="decode this many copies of the layer in one launch (input-size scaling; not the headline)")
    ap.add_argument("--full-model", type=int, default=0, metavar="LAYERS",
                    help="instead of the headline: decode LAYERS distinct layers (32 = the whole model) in one launch, "
                         "sweeping the chunk size")
    ap.add_argument("--no-extras", action="store_true", help="skip fused/raw-fraction/copy side measurements")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-side", action="store_true",
                    help="skip the side timings of the headline launch (timed alone, same buffers, two streams), "
                         "so that a profiler sees the timed launches only")
    args = ap.parse_args()
    if args.codec == "tans":
        args.no_extras = True  # the side measurements (fused calls, device compressor) take Huffman blobs
    if args.gpus != 1:
        print("bench.py: this build targets one GPU; decode shards by chunk range with no exchange step, "
              "but no multi-GPU path is built. Run with --gpus 1.", file=sys.stderr)
        return 2

    import torch

    import paper_2502_15443_amd as dc
    import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    if args.full_model:
        return full_model(torch, dc, synth, args.full_model,
                          [(65536, 64), (65536, 256), (16384, 64), (262144, 64), (262144, 256)])
    stream = torch.cuda.current_stream().cuda_stream
    S, C = args.streams, args.chunk
    params = dc.Params(C, S, codec=dc.CODEC_TANS if args.codec == "tans" else dc.CODEC_HUFFMAN)

    layer = build_layer("llama7b", 0, True, params, dc, synth)
    blob, table, q = layer["blob"], layer["table"], layer["q"]
    if args.tile > 1:
        tables = []
        for i in range(args.tile):
            t = table.copy()
            t["off"] += i * blob.size
            tables.append(t)
        blob, table, q = np.tile(blob, args.tile), np.concatenate(tables), np.tile(q, args.tile)
    raw_bytes, n_chunks = q.size, len(table)
    ratio = raw_bytes / (blob.size + table.nbytes)

    def up(a):
        return torch.from_numpy(np.ascontiguousarray(a).view(np.uint8).reshape(-1)).cuda()

    nbuf = max(2, int(np.ceil(640e6 / (raw_bytes + blob.size))))
    blobs_d = [up(blob) for _ in range(nbuf)]
    table_d = up(table)
    dsts = [torch.empty(raw_bytes, dtype=torch.uint8, device="cuda") for _ in range(nbuf)]

    def decode(i):
        b = i % nbuf
        dc.decompress_chunks(blobs_d[b], blob.size, table_d, n_chunks, params, dsts[b], raw_bytes, stream)

    ms, wall_ms = time_launches(torch, decode, args.steps, args.warmup)
    side_timings = None
    if not args.no_side:
        side_timings = headline_side_timings(torch, dc, decode, blobs_d, blob, table_d, n_chunks, params, dsts, raw_bytes,
                                             args.warmup + args.steps)
    ok = all(bool(torch.equal(d.cpu(), torch.from_numpy(q.view(np.uint8)))) for d in dsts)
    if not ok:
        print("bench.py: decoded bytes differ from the quantised input", file=sys.stderr)
        return 1
    decoded_gbps = raw_bytes / ms / 1e6
    algo_bytes = raw_bytes + blob.size + table.nbytes
    achieved = algo_bytes / ms / 1e6

    traffic = None
    if S in MEASURED_TRAFFIC_KIB and args.tile == 1 and C == 65536 and args.codec == "huffman":
        f_kib, w_kib = MEASURED_TRAFFIC_KIB[S]
        traffic = int((2.0 * f_kib + 1.0 * w_kib) * 1024)

    out = {
        "metric": "decoded weight GB/s on 1 MI355X (and % HBM roofline); compression ratio",
        "value": round(decoded_gbps, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u8",
        "data": "synthetic",
        "config": {"workload": "llama7b decoder layer, 7 matrices, compression-aware INT8 (s=a^0.5), 64 KiB chunks, "
                               + ("all chunks Huffman coded" if args.codec == "huffman" else "all chunks tANS coded"),
                   "raw_bytes": raw_bytes, "chunk_bytes": C,
                   "n_streams": S, "n_chunks": n_chunks, "blob_bytes": int(blob.size),
                   "compression_ratio": round(ratio, 5), "buffers_rotated": nbuf},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
                     "kernel": f"dc_decode_kernel<{S},int8" + (",tANS>" if args.codec == "tans" else ">"),
                     "algorithmic_bytes_per_launch": int(algo_bytes),
                     "avg_launch_ms": round(ms, 5)},
        "wall_ms_per_step": round(wall_ms, 5),
        "roofline_limited_decoded_gbps": round(HBM_PEAK_GBPS / (1 + 1 / ratio), 1),
    }

    if side_timings:
        out.update(side_timings)
    if not args.no_extras:
        extras = {}
        # plain copy kernel: the achievable-bandwidth line
        n_copy = raw_bytes // 16 * 16
        cms, _ = time_launches(torch, lambda i: dc.device_copy(dsts[i % nbuf], dsts[(i + 1) % nbuf], n_copy, stream),
                               50, 5)
        extras["copy_kernel_GBps_read_plus_write"] = round(2 * n_copy / cms / 1e6, 1)
        extras["decode_frac_of_copy_bandwidth"] = round(achieved / (2 * n_copy / cms / 1e6), 4)

        # sub-stream count: compression ratio against parallelism, same layer
        sweep_s = []
        for s2 in (64, 128, 256):
            if s2 == S:
                sweep_s.append({"n_streams": s2, "decoded_GBps": round(decoded_gbps, 1), "compression_ratio": round(ratio, 5)})
                continue
            p2 = dc.Params(C, s2)
            l2 = build_layer("llama7b", 0, True, p2, dc, synth)
            b2 = [up(l2["blob"]) for _ in range(nbuf)]
            t2 = up(l2["table"])
            ms2, _ = time_launches(
                torch, lambda i: dc.decompress_chunks(b2[i % nbuf], l2["blob"].size, t2, len(l2["table"]), p2,
                                                      dsts[i % nbuf], raw_bytes, stream), 50, 5)
            good = bool(torch.equal(dsts[(50 + 5 - 1) % nbuf].cpu(), torch.from_numpy(l2["q"].view(np.uint8))))
            sweep_s.append({"n_streams": s2, "decoded_GBps": round(raw_bytes / ms2 / 1e6, 1),
                            "compression_ratio": round(raw_bytes / (l2["blob"].size + l2["table"].nbytes), 5),
                            "exact": good})
            del b2, t2, l2
        extras["n_streams_sweep"] = sweep_s

        # the container's second coder (tANS, 2048 states; the paper settles on ANS in Section 4.2) on the same
        # layer: at the headline's shape, and with few streams and big chunks, where its shorter streams count
        tans_rows = []
        for c2, s2 in ((C, S), (262144, 64), (262144, 256)):
            row = {"chunk_bytes": c2, "n_streams": s2}
            for name, codec in (("huffman", dc.CODEC_HUFFMAN), ("tans", dc.CODEC_TANS)):
                if codec == dc.CODEC_HUFFMAN and (c2, s2) == (C, S):
                    row[name] = {"decoded_GBps": round(decoded_gbps, 1), "compression_ratio": round(ratio, 5)}
                    continue
                p2 = dc.Params(c2, s2, codec=codec)
                l2 = build_layer("llama7b", 0, True, p2, dc, synth)
                b2 = [up(l2["blob"]) for _ in range(nbuf)]
                t2 = up(l2["table"])
                ms2, _ = time_launches(
                    torch, lambda i: dc.decompress_chunks(b2[i % nbuf], l2["blob"].size, t2, len(l2["table"]), p2,
                                                          dsts[i % nbuf], raw_bytes, stream), 200, 20)
                good = bool(torch.equal(dsts[(200 + 20 - 1) % nbuf].cpu(), torch.from_numpy(l2["q"].view(np.uint8))))
                row[name] = {"decoded_GBps": round(raw_bytes / ms2 / 1e6, 1),
                             "compression_ratio": round(raw_bytes / (l2["blob"].size + l2["table"].nbytes), 5),
                             "exact": good}
                del b2, t2, l2
            tans_rows.append(row)
        extras["tans_against_huffman"] = tans_rows

        # fused paths on the Llama-13B-shaped layer (hidden 5120, FFN 13824, quantised without rescale),
        # one call per matrix as the entry points take one matrix
        l13 = build_layer("llama13b", 0, False, params, dc, synth)
        b13 = [up(l13["blob"]) for _ in range(2)]
        t13 = up(l13["table"])
        raw13, blob13 = l13["q"].size, l13["blob"].size
        scales_d = [torch.from_numpy(s).cuda() for s in l13["scales"]]
        big = max(sl["rows"] * sl["cols"] for sl in l13["slices"])
        out16 = [torch.empty(big, dtype=torch.int16, device="cuda") for _ in range(2)]

        def dequant(i):
            for j, sl in enumerate(l13["slices"]):
                dc.decompress_dequant_bf16(b13[i % 2], blob13, t13.data_ptr() + 16 * sl["k0"], sl["n_chunks"], params,
                                           scales_d[j], sl["rows"], sl["cols"], out16[(i + j) % 2], big, stream)

        dms, _ = time_launches(torch, dequant, 30, 3)
        # fused batch-1 GEMV
        xs = [torch.from_numpy(synth.gen_activation_bf16(sl["cols"], sl["seed"]).view(np.int16)).cuda()
              for sl in l13["slices"]]
        ys = [torch.empty(sl["rows"], dtype=torch.float32, device="cuda") for sl in l13["slices"]]

        ws13_bytes = dc.decompress_gemv_workspace(len(l13["table"]))
        ws13 = torch.empty(ws13_bytes, dtype=torch.uint8, device="cuda")

        def gemv(i):
            for j, sl in enumerate(l13["slices"]):
                dc.decompress_gemv(b13[i % 2], blob13, t13.data_ptr() + 16 * sl["k0"], sl["n_chunks"], params,
                                   scales_d[j], sl["rows"], sl["cols"], xs[j], ys[j], None, ws13, ws13_bytes, stream)

        gms, _ = time_launches(torch, gemv, 30, 3)
        # the same through the whole-layer calls: one launch over all 4840 chunks
        mats_b = [dc.Matrix(sl["k0"], sl["rows"], sl["cols"], scales_d[j], dst_bf16_dev=None, dst_cap_elems=sl["rows"] * sl["cols"])
                  for j, sl in enumerate(l13["slices"])]
        layer16 = [torch.empty(raw13, dtype=torch.int16, device="cuda") for _ in range(2)]
        offs13 = np.cumsum([0] + [sl["rows"] * sl["cols"] for sl in l13["slices"]])

        def dequant_layer(i):
            for j, m in enumerate(mats_b):
                m.dst_bf16_dev = layer16[i % 2].data_ptr() + 2 * int(offs13[j])
            dc.decompress_dequant_bf16_layer(b13[i % 2], blob13, t13, len(l13["table"]), params, mats_b, stream)

        dlms, _ = time_launches(torch, dequant_layer, 30, 3)
        mats_g = [dc.Matrix(sl["k0"], sl["rows"], sl["cols"], scales_d[j], x_bf16_dev=xs[j], y_accum_dev=ys[j])
                  for j, sl in enumerate(l13["slices"])]
        glms, _ = time_launches(
            torch, lambda i: dc.decompress_gemv_layer(b13[i % 2], blob13, t13, len(l13["table"]), params, mats_g,
                                                      ws13, ws13_bytes, stream), 30, 3)
        del layer16
        extras["fused_llama13b_layer"] = {
            "whole_layer_call": {"dequant_bf16_int8_GBps": round(raw13 / dlms / 1e6, 1),
                                 "dequant_bf16_hbm_frac": round((blob13 + 2 * raw13) / dlms / 1e6 / HBM_PEAK_GBPS, 4),
                                 "gemv_weights_GBps": round(raw13 / glms / 1e6, 1),
                                 "gemv_hbm_frac": round(blob13 / glms / 1e6 / HBM_PEAK_GBPS, 4)},
            "raw_bytes": int(raw13), "n_chunks": len(l13["table"]),
            "compression_ratio": round(raw13 / (blob13 + l13["table"].nbytes), 5),
            "dequant_bf16_int8_GBps": round(raw13 / dms / 1e6, 1),
            "dequant_bf16_hbm_frac": round((blob13 + 2 * raw13) / dms / 1e6 / HBM_PEAK_GBPS, 4),
            "gemv_weights_GBps": round(raw13 / gms / 1e6, 1),
            "gemv_hbm_frac": round(blob13 / gms / 1e6 / HBM_PEAK_GBPS, 4),
            "calls_per_pass": len(l13["slices"])}
        del b13, t13, out16

        # speed-adaptive partial compression: fraction f of chunks raw (lowest Huffman gain first)
        sweep = []
        for f in (0.0, 0.25, 0.5, 0.75, 1.0):
            pf = dc.Params(C, S, dc.POLICY_RAW_FRACTION, f)
            lf = build_layer("llama7b", 0, True, pf, dc, synth)
            bd = [up(lf["blob"]) for _ in range(nbuf)]
            td = up(lf["table"])
            nb, nc = lf["q"].size, len(lf["table"])
            fms, _ = time_launches(
                torch, lambda i: dc.decompress_chunks(bd[i % nbuf], lf["blob"].size, td, nc, pf, dsts[i % nbuf], nb, stream),
                50, 5)
            good = bool(torch.equal(dsts[(50 + 5 - 1) % nbuf][:nb].cpu(), torch.from_numpy(lf["q"].view(np.uint8))))
            sweep.append({"raw_fraction": f, "decoded_GBps": round(nb / fms / 1e6, 1),
                          "compression_ratio": round(nb / (lf["blob"].size + lf["table"].nbytes), 5),
                          "hbm_frac": round((nb + lf["blob"].size) / fms / 1e6 / HBM_PEAK_GBPS, 4), "exact": good})
            del bd, td
        # Section 3.3's throughput reasoning for a mix: time per byte = (1-f)/D_coded + f/D_raw
        d0, d1 = sweep[0]["decoded_GBps"], sweep[-1]["decoded_GBps"]
        for r in sweep:
            f = r["raw_fraction"]
            r["model_GBps"] = round(1.0 / ((1 - f) / d0 + f / d1), 1)
        extras["raw_fraction_sweep"] = sweep
        # The paper's own rule (Section 3.3: of every block of N chunks only the last is compressed) beside the
        # gain-ranked rule at the same share of raw chunks, 1 - 1/N
        pareto = []
        for n_block in (2, 4, 5):
            row = {"block_chunks": n_block, "raw_fraction": round(1 - 1 / n_block, 4)}
            for name, pf in (("positional", dc.Params(C, S, dc.POLICY_BLOCK_LAST, 0.0, n_block)),
                             ("gain_ranked", dc.Params(C, S, dc.POLICY_RAW_FRACTION, 1 - 1 / n_block))):
                lf = build_layer("llama7b", 0, True, pf, dc, synth)
                bd = [up(lf["blob"]) for _ in range(nbuf)]
                td = up(lf["table"])
                nb, nc = lf["q"].size, len(lf["table"])
                fms, _ = time_launches(
                    torch, lambda i: dc.decompress_chunks(bd[i % nbuf], lf["blob"].size, td, nc, pf, dsts[i % nbuf], nb,
                                                          stream), 50, 5)
                good = bool(torch.equal(dsts[(50 + 5 - 1) % nbuf][:nb].cpu(), torch.from_numpy(lf["q"].view(np.uint8))))
                is_raw = (lf["table"]["raw_bytes_flags"] >> 31) & 1
                row[name] = {"compression_ratio": round(nb / (lf["blob"].size + lf["table"].nbytes), 5),
                             "decoded_GBps": round(nb / fms / 1e6, 1), "raw_chunks": int(is_raw.sum()), "exact": good}
                del bd, td
            pareto.append(row)
        extras["positional_rule_against_gain_ranked"] = pareto
        # compression of the same layer on the GPU (Section 4.2 reports compression speed as well)
        q_d = up(q)
        cap_c, nc_c = dc.compress_bound(raw_bytes, params)
        blob_c = torch.empty(cap_c, dtype=torch.uint8, device="cuda")
        table_c = torch.empty(nc_c * 16, dtype=torch.uint8, device="cuda")
        ws_n = dc.compress_chunks_dev_workspace(raw_bytes, params)
        ws_c = torch.empty(ws_n, dtype=torch.uint8, device="cuda")
        res_c = torch.zeros(2, dtype=torch.int64, device="cuda")
        cms2, _ = time_launches(
            torch, lambda i: dc.compress_chunks_dev(q_d, raw_bytes, params, blob_c, cap_c, table_c, nc_c, ws_c, ws_n,
                                                    res_c, stream), 20, 3)
        used_c = int(res_c.cpu()[0])
        # one layer is one matrix set compressed in one go here; bench's blob is per matrix, so compare sizes only
        extras["compress_on_gpu"] = {"GBps": round(raw_bytes / cms2 / 1e6, 1), "ms": round(cms2, 4),
                                     "blob_bytes": used_c, "workspace_bytes": ws_n}
        t0 = time.perf_counter()
        dc.compress_chunks(q, params)
        extras["compress_on_host"] = {"GBps": round(raw_bytes / (time.perf_counter() - t0) / 1e9, 3),
                                      "threads": os.cpu_count()}
        del blob_c, table_c, ws_c
        # the same with the second coder
        pt = dc.Params(C, S, codec=dc.CODEC_TANS)
        cap_t, nc_t = dc.compress_bound(raw_bytes, pt)
        blob_t = torch.empty(cap_t, dtype=torch.uint8, device="cuda")
        table_t = torch.empty(nc_t * 16, dtype=torch.uint8, device="cuda")
        ws_tn = dc.compress_chunks_dev_workspace(raw_bytes, pt)
        ws_t = torch.empty(ws_tn, dtype=torch.uint8, device="cuda")
        tms, _ = time_launches(
            torch, lambda i: dc.compress_chunks_dev(q_d, raw_bytes, pt, blob_t, cap_t, table_t, nc_t, ws_t, ws_tn,
                                                    res_c, stream), 20, 3)
        extras["compress_on_gpu_tans"] = {"GBps": round(raw_bytes / tms / 1e6, 1), "ms": round(tms, 4),
                                          "blob_bytes": int(res_c.cpu()[0]), "workspace_bytes": ws_tn}
        del q_d, blob_t, table_t, ws_t
        extras["layer_streaming"] = layer_streaming(torch, dc, synth, params)
        out["extras"] = extras

    if not args.no_cpu:
        import oracle.codec as oc

        threads = min(os.cpu_count() or 1, 16)
        n_sample = min(n_chunks, 1024)  # first 64 MiB of the layer
        sample_raw = min(raw_bytes, n_sample * C)
        t0 = time.perf_counter()
        reps = 0
        while True:
            ref = oc.decompress(blob, table[:n_sample], C, S, sample_raw, threads=threads, codec=params.codec)
            reps += 1
            if time.perf_counter() - t0 > 1.5 and reps >= 3:
                break
        dt = (time.perf_counter() - t0) / reps
        assert np.array_equal(ref, q[:sample_raw].view(np.uint8))
        # one thread, and the oracle's encoder, on the first 128 chunks
        n_small = min(128, layer["slices"][0]["n_chunks"])  # inside the first matrix, whose blob the library made alone
        small_raw = min(raw_bytes, n_small * C)
        t0 = time.perf_counter()
        oc.decompress(blob, table[:n_small], C, S, small_raw, threads=1, codec=params.codec)
        one_thread = small_raw / (time.perf_counter() - t0) / 1e9
        t0 = time.perf_counter()
        enc = oc.compress(q[:small_raw], C, S, threads=threads, codec=params.codec)
        encode = small_raw / (time.perf_counter() - t0) / 1e9
        assert np.array_equal(enc.blob[:-64], blob[:int(table["off"][n_small - 1]) + int(table["comp_bytes"][n_small - 1])])
        out["cpu_baseline"] = {"value": round(sample_raw / dt / 1e9, 3), "unit": "GB/s", "cores": threads,
                               "kind": "oracle",
                               "sample": f"first {n_sample} chunks ({sample_raw} decoded bytes) of the same blob, "
                                         f"{reps} passes, bit-serial C oracle, chunk range split over {threads} threads",
                               "one_thread_GBps": round(one_thread, 4),
                               "encode_GBps": round(encode, 4),
                               "encode_sample": f"first {n_small} chunks compressed by the oracle on {threads} threads; "
                                                "its blob equals the library's"}

    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
