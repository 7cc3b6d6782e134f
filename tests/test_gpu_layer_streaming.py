"""The runtime loop of the paper (Section 3.3, "Inference Process": the GPU decompresses the weights of the
layer that is needed next into a decompression buffer while inference computes on the layer before; Eqs. 11-12
model its latency) as a caller would write it with this library: two decompression buffers, the decode of
layer l+1 on a second stream (same priority) while the matrix-vector products of layer l read the other
buffer, events in both directions.  Layers have distinct weights.  After every layer the buffer must hold the
oracle-quantised bytes of that layer and every product must meet the tolerance against the fp64 reference;
the one-stream loop and the fused call must give the same."""
import numpy as np
import pytest

import oracle.codec as oc
import oracle.quant as oq
import paper_2502_15443_amd as dc
import synth
from tests.helpers import gemv_workspace, oracle_matrix

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

SHAPES = [(192, 1024), (320, 1024), (128, 2560)]  # three matrices a layer: 196608 + 327680 + 327680 bytes
N_LAYERS = 6


def dev(a: np.ndarray):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.uint8).reshape(-1)).cuda()


def make_layers(C, S, policy, f):
    """Per layer: matrices quantised by the oracle from the layer's own seeds, each compressed alone by the
    oracle, blobs appended (the layout of the whole-layer calls), activations per matrix."""
    layers = []
    for layer in range(N_LAYERS):
        qs, scales, blobs, tables, firsts, xs = [], [], [], [], [], []
        k = 0
        for m, (rows, cols) in enumerate(SHAPES):
            q, scale = oracle_matrix(rows, cols, synth.matrix_seed(10 + layer, m), m == 1)
            c = oc.compress(q, C, S, policy, f)
            t = c.table.copy()
            t["off"] += sum(b.size for b in blobs)
            qs.append(q), scales.append(scale), blobs.append(c.blob), tables.append(t), firsts.append(k)
            xs.append(synth.gen_activation_bf16(cols, 1000 * layer + m))
            k += c.n_chunks
        layers.append(dict(q=qs, scale=scales, blob=np.concatenate(blobs), table=np.concatenate(tables), first=firsts, x=xs,
                           flat=np.concatenate([q.view(np.uint8).ravel() for q in qs])))
    return layers


def check_products(y, layer, what):
    for m in range(len(SHAPES)):
        ref = oq.gemv_ref(layer["q"][m], layer["scale"][m], layer["x"][m])
        rms = float(np.sqrt(np.mean(ref ** 2)))
        got = y[m].cpu().numpy().astype(np.float64)
        assert (np.abs(got - ref) <= 1e-2 * np.abs(ref) + 1e-2 * rms).all(), (what, m)


@pytest.mark.parametrize("S,policy,f", [(256, oc.ALL_HUFF, 0.0), (64, oc.RAW_FRACTION, 0.4)])
def test_decode_of_the_next_layer_overlaps_the_products_of_this_one(S, policy, f):
    print(f"case layer streaming S={S} policy={policy} f={f}", flush=True)
    C = 16384
    p = dc.Params(C, S)
    layers = make_layers(C, S, policy, f)
    assert len({l["flat"].tobytes()[:64] for l in layers}) == N_LAYERS  # distinct weights
    n = layers[0]["flat"].size
    offs = np.cumsum([0] + [r * c for r, c in SHAPES])
    main, side = torch.cuda.current_stream(), torch.cuda.Stream()  # default priority both
    on_dev = [dict(blob=dev(l["blob"]), table=dev(l["table"]), scale=[torch.from_numpy(s).cuda() for s in l["scale"]],
                   x=[torch.from_numpy(x.view(np.int16)).cuda() for x in l["x"]]) for l in layers]
    bufs = [torch.full((n,), 0xEE, dtype=torch.uint8, device="cuda") for _ in range(2)]
    seen = [torch.zeros(n, dtype=torch.uint8, device="cuda") for _ in range(N_LAYERS)]  # the buffer as each layer's products saw it
    ys = [[torch.full((r,), 7.0, dtype=torch.float32, device="cuda") for r, _ in SHAPES] for _ in range(N_LAYERS)]

    def decode(i, st):
        d, l = on_dev[i], layers[i]
        dc.decompress_chunks(d["blob"], l["blob"].size, d["table"], len(l["table"]), p, bufs[i % 2], n, st.cuda_stream)

    def compute(i, st):
        d = on_dev[i]
        for m, (rows, cols) in enumerate(SHAPES):
            dc.gemv_i8(bufs[i % 2].data_ptr() + int(offs[m]), d["scale"][m], rows, cols, d["x"][m], ys[i][m], None, st.cuda_stream)
        with torch.cuda.stream(st):
            seen[i].copy_(bufs[i % 2])

    # decode of layer i on the side stream, products of layer i on the main stream
    side.wait_stream(main)
    done = [None, None]  # the products (and the snapshot) that last read each buffer
    for i in range(N_LAYERS):
        if done[i % 2] is not None:
            side.wait_event(done[i % 2])  # the buffer is free again
        decode(i, side)
        ready = torch.cuda.Event()
        ready.record(side)
        main.wait_event(ready)  # the products wait for their weights only
        compute(i, main)
        done[i % 2] = torch.cuda.Event()
        done[i % 2].record(main)
    main.wait_stream(side)
    torch.cuda.synchronize()
    for i, l in enumerate(layers):
        assert np.array_equal(seen[i].cpu().numpy(), l["flat"]), f"buffer of layer {i}"
        check_products(ys[i], l, f"two streams, layer {i}")
    overlapped = [[y.clone() for y in row] for row in ys]

    # the same on one stream: identical bits (same kernels on the same bytes)
    for row in ys:
        for y in row:
            y.fill_(7.0)
    for i in range(N_LAYERS):
        decode(i, main)
        compute(i, main)
    torch.cuda.synchronize()
    for i in range(N_LAYERS):
        for m in range(len(SHAPES)):
            assert torch.equal(ys[i][m], overlapped[i][m]), (i, m)

    # and through the fused call, which is what a caller should use on this GPU: nothing decoded reaches memory
    ws, ws_bytes = gemv_workspace(max(len(l["table"]) for l in layers))
    for i, l in enumerate(layers):
        d = on_dev[i]
        mats = [dc.Matrix(l["first"][m], r, c_, d["scale"][m], x_bf16_dev=d["x"][m], y_accum_dev=ys[i][m])
                for m, (r, c_) in enumerate(SHAPES)]
        for y in ys[i]:
            y.fill_(7.0)
        dc.decompress_gemv_layer(d["blob"], l["blob"].size, d["table"], len(l["table"]), p, mats, ws, ws_bytes, main.cuda_stream)
    torch.cuda.synchronize()
    for i, l in enumerate(layers):
        check_products(ys[i], l, f"fused, layer {i}")
