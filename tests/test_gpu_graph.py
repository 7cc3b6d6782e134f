"""The library's calls recorded into a HIP graph: every entry point of the decode path only enqueues kernels
on the caller's stream (no allocation, no host copy, no memset), so a capture holds the whole call.  Each
graph is replayed several times with eager work of the program and synchronisations in between, and every
replay is held to the same bar as the eager call: decoded bytes, bf16 values and the integer product
bit-exact against the oracle, the bf16 product inside its tolerance and within rounding of the eager
call's."""
import numpy as np
import pytest

import oracle.codec as oc
import oracle.quant as oq
import paper_2502_15443_amd as dc
import synth
from tests.helpers import gemv_workspace, oracle_matrix, weightlike_bytes

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def dev(a: np.ndarray):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.uint8).reshape(-1).copy()).cuda()


def capture(fn):
    """fn(stream handle) run once eagerly on a side stream (so that nothing is first touched inside the
    capture), then recorded."""
    cap = torch.cuda.Stream()
    cap.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(cap):
        fn(cap.cuda_stream)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=cap):
        fn(cap.cuda_stream)
    torch.cuda.synchronize()
    return g


@pytest.mark.parametrize("codec", [oc.HUFFMAN, oc.TANS])
def test_replays_of_a_recorded_decode(codec):
    C, S = 16384, 64
    n = 37 * C + 1234
    print(f"case graph decode codec={codec} n={n}", flush=True)
    data = weightlike_bytes(n, 4242)
    other = weightlike_bytes(n, 4243)
    c = oc.compress(data, C, S, oc.RAW_FRACTION, 0.2, codec=codec)
    c2 = oc.compress(other, C, S, codec=codec)
    p = dc.Params(C, S, codec=codec)
    blob_d, table_d = dev(c.blob), dev(c.table)
    blob2_d, table2_d = dev(c2.blob), dev(c2.table)
    dst = torch.zeros(n + 64, dtype=torch.uint8, device="cuda")

    g = capture(lambda st: dc.decompress_chunks(blob_d, c.blob.size, table_d, c.n_chunks, p, dst, n, st))
    for rep in range(4):
        # the program's own eager work between the replays: another blob into the same buffer, then a fill
        dc.decompress_chunks(blob2_d, c2.blob.size, table2_d, c2.n_chunks, p, dst, n,
                             torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        assert np.array_equal(dst.cpu().numpy()[:n], other)
        dst.fill_(0x5A)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        out = dst.cpu().numpy()
        assert np.array_equal(out[:n], data), f"replay {rep}"
        assert (out[n:] == 0x5A).all()


def test_replays_of_a_recorded_layer_of_fused_calls():
    """Three matrices of one blob: whole-layer dequantisation, whole-layer bf16 product (decode kernel that
    leaves ordered partial sums in the workspace, finishing kernel) and whole-layer integer product in one
    graph.  The bf16 product adds in a fixed order: every replay must give the bits of the eager call."""
    C, S = 16384, 128
    shapes = [(96, 2048), (160, 1024), (64, 4096)]
    print(f"case graph fused layer shapes={shapes}", flush=True)
    p = dc.Params(C, S)
    qs, scales, blobs, tables, firsts = [], [], [], [], []
    n_chunks = 0
    for m, (rows, cols) in enumerate(shapes):
        q, scale = oracle_matrix(rows, cols, synth.matrix_seed(3, m), m == 1)
        cm = oc.compress(q, C, S)
        t = cm.table.copy()
        t["off"] += sum(b.size for b in blobs)
        qs.append(q), scales.append(scale), blobs.append(cm.blob), tables.append(t), firsts.append(n_chunks)
        n_chunks += cm.n_chunks
    blob, table = np.concatenate(blobs), np.concatenate(tables)
    blob_d, table_d = dev(blob), dev(table)
    scale_d = [torch.from_numpy(s).cuda() for s in scales]
    xs = [synth.gen_activation_bf16(cols, 77 + m) for m, (_, cols) in enumerate(shapes)]
    xq = [oq.quantise_vector(np.random.default_rng(50 + m).standard_normal(cols).astype(np.float32))
          for m, (_, cols) in enumerate(shapes)]
    x_d = [torch.from_numpy(x.view(np.int16)).cuda() for x in xs]
    xq_d = [torch.from_numpy(v).cuda() for v, _ in xq]
    w16 = [torch.zeros(r * c_, dtype=torch.int16, device="cuda") for r, c_ in shapes]
    y = [torch.zeros(r, dtype=torch.float32, device="cuda") for r, _ in shapes]
    y8 = [torch.zeros(r, dtype=torch.float32, device="cuda") for r, _ in shapes]
    ws, ws_bytes = gemv_workspace(n_chunks)  # lives as long as the graph does

    def mats(kind):
        out = []
        for m, (rows, cols) in enumerate(shapes):
            mt = dc.Matrix(firsts[m], rows, cols, scale_d[m])
            if kind == "dequant":
                mt.dst_bf16_dev, mt.dst_cap_elems = w16[m], rows * cols
            elif kind == "gemv":
                mt.x_bf16_dev, mt.y_accum_dev = x_d[m], y[m]
            else:
                mt.x_i8_dev, mt.x_scale, mt.y_accum_dev = xq_d[m], float(xq[m][1]), y8[m]
            out.append(mt)
        return out

    def layer(st):
        dc.decompress_dequant_bf16_layer(blob_d, blob.size, table_d, n_chunks, p, mats("dequant"), st)
        dc.decompress_gemv_layer(blob_d, blob.size, table_d, n_chunks, p, mats("gemv"), ws, ws_bytes, st)
        dc.decompress_gemv_w8a8_layer(blob_d, blob.size, table_d, n_chunks, p, mats("w8a8"), st)

    layer(torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    eager_y = [t.cpu().numpy().copy() for t in y]
    for t in y:
        t.fill_(7)
    ws.fill_(0xFF)
    layer(torch.cuda.current_stream().cuda_stream)  # a second eager run: the same bits
    torch.cuda.synchronize()
    for m in range(len(shapes)):
        assert np.array_equal(y[m].cpu().numpy().view(np.uint32), eager_y[m].view(np.uint32)), m
    want_w = [oq.dequant_bf16(q, s) for q, s in zip(qs, scales)]
    want_y8 = [oq.gemv_w8a8(q, s, v, np.float32(xs_)) for q, s, (v, xs_) in zip(qs, scales, xq)]
    for m in range(len(shapes)):
        assert np.array_equal(w16[m].cpu().numpy().view(np.uint16).reshape(shapes[m]), want_w[m])
        assert np.array_equal(y8[m].cpu().numpy().view(np.uint32), want_y8[m].view(np.uint32))

    g = capture(layer)
    for rep in range(4):
        for t in w16 + y + y8:      # eager work between the replays: every output overwritten
            t.fill_(7)
        ws.fill_(0xFF)
        dc.decompress_gemv_layer(blob_d, blob.size, table_d, firsts[1], p, mats("gemv")[:1], ws, ws_bytes,
                                 torch.cuda.current_stream().cuda_stream)
        for t in y:
            t.add_(1.0)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for m in range(len(shapes)):
            assert np.array_equal(w16[m].cpu().numpy().view(np.uint16).reshape(shapes[m]), want_w[m]), (rep, m)
            assert np.array_equal(y8[m].cpu().numpy().view(np.uint32), want_y8[m].view(np.uint32)), (rep, m)
            got = y[m].cpu().numpy()
            ref = oq.gemv_ref(qs[m], scales[m], xs[m])
            assert np.all(np.abs(got - ref) <= 1e-2 * np.abs(ref) + 1e-2 * np.sqrt(np.mean(ref ** 2))), (rep, m)
            # every addition of the bf16 product has a fixed place in a fixed order: the bits of the eager call
            assert np.array_equal(got.view(np.uint32), eager_y[m].view(np.uint32)), (rep, m)
