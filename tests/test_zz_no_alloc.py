"""dc_compress_chunks_dev_static, the compression call that allocates nothing (its workspace is a fixed
array in device memory), against dc_compress_chunks_dev through the C ABI: blob, chunk table and result
words must be the same bytes.  Two calls in a row share the array; the second has the smaller input."""
import numpy as np
import pytest

import paper_2502_15443_amd as dc
from tests.helpers import weightlike_bytes

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def run_both(data: np.ndarray, params):
    """(blob, table, result words) of the workspace call and of the static call on the same input."""
    n = data.size
    st = torch.cuda.current_stream().cuda_stream
    src = torch.from_numpy(np.ascontiguousarray(data).view(np.uint8).reshape(-1)).cuda()
    cap, nc = dc.compress_bound(n, params)
    outs = []
    for static in (False, True):
        blob_d = torch.full((cap + 64,), 0xEE, dtype=torch.uint8, device="cuda")
        table_d = torch.full((nc * 16,), 0xEE, dtype=torch.uint8, device="cuda")
        res = torch.full((2,), -1, dtype=torch.int64, device="cuda")
        if static:
            dc.compress_chunks_dev_static(src, n, params, blob_d, cap, table_d, nc, res, st)
        else:
            ws_bytes = dc.compress_chunks_dev_workspace(n, params)
            ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
            dc.compress_chunks_dev(src, n, params, blob_d, cap, table_d, nc, ws, ws_bytes, res, st)
        torch.cuda.synchronize()
        r = res.cpu().numpy().view(np.uint64)
        assert (blob_d[cap:].cpu().numpy() == 0xEE).all()
        used = int(r[0])
        outs.append((blob_d[:used].cpu().numpy(), table_d.cpu().numpy(), used, int(r[1])))
    return outs


@pytest.mark.parametrize("codec,S", [(dc.CODEC_HUFFMAN, 256), (dc.CODEC_HUFFMAN, 32), (dc.CODEC_TANS, 64)])
def test_static_workspace_call_equals_workspace_call_twice_in_a_row(codec, S):
    C = 16384
    first = weightlike_bytes(37 * C + 1234, 71 + S)
    second = weightlike_bytes(5 * C + 77, 72 + S)  # smaller: the array still holds the first call's figures
    for i, data in enumerate((first, second)):
        print(f"case static compress codec={codec} S={S} call={i} n={data.size}", flush=True)
        p = dc.Params(C, S, dc.POLICY_RAW_FRACTION, 0.25, codec=codec)
        (blob_w, table_w, used_w, st_w), (blob_s, table_s, used_s, st_s) = run_both(data, p)
        assert st_w == 0 and st_s == 0 and used_w == used_s
        assert np.array_equal(table_w, table_s)
        assert np.array_equal(blob_w, blob_s)
        dc.validate(blob_s, table_s.view(dc.CHUNK_DTYPE), p)


def test_static_workspace_call_refuses_what_the_array_cannot_serve():
    C = 65536
    p = dc.Params(C, 256)
    n = 20000 * C  # about 25 MB of workspace: more than the fixed array
    assert dc.compress_chunks_dev_workspace(n, p) > dc.STATIC_SCRATCH_BYTES
    dummy = torch.zeros(64, dtype=torch.uint8, device="cuda")
    with pytest.raises(dc.DCError) as e:
        dc.compress_chunks_dev_static(dummy, n, p, dummy, 64, dummy, 20000, dummy, torch.cuda.current_stream().cuda_stream)
    assert e.value.code == -2
