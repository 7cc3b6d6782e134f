"""The traced form of the decode launch: same bytes as the plain call, and a record per workgroup that agrees
with the chunk table."""
import numpy as np
import pytest

from helpers import weightlike_bytes

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2502_15443_amd as dc
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    torch.cuda.set_device(0)
    return torch, dc


def _up(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.uint8).reshape(-1)).cuda()


@pytest.mark.parametrize("policy", ["coded", "every third coded", "damaged entry"])
def test_traced_launch_decodes_the_same_bytes_and_records_every_workgroup(env, policy):
    torch, dc = env
    chunk = 4096
    q = weightlike_bytes(300 * chunk + 1000, 11)
    p = dc.Params(chunk, 256) if policy != "every third coded" else dc.Params(chunk, 256, dc.POLICY_BLOCK_LAST, 0.0, 3)
    blob, table = dc.compress_chunks(q, p)
    n = len(table)
    if policy == "damaged entry":
        table = table.copy()
        table["off"][5] += 8  # not a multiple of 16: the kernel leaves chunk 5 alone
    stream = torch.cuda.current_stream().cuda_stream
    blob_d, table_d = _up(torch, blob), _up(torch, table)
    plain = torch.full((q.size,), 0xA5, dtype=torch.uint8, device="cuda")
    traced = torch.full((q.size,), 0xA5, dtype=torch.uint8, device="cuda")
    trace = torch.full((4 * n,), -1, dtype=torch.int64, device="cuda")
    dc.decompress_chunks(blob_d, blob.size, table_d, n, p, plain, q.size, stream)
    dc.decompress_chunks_traced(blob_d, blob.size, table_d, n, p, traced, q.size, trace, stream)
    torch.cuda.synchronize()
    assert torch.equal(plain, traced)
    if policy != "damaged entry":
        assert torch.equal(traced, _up(torch, q))
    t = trace.cpu().numpy().reshape(n, 4)
    assert (t[:, 1] >= t[:, 0]).all() and (t[:, 0] > 0).all()
    assert ((t[:, 2] >> 32) & 0xF).max() < 8
    want = np.where((table["raw_bytes_flags"] >> 31) & 1, dc.TRACE_COPIED, dc.TRACE_DECODED)
    if policy == "damaged entry":
        want[5] = dc.TRACE_SKIPPED
    assert np.array_equal(t[:, 3], want)
    # 100 MHz clock: a launch of 300 small chunks is over within a few milliseconds
    assert (t[:, 1].max() - t[:, 0].min()) < 100 * 5000


def test_traced_launch_is_for_huffman_at_256_sub_streams(env):
    torch, dc = env
    q = weightlike_bytes(8 * 4096, 12)
    for p in (dc.Params(4096, 64), dc.Params(4096, 256, codec=dc.CODEC_TANS)):
        blob, table = dc.compress_chunks(q, p)
        dst = torch.zeros(q.size, dtype=torch.uint8, device="cuda")
        trace = torch.zeros(4 * len(table), dtype=torch.int64, device="cuda")
        with pytest.raises(dc.DCError) as e:
            dc.decompress_chunks_traced(_up(torch, blob), blob.size, _up(torch, table), len(table), p, dst, q.size, trace, 0)
        assert e.value.code == -1  # DC_E_ARG


def test_issue_rate_probe_separates_the_two_classes_of_instruction(env):
    """The figures behind the ALU peak of the bench line: plain 32-bit logic and addition issue about twice as fast
    as three-operand, 64-bit, SDWA and conversion instructions."""
    torch, dc = env
    sink = torch.zeros(1024, dtype=torch.uint8, device="cuda")
    names = dc.issue_rate_names()
    assert len(names) == len(set(names)) >= 20
    ns = {n: min(dc.issue_rate(i, sink, 1024, 0) for _ in range(2)) for i, n in enumerate(names)}
    fast = [ns[n] for n in ("v_and_b32", "v_or_b32", "v_add_u32", "v_lshrrev_b32")]
    slow = [ns[n] for n in ("v_alignbit_b32", "v_perm_b32", "v_add3_u32", "v_lshrrev_b64", "v_sub_u32_sdwa", "v_cvt_f32_i32")]
    assert 0.5 < min(fast) and max(slow) < 5.0  # ns: two to four cycles at 1.5-2.5 GHz
    assert max(fast) < 0.7 * min(slow)
    with pytest.raises(dc.DCError):
        dc.issue_rate(len(names), sink, 1024, 0)
    with pytest.raises(dc.DCError):
        dc.issue_rate(0, sink, 512, 0)
