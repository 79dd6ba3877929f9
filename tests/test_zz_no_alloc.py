"""nqkv_decode_attention_static -- the entry point for callers that cannot allocate -- against
nqkv_decode_attention on the same inputs: same kernels, same split plan, so the outputs must be
equal bit for bit (and therefore within the 2e-3 bound of the fp64 oracle wherever the existing
entry point is).  Two calls in a row share the library's fixed scratch array, the second with a
smaller input, then a third after the array has been used by a different geometry.

Collected last (file name) so that a failure here cannot hide another test under `pytest -x`."""
import ctypes

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

ATTN_TOL = 2e-3


@pytest.fixture(scope="module")
def nqkv():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2505_16210_amd import nqkv as mod
    return mod


def _cache(nqkv, k, D, blk, B, H, S, seed):
    g = torch.Generator(device="cuda").manual_seed(seed)
    K = (torch.randn(B, H, S, D, device="cuda", generator=g) * 1.5).to(torch.float16)
    V = torch.randn(B, H, S, D, device="cuda", generator=g).to(torch.float16)
    q = (torch.randn(B, H, D, device="cuda", generator=g) / D ** 0.5).to(torch.float16)
    lv = nqkv.build_codebook(k)
    desc = nqkv.make_desc(B, H, D, k, blk, S)
    kc, ks = nqkv.alloc_cache(desc, "cuda")
    vc, vs = nqkv.alloc_cache(desc, "cuda")
    nqkv.quantize_kv_pair(desc, lv, K, V, kc, ks, vc, vs, 0)
    return lv, desc, q, kc, ks, vc, vs


def _both(nqkv, args, seq_len, num_splits):
    lv, desc, q, kc, ks, vc, vs = args
    out_s = torch.full_like(q, float("nan"))
    nqkv.decode_attention_static(desc, lv, q, kc, ks, vc, vs, seq_len, 0.9, out=out_s, num_splits=num_splits)
    ref = nqkv.decode_attention(desc, lv, q, kc, ks, vc, vs, seq_len, 0.9, num_splits=num_splits)
    torch.cuda.synchronize()
    return out_s, ref


def test_static_entry_equals_workspace_entry_two_calls_second_smaller(nqkv, oracle):
    big = _cache(nqkv, 4, 128, 64, 2, 4, 9000, seed=5)        # auto plan: 32 pieces per sequence
    small = _cache(nqkv, 4, 128, 64, 1, 3, 700, seed=6)       # fewer sequences, fewer pieces
    assert nqkv.decode_workspace_bytes(big[1], 9000, 0)[1] > nqkv.decode_workspace_bytes(small[1], 700, 0)[1] > 1
    out_big, ref_big = _both(nqkv, big, 9000, 0)
    out_small, ref_small = _both(nqkv, small, 700, 0)          # right after, on the same scratch array
    assert torch.equal(out_big, ref_big)
    assert torch.equal(out_small, ref_small)
    # and against the oracle itself, to the bound of the existing entry point
    lv, desc, q, kc, ks, vc, vs = small
    host = [t.cpu().numpy() for t in (q, kc, ks, vc, vs)]
    host = [a.view(np.uint16) if a.dtype == np.float16 else a for a in host]
    want = oracle.decode_attention(host[0], host[1], host[2], host[3], host[4], 4, 64, lv, 700, 0.9, n_threads=8)
    got = out_small.cpu().numpy().astype(np.float64)
    assert float((np.abs(got - want).max(-1) / np.abs(want).max(-1)).max()) <= ATTN_TOL


@pytest.mark.parametrize("k,D,blk", [(4, 64, 64), (3, 128, 128), (2, 128, 64)])
def test_static_entry_every_split_count_and_reuse(nqkv, k, D, blk):
    args = _cache(nqkv, k, D, blk, 2, 3, 1237, seed=40 + k)
    for seq_len, ns in ((1237, 64), (1237, 7), (65, 2), (1000, 1), (1, 0), (1237, 0), (129, 5)):
        out_s, ref = _both(nqkv, args, seq_len, ns)
        assert torch.equal(out_s, ref), (k, D, blk, seq_len, ns)


def test_static_entry_refuses_what_does_not_fit_and_bad_arguments(nqkv):
    lv = nqkv.build_codebook(4)
    # 4096 sequences x 8 pieces x 130 floats: beyond the 2 MiB array -> refused, nothing launched
    desc = nqkv.make_desc(64, 64, 128, 4, 64, 4096)
    need, _ = nqkv.decode_workspace_bytes(desc, 4096, 8)
    assert need > nqkv.STATIC_SCRATCH_BYTES
    q = torch.zeros(64, 64, 128, dtype=torch.float16, device="cuda")
    out = torch.full_like(q, 7.0)
    dummy = torch.zeros(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(nqkv.NqkvError) as e:
        nqkv.decode_attention_static(desc, lv, q, dummy, dummy, dummy, dummy, 4096, 1.0, out=out, num_splits=8)
    assert e.value.status == nqkv.EWORKSPACE
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())
    rc = nqkv.lib.nqkv_decode_attention_static(ctypes.byref(desc), None, None, None, None, None, None, 4096, 1.0, None, 1, None)
    assert rc == nqkv.EINVAL


def test_static_entry_captured_into_a_hip_graph_and_replayed(nqkv):
    """What the entry point is for: a launch that carries no allocation and no workspace argument can
    be recorded into a HIP graph.  (The array's address is looked up on the first call on a device,
    so one eager call comes first.)  Three replays with the program's own eager work between them;
    every replay equals the eager result bit for bit -- the counters are cleared by a kernel, not by
    a memset node."""
    args = _cache(nqkv, 4, 128, 64, 2, 4, 9000, seed=9)
    lv, desc, q, kc, ks, vc, vs = args
    assert nqkv.decode_workspace_bytes(desc, 9000, 0)[1] > 1
    eager = torch.empty_like(q)
    nqkv.decode_attention_static(desc, lv, q, kc, ks, vc, vs, 9000, 0.9, out=eager)
    torch.cuda.synchronize()
    out = torch.empty_like(q)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            nqkv.decode_attention_static(desc, lv, q, kc, ks, vc, vs, 9000, 0.9, out=out, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    other = _cache(nqkv, 2, 64, 64, 3, 2, 500, seed=10)
    for rep in range(3):
        out.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), rep
        # eager work on the same scratch array between the replays, with another geometry
        o2, r2 = _both(nqkv, other, 500, 0)
        assert torch.equal(o2, r2)
