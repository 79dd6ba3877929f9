"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times
(library-chosen split counts, K and V quantized in one launch).

C1-C4 are compared in full against the oracle.  For C5 (3.8 G elements per tensor) the GPU runs
the full tensors and the oracle checks whole (batch, head) slabs of two batch rows (first and
last) -- the path is independent per (batch, head), so a slab is a complete unit of work."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

ATTN_TOL = 2e-3
THREADS = 16


@pytest.fixture(scope="module")
def env():
    assert torch.cuda.is_available()
    from paper_2505_16210_amd import nqkv, workloads
    return nqkv, workloads


def bits(t):
    a = t.detach().cpu().numpy()
    return a.view(np.uint16) if a.dtype == np.float16 else a


def attn_err(out, ref):
    out = out.astype(np.float64)
    return float((np.abs(out - ref).max(-1) / np.abs(ref).max(-1)).max())


def quantize_and_attend(nqkv, workloads, cfg, k, blk, oracle, batch_rows=None):
    dev = torch.device("cuda:0")
    g = workloads.make_generator(cfg, dev)
    K, V = workloads.make_kv(cfg, dev, g)
    q = workloads.make_q(cfg, dev, g)
    lv = nqkv.build_codebook(k)
    desc = nqkv.make_desc(cfg.B, cfg.H, cfg.D, k, blk, cfg.S)
    kc, ks = nqkv.alloc_cache(desc, dev)
    vc, vs = nqkv.alloc_cache(desc, dev)
    nqkv.quantize_kv_pair(desc, lv, K, V, kc, ks, vc, vs, 0)
    out = nqkv.decode_attention(desc, lv, q, kc, ks, vc, vs, cfg.S, 1.0)
    torch.cuda.synchronize()
    rows = range(cfg.B) if batch_rows is None else batch_rows
    worst = 0.0
    for b in rows:
        sl = slice(b, b + 1)
        okc, oks = oracle.new_cache(1, cfg.H, cfg.D, k, blk, cfg.S)
        ovc, ovs = oracle.new_cache(1, cfg.H, cfg.D, k, blk, cfg.S)
        oracle.quantize_kv(bits(K[sl]), k, blk, lv, okc, oks, n_threads=THREADS)
        oracle.quantize_kv(bits(V[sl]), k, blk, lv, ovc, ovs, n_threads=THREADS)
        assert np.array_equal(bits(ks[sl]), oks) and np.array_equal(bits(vs[sl]), ovs), (cfg.name, k, blk, b)
        assert np.array_equal(bits(kc[sl]), okc) and np.array_equal(bits(vc[sl]), ovc), (cfg.name, k, blk, b)
        ref = oracle.decode_attention(bits(q[sl]), okc, oks, ovc, ovs, k, blk, lv, cfg.S, 1.0, n_threads=THREADS)
        worst = max(worst, attn_err(out[sl].cpu().numpy(), ref))
    assert worst <= ATTN_TOL, (cfg.name, k, blk, worst)
    return worst


def test_c1_full(env, oracle):
    nqkv, workloads = env
    quantize_and_attend(nqkv, workloads, workloads.C1, 4, 64, oracle)


def test_c3_full(env, oracle):
    nqkv, workloads = env
    quantize_and_attend(nqkv, workloads, workloads.C3, 4, 64, oracle)


def test_c4_full_long_context_split_k(env, oracle):
    nqkv, workloads = env
    cfg = workloads.C4
    desc = nqkv.make_desc(cfg.B, cfg.H, cfg.D, 4, 64, cfg.S)
    assert nqkv.decode_workspace_bytes(desc, cfg.S, 0)[1] > 1        # the bench configuration cuts the sequence
    quantize_and_attend(nqkv, workloads, cfg, 4, 64, oracle)


@pytest.mark.parametrize("k,blk", [(4, 64), (4, 128), (3, 64), (3, 128), (2, 64), (2, 128)])
def test_c5_sweep_sampled_slabs(env, oracle, k, blk):
    nqkv, workloads = env
    cfg = workloads.C5
    quantize_and_attend(nqkv, workloads, cfg, k, blk, oracle, batch_rows=(0, cfg.B - 1))
    torch.cuda.empty_cache()


def test_c5_bench_step_prefill_then_fused_decode_step(env, oracle):
    """The step bench.py times, as it launches it: the whole C5 prefill quantized in one launch into
    a cache with room after the prompt (the bench's own capacity), then ONE fused decode step that
    appends row S and attends over S + 1 tokens.  The oracle follows two whole batch rows."""
    import importlib.util, os
    nqkv, workloads = env
    spec = importlib.util.spec_from_file_location("bench", os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    cfg = workloads.C5
    B, H, D, S, k, blk = cfg.B, cfg.H, cfg.D, cfg.S, cfg.bits, cfg.block
    cap = S + bench.STEP_HEADROOM
    dev = torch.device("cuda:0")
    g = workloads.make_generator(cfg, dev)
    K, V = workloads.make_kv(cfg, dev, g, n_tokens=S + 1)
    q = workloads.make_q(cfg, dev, g)
    lv = nqkv.build_codebook(k)
    desc = nqkv.make_desc(B, H, D, k, blk, cap)
    kc, ks = nqkv.alloc_cache(desc, dev)
    vc, vs = nqkv.alloc_cache(desc, dev)
    nqkv.quantize_kv_pair(desc, lv, K[:, :, :S], V[:, :, :S], kc, ks, vc, vs, 0)
    out = nqkv.decode_step(desc, lv, q, K[:, :, S:], V[:, :, S:], kc, ks, vc, vs, S, 1.0)
    torch.cuda.synchronize()
    for b in (0, B - 1):
        sl = slice(b, b + 1)
        okc, oks = oracle.new_cache(1, H, D, k, blk, S + 1)
        ovc, ovs = oracle.new_cache(1, H, D, k, blk, S + 1)
        oracle.quantize_kv(bits(K[sl]), k, blk, lv, okc, oks, n_threads=THREADS)
        oracle.quantize_kv(bits(V[sl]), k, blk, lv, ovc, ovs, n_threads=THREADS)
        assert np.array_equal(bits(kc[sl, :, :S + 1]), okc) and np.array_equal(bits(ks[sl, :, :S + 1]), oks), b
        assert np.array_equal(bits(vc[sl, :, :S + 1]), ovc) and np.array_equal(bits(vs[sl, :, :S + 1]), ovs), b
        ref = oracle.decode_attention(bits(q[sl]), okc, oks, ovc, ovs, k, blk, lv, S + 1, 1.0, n_threads=THREADS)
        assert attn_err(out[sl].cpu().numpy(), ref) <= ATTN_TOL, b
    del K, V, kc, ks, vc, vs
    torch.cuda.empty_cache()


@pytest.mark.parametrize("name,q_len,rows,k", [("C3", 4, (0, 31), 4), ("C4", 16, (0,), 4), ("C2", 5, (0, 7), 4),
                                               ("C3", 7, (5,), 3), ("C3", 16, (17,), 2), ("C2", 3, (3,), 3)])
def test_multi_query_attention_full_size(env, oracle, name, q_len, rows, k):
    """Several queries per sequence at the bench sizes and the library's own split count: the
    queries of the last q_len cached tokens, each over its causal prefix, against the oracle on
    whole batch rows."""
    nqkv, workloads = env
    cfg = workloads.CONFIGS[name]
    dev = torch.device("cuda:0")
    g = workloads.make_generator(cfg, dev)
    K, V = workloads.make_kv(cfg, dev, g)
    q = (torch.randn(cfg.B, cfg.H, q_len, cfg.D, device=dev, generator=g) / cfg.D ** 0.5).to(torch.float16)
    lv = nqkv.build_codebook(k)
    desc = nqkv.make_desc(cfg.B, cfg.H, cfg.D, k, 64, cfg.S)
    kc, ks = nqkv.alloc_cache(desc, dev)
    vc, vs = nqkv.alloc_cache(desc, dev)
    nqkv.quantize_kv_pair(desc, lv, K, V, kc, ks, vc, vs, 0)
    if name == "C4":
        assert nqkv.decode_multi_workspace_bytes(desc, cfg.S, q_len, 0)[1] > 1
    out = nqkv.decode_attention_multi(desc, lv, q, kc, ks, vc, vs, cfg.S, 1.0)
    torch.cuda.synchronize()
    for b in rows:
        sl = slice(b, b + 1)
        ref = oracle.decode_attention_multi(bits(q[sl]), bits(kc[sl]), bits(ks[sl]), bits(vc[sl]), bits(vs[sl]),
                                            k, 64, lv, cfg.S, 1.0, n_threads=THREADS)
        o = out[sl].cpu().numpy().reshape(1, -1, cfg.D)
        assert np.isfinite(o.astype(np.float32)).all()
        assert attn_err(o, ref.reshape(1, -1, cfg.D)) <= ATTN_TOL, (name, q_len, k, b)


@pytest.mark.parametrize("fused", [False, True])
def test_c2_prefill_then_128_decode_steps(env, oracle, fused):
    """The bench workload itself: quantize the 2048-token prefill, then 128 x (append one token,
    attend over everything cached) -- as two launches per iteration, and as the single fused
    launch bench.py times.  Attention is checked against the oracle at steps
    0, 1, 31, 64, 126, 127; the final caches must equal the oracle's bit for bit."""
    nqkv, workloads = env
    cfg = workloads.C2
    dev = torch.device("cuda:0")
    g = workloads.make_generator(cfg, dev)
    B, H, D, S, n_dec, cap = cfg.B, cfg.H, cfg.D, cfg.S, cfg.decode_steps, cfg.cap_tokens
    K, V = workloads.make_kv(cfg, dev, g, n_tokens=cap)
    qs = [workloads.make_q(cfg, dev, g) for _ in range(n_dec)]
    k, blk = cfg.bits, cfg.block
    lv = nqkv.build_codebook(k)
    desc = nqkv.make_desc(B, H, D, k, blk, cap)
    kc, ks = nqkv.alloc_cache(desc, dev)
    vc, vs = nqkv.alloc_cache(desc, dev)
    nqkv.quantize_kv_pair(desc, lv, K[:, :, :S], V[:, :, :S], kc, ks, vc, vs, 0)
    outs = {}
    check_at = {0, 1, 31, 64, 126, 127}
    for i in range(n_dec):
        pos = S + i
        if fused:
            o = nqkv.decode_step(desc, lv, qs[i], K[:, :, pos:pos + 1], V[:, :, pos:pos + 1], kc, ks, vc, vs, pos, 1.0)
        else:
            nqkv.quantize_kv_pair(desc, lv, K[:, :, pos:pos + 1], V[:, :, pos:pos + 1], kc, ks, vc, vs, pos)
            o = nqkv.decode_attention(desc, lv, qs[i], kc, ks, vc, vs, pos + 1, 1.0)
        if i in check_at:
            outs[i] = o.clone()
    torch.cuda.synchronize()
    okc, oks = oracle.new_cache(B, H, D, k, blk, cap)
    ovc, ovs = oracle.new_cache(B, H, D, k, blk, cap)
    oracle.quantize_kv(bits(K), k, blk, lv, okc, oks, n_threads=THREADS)
    oracle.quantize_kv(bits(V), k, blk, lv, ovc, ovs, n_threads=THREADS)
    assert np.array_equal(bits(kc), okc) and np.array_equal(bits(ks), oks)
    assert np.array_equal(bits(vc), ovc) and np.array_equal(bits(vs), ovs)
    for i in sorted(check_at):
        ref = oracle.decode_attention(bits(qs[i]), okc, oks, ovc, ovs, k, blk, lv, S + i + 1, 1.0, n_threads=THREADS)
        assert attn_err(outs[i].cpu().numpy(), ref) <= ATTN_TOL, i


def test_largest_slab_the_library_accepts(env, oracle):
    """Maximum size: one (batch, head) slab just under the 2 GiB the 32-bit lane offsets can address
    (D 128: 2^23 - 1 tokens, 1.07 G elements per tensor), one token more being refused.  The GPU
    quantizes K and V whole; the oracle (given the same fp16 bits) quantizes them in 16 token
    windows on 16 threads; codes, scales and a 64-way split-K attention over all 8.4 M tokens
    are compared in full."""
    import concurrent.futures
    nqkv, workloads = env
    dev = torch.device("cuda:0")
    D, k, blk = 128, 4, 64
    n = (1 << 23) - 1
    lv = nqkv.build_codebook(k)
    desc = nqkv.make_desc(1, 1, D, k, blk, n + 1)
    g = torch.Generator(device=dev).manual_seed(123)
    K = torch.empty(1, 1, n + 1, D, dtype=torch.float16, device=dev)
    V = torch.empty_like(K)
    step = 1 << 20
    for t0 in range(0, n + 1, step):                       # fp32 noise in slices, cast to fp16
        t1 = min(t0 + step, n + 1)
        K[0, 0, t0:t1] = (torch.randn(t1 - t0, D, device=dev, generator=g) *
                          torch.exp(0.5 * torch.randn(1, D, device=dev, generator=g))).to(torch.float16)
        V[0, 0, t0:t1] = torch.randn(t1 - t0, D, device=dev, generator=g).to(torch.float16)
    q = (torch.randn(1, 1, D, device=dev, generator=g) / 128 ** 0.5).to(torch.float16)
    kc, ks = nqkv.alloc_cache(desc, dev)
    vc, vs = nqkv.alloc_cache(desc, dev)
    with pytest.raises(nqkv.NqkvError) as e:               # 2^23 tokens: one past the limit
        nqkv.quantize_kv_pair(desc, lv, K, V, kc, ks, vc, vs, 0)
    assert e.value.status == nqkv.EUNSUPPORTED
    nqkv.quantize_kv_pair(desc, lv, K[:, :, :n], V[:, :, :n], kc, ks, vc, vs, 0)
    out = nqkv.decode_attention(desc, lv, q, kc, ks, vc, vs, n, 1.0, num_splits=64)
    torch.cuda.synchronize()
    Kh, Vh = bits(K), bits(V)
    okc, oks = oracle.new_cache(1, 1, D, k, blk, n + 1)
    ovc, ovs = oracle.new_cache(1, 1, D, k, blk, n + 1)
    edges = np.linspace(0, n, THREADS + 1).astype(np.int64)

    def window(i):
        a, b = int(edges[i]), int(edges[i + 1])
        oracle.quantize_kv(Kh[:, :, a:b], k, blk, lv, okc, oks, dst_off=a)
        oracle.quantize_kv(Vh[:, :, a:b], k, blk, lv, ovc, ovs, dst_off=a)

    with concurrent.futures.ThreadPoolExecutor(THREADS) as pool:
        list(pool.map(window, range(THREADS)))
    assert np.array_equal(bits(ks), oks) and np.array_equal(bits(vs), ovs)
    assert np.array_equal(bits(kc), okc) and np.array_equal(bits(vc), ovc)
    ref = oracle.decode_attention(bits(q), okc, oks, ovc, ovs, k, blk, lv, n, 1.0, n_threads=1)
    assert attn_err(out.cpu().numpy(), ref) <= ATTN_TOL


def test_largest_batch_row_of_the_hidden_block_quantizer(env, oracle):
    """Maximum size of nqkv_quantize_kv_hidden: one batch row of token-major source just under
    2 GiB (16 heads of 64: 2^20 - 1 tokens, 1.07 G elements), compared in full; one token more
    is refused."""
    nqkv, workloads = env
    dev = torch.device("cuda:0")
    H, D, k = 16, 64, 4
    n = (1 << 20) - 1
    lv = nqkv.build_codebook(k)
    desc = nqkv.make_desc(1, H, D, k, D, n + 1)
    g = torch.Generator(device=dev).manual_seed(321)
    X = torch.empty(1, n + 1, H, D, dtype=torch.float16, device=dev)      # token-major storage
    step = 1 << 18
    for t0 in range(0, n + 1, step):
        t1 = min(t0 + step, n + 1)
        X[0, t0:t1] = (torch.randn(t1 - t0, H, D, device=dev, generator=g) *
                       torch.exp(torch.randn(t1 - t0, 1, 1, device=dev, generator=g))).to(torch.float16)
    view = X.transpose(1, 2)                                               # [1,H,n+1,D]
    kc, ks = nqkv.alloc_cache(desc, dev)
    with pytest.raises(nqkv.NqkvError) as e:
        nqkv.quantize_kv_hidden(desc, lv, view, None, kc, ks, None, None, 0, 256)
    assert e.value.status == nqkv.EUNSUPPORTED
    nqkv.quantize_kv_hidden(desc, lv, view[:, :, :n], None, kc, ks, None, None, 0, 256)
    torch.cuda.synchronize()
    okc, oks = oracle.new_cache(1, H, D, k, D, n + 1)
    oracle.quantize_kv_hidden(bits(X).transpose(0, 2, 1, 3)[:, :, :n], k, 256, lv, okc, oks, n_threads=THREADS)
    assert np.array_equal(bits(ks), oks)
    assert np.array_equal(bits(kc), okc)


def test_c2_step_as_hip_graph_replays(env, oracle):
    """The launch configuration bench.py times: the C2 step (prefill + 128 fused decode launches)
    captured once into a HIP graph and replayed.  Three replays, with the program's own eager
    work between them (caches and outputs overwritten with other data, an eager split-K call that
    dirties the workspace counters' neighbourhood), must each reproduce the eager run bit for
    bit; the eager run itself is checked against the oracle at six steps."""
    nqkv, workloads = env
    cfg = workloads.C2
    dev = torch.device("cuda:0")
    g = workloads.make_generator(cfg, dev)
    B, H, D, S, n_dec, cap = cfg.B, cfg.H, cfg.D, cfg.S, cfg.decode_steps, cfg.cap_tokens
    K, V = workloads.make_kv(cfg, dev, g, n_tokens=cap)
    qs = [workloads.make_q(cfg, dev, g) for _ in range(n_dec)]
    k, blk = cfg.bits, cfg.block
    lv = nqkv.build_codebook(k)
    desc = nqkv.make_desc(B, H, D, k, blk, cap)
    kc, ks = nqkv.alloc_cache(desc, dev)
    vc, vs = nqkv.alloc_cache(desc, dev)
    outs = torch.zeros(n_dec, B, H, D, dtype=torch.float16, device=dev)
    ws_bytes, _ = nqkv.decode_workspace_bytes(desc, cap, 0)
    ws = torch.zeros(max(ws_bytes, 16), dtype=torch.uint8, device=dev)
    new = [(K[:, :, S + i:S + i + 1], V[:, :, S + i:S + i + 1]) for i in range(n_dec)]

    def step():
        nqkv.quantize_kv_pair(desc, lv, K[:, :, :S], V[:, :, :S], kc, ks, vc, vs, 0)
        for i in range(n_dec):
            nqkv.decode_step(desc, lv, qs[i], *new[i], kc, ks, vc, vs, S + i, 1.0, out=outs[i], workspace=ws)

    step()
    torch.cuda.synchronize()
    eager = [t.clone() for t in (outs, kc, ks, vc, vs)]
    okc, oks = oracle.new_cache(B, H, D, k, blk, cap)
    ovc, ovs = oracle.new_cache(B, H, D, k, blk, cap)
    oracle.quantize_kv(bits(K), k, blk, lv, okc, oks, n_threads=THREADS)
    oracle.quantize_kv(bits(V), k, blk, lv, ovc, ovs, n_threads=THREADS)
    assert np.array_equal(bits(kc), okc) and np.array_equal(bits(vs), ovs)
    for i in (0, 1, 31, 64, 126, 127):
        ref = oracle.decode_attention(bits(qs[i]), okc, oks, ovc, ovs, k, blk, lv, S + i + 1, 1.0, n_threads=THREADS)
        assert attn_err(outs[i].cpu().numpy(), ref) <= ATTN_TOL, i

    main = torch.cuda.current_stream()
    side = torch.cuda.Stream()
    side.wait_stream(main)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    # a second, split-K shape for the eager work between replays (its own workspace and caches)
    d2 = nqkv.make_desc(1, 4, D, k, blk, 4096)
    kc2, ks2 = nqkv.alloc_cache(d2, dev)
    vc2, vs2 = nqkv.alloc_cache(d2, dev)
    nqkv.quantize_kv_pair(d2, lv, K[:1, :4, :cap].repeat(1, 1, 2, 1)[:, :, :4096].contiguous(),
                          V[:1, :4, :cap].repeat(1, 1, 2, 1)[:, :, :4096].contiguous(), kc2, ks2, vc2, vs2, 0)
    ref2 = nqkv.decode_attention(d2, lv, qs[0][:1, :4].contiguous(), kc2, ks2, vc2, vs2, 4096, 1.0, num_splits=8).clone()
    for rep in range(3):
        for t in (kc, vc):
            t.fill_(0x5A)
        for t in (ks, vs, outs):
            t.fill_(1.0)
        o2 = nqkv.decode_attention(d2, lv, qs[0][:1, :4].contiguous(), kc2, ks2, vc2, vs2, 4096, 1.0, num_splits=8)
        torch.cuda.synchronize()
        assert torch.equal(o2, ref2)
        graph.replay()
        torch.cuda.synchronize()
        for name, got, want in zip(("outs", "kc", "ks", "vc", "vs"), (outs, kc, ks, vc, vs), eager):
            assert torch.equal(got, want), (rep, name)


@pytest.mark.parametrize("q_len", [1, 4])
def test_split_k_launches_as_hip_graph_replays(env, oracle, q_len):
    """Split-K attention (the ticket counters of the one-query kernel, the partial buffers and
    combine launch of the several-queries kernel) captured into a HIP graph: every replay equals
    the eager result bit for bit, with eager calls on the same workspace between the replays."""
    nqkv, workloads = env
    dev = torch.device("cuda:0")
    k, D, blk, B, H, S = 4, 128, 64, 1, 8, 8192 + 37
    lv = nqkv.build_codebook(k)
    desc = nqkv.make_desc(B, H, D, k, blk, S)
    g = torch.Generator(device=dev).manual_seed(5)
    Kx = torch.randn(B, H, S, D, device=dev, generator=g).to(torch.float16)
    Vx = torch.randn(B, H, S, D, device=dev, generator=g).to(torch.float16)
    kc, ks = nqkv.alloc_cache(desc, dev)
    vc, vs = nqkv.alloc_cache(desc, dev)
    nqkv.quantize_kv_pair(desc, lv, Kx, Vx, kc, ks, vc, vs, 0)
    n_calls = 6
    if q_len == 1:
        q = (torch.randn(n_calls, B, H, D, device=dev, generator=g) / D ** 0.5).to(torch.float16)
        nbytes, splits = nqkv.decode_workspace_bytes(desc, S, 0)
        call = lambda i, o, w: nqkv.decode_attention(desc, lv, q[i], kc, ks, vc, vs, S - i, 1.0, out=o[i], workspace=w)
        ref_of = lambda i: oracle.decode_attention(bits(q[i]), bits(kc), bits(ks), bits(vc), bits(vs), k, blk, lv, S - i, 1.0,
                                                   n_threads=THREADS)
    else:
        q = (torch.randn(n_calls, B, H, q_len, D, device=dev, generator=g) / D ** 0.5).to(torch.float16)
        nbytes, splits = nqkv.decode_multi_workspace_bytes(desc, S, q_len, 0)
        call = lambda i, o, w: nqkv.decode_attention_multi(desc, lv, q[i], kc, ks, vc, vs, S - i, 1.0, out=o[i], workspace=w)
        ref_of = lambda i: oracle.decode_attention_multi(bits(q[i]), bits(kc), bits(ks), bits(vc), bits(vs), k, blk, lv,
                                                         S - i, 1.0, n_threads=THREADS)
    assert splits > 1 and nbytes > 0
    ws = torch.zeros(nbytes, dtype=torch.uint8, device=dev)
    out = torch.zeros_like(q)
    for i in range(n_calls):
        call(i, out, ws)
    torch.cuda.synchronize()
    eager = out.clone()
    for i in (0, n_calls - 1):
        assert attn_err(eager[i].cpu().numpy(), ref_of(i)) <= ATTN_TOL
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            for i in range(n_calls):
                call(i, out, ws)
    torch.cuda.synchronize()
    scratch_out = torch.zeros_like(q)
    for rep in range(3):
        out.fill_(2.0)
        call(rep, scratch_out, ws)                  # eager work on the same workspace
        torch.cuda.synchronize()
        assert torch.equal(scratch_out[rep], eager[rep])
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), rep


@pytest.mark.parametrize("name,k,blk,rows", [("C2", 4, 64, (0, 7)), ("C3", 4, 64, (0, 31)), ("C4", 4, 64, (0,)),
                                             ("C5", 4, 64, (0, 15)), ("C5", 3, 128, (15,)), ("C5", 2, 64, (7,))])
def test_dequantize_full_size(env, oracle, name, k, blk, rows):
    """nqkv_dequantize_kv over a whole cache of the benchmark's size in one call (random code bytes,
    every finite non-negative fp16 scale), whole batch rows compared bit for bit; then a ragged
    token window into a token-major destination."""
    nqkv, workloads = env
    cfg = workloads.CONFIGS[name]
    dev = torch.device("cuda:0")
    B, H, D, S = cfg.B, cfg.H, cfg.D, cfg.S
    lv = nqkv.build_codebook(k)
    desc = nqkv.make_desc(B, H, D, k, blk, S)
    codes, scales = nqkv.alloc_cache(desc, dev)
    g = torch.Generator(device=dev).manual_seed(1000 + k)
    codes.copy_(torch.randint(0, 256, codes.shape, device=dev, generator=g, dtype=torch.uint8))
    scales.view(torch.int16).copy_(torch.randint(0, 0x7C00, scales.shape, device=dev, generator=g, dtype=torch.int16))
    out = nqkv.dequantize_kv(desc, lv, codes, scales, 0, S)
    off, n = 1003, S - 2007
    out_tm = torch.zeros(B, n + 2, H, D, dtype=torch.float16, device=dev)         # rows 0 and n + 1 stay untouched
    nqkv.dequantize_kv(desc, lv, codes, scales, off, n, out=out_tm[:, 1:n + 1].permute(0, 2, 1, 3))
    torch.cuda.synchronize()
    assert not out_tm[:, 0].any() and not out_tm[:, n + 1].any()
    for b in rows:
        sl = slice(b, b + 1)
        ref = oracle.dequantize_kv(bits(codes[sl]), bits(scales[sl]), k, blk, lv, 0, S, n_threads=THREADS)
        assert np.array_equal(bits(out[sl]), ref), (name, k, blk, b)
        assert np.array_equal(bits(out_tm[sl, 1:n + 1].permute(0, 2, 1, 3).contiguous()), ref[:, :, off:off + n]), (name, b)
