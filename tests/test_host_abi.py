"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares,
its host-side quantile table equals the oracle's, and every argument error is reported before
any GPU work (so these run on a machine without a GPU)."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def nqkv():
    from paper_2505_16210_amd import nqkv as mod
    return mod


def test_library_exports_every_declared_symbol(nqkv):
    header = open(os.path.join(ROOT, "include", "nqkv.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(nqkv_[a-z_0-9]+)\s*\(", header))
    assert declared == set(nqkv.EXPORTS)
    raw = ctypes.CDLL(nqkv.LIB_PATH)
    for name in declared:
        assert hasattr(raw, name), name
    assert nqkv.version() == 100
    assert nqkv.strerror(0) == "ok" and "workspace" in nqkv.strerror(nqkv.EWORKSPACE)


def test_header_is_plain_c_and_links(nqkv, tmp_path):
    """The boundary is a C ABI: the header compiles as C99 and as C++11 with pedantic warnings as
    errors, and a C program that uses it links against the library and runs (host-only calls)."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no C compiler")
    src = tmp_path / "use_nqkv.c"
    src.write_text('#include "nqkv.h"\n#include <stdio.h>\n'
                   'int main(void) {\n  float lv[16];\n  nqkv_cache_desc d = {1, 2, 64, 4, 64, 0, 128};\n'
                   '  size_t bytes = 1; int splits = 0;\n'
                   '  if (nqkv_build_codebook(4, 0, lv) != NQKV_OK || lv[0] != -1.0f || lv[15] != 1.0f) return 1;\n'
                   '  if (nqkv_decode_workspace_bytes(&d, 100, 1, &bytes, &splits) != NQKV_OK || bytes != 0 || splits != 1) return 2;\n'
                   '  if (nqkv_build_codebook(0, 0, lv) != NQKV_EINVAL) return 3;\n'
                   '  printf("%d %s\\n", nqkv_version(), nqkv_strerror(NQKV_EWORKSPACE));\n  return 0;\n}\n')
    inc = os.path.join(ROOT, "include")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-I", inc, str(src)], check=True)
    subprocess.run(["g++", "-std=c++11", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c++", "-I", inc, str(src)],
                   check=True)
    exe = tmp_path / "use_nqkv"
    libdir = os.path.dirname(nqkv.LIB_PATH)
    subprocess.run(["gcc", "-std=c99", "-I", inc, str(src), "-o", str(exe), "-L", libdir, "-l:libnqkv.so",
                    "-Wl,-rpath," + libdir], check=True)
    r = subprocess.run([str(exe)], capture_output=True, text=True)
    assert r.returncode == 0, (r.returncode, r.stdout, r.stderr)
    assert r.stdout.split()[0] == "100"


def test_desc_struct_layout(nqkv):
    assert ctypes.sizeof(nqkv.CacheDesc) == 32
    assert nqkv.CacheDesc.cap_tokens.offset == 24


@pytest.mark.parametrize("variant", [0, 1])
@pytest.mark.parametrize("k", range(1, 9))
def test_codebook_equals_oracle_table(nqkv, oracle, k, variant):
    if variant == 1 and k < 2:
        with pytest.raises(nqkv.NqkvError):
            nqkv.build_codebook(k, variant)
        return
    got = nqkv.build_codebook(k, variant)
    _, want, _ = oracle.codebook(k, variant)
    assert got.dtype == np.float32 and np.array_equal(got, want)


def test_codebook_errors(nqkv):
    for k, v in ((0, 0), (9, 0), (4, 2), (-1, 0)):
        with pytest.raises(nqkv.NqkvError) as e:
            nqkv.build_codebook(k, v)
        assert e.value.status == nqkv.EINVAL
    assert nqkv.lib.nqkv_build_codebook(4, 0, None) == nqkv.EINVAL


# ---------------------------------------------------------------- argument validation (no launch)
FAKE = 0x10000   # non-null, 16-byte aligned; never dereferenced because validation fails first


def _levels(nqkv, k=4):
    lv = nqkv.build_codebook(k)
    return lv, lv.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _quant(nqkv, desc, lvp, src=FAKE, sb=0, sh=0, st=64, n=1, off=0, codes=FAKE, scales=FAKE):
    return nqkv.lib.nqkv_quantize_kv(ctypes.byref(desc) if desc is not None else None, lvp,
                                     src, sb, sh, st, n, off, codes, scales, None)


def test_quantize_argument_errors(nqkv):
    lv, lvp = _levels(nqkv)
    good = nqkv.make_desc(2, 4, 64, 4, 64, 16)
    assert _quant(nqkv, None, lvp) == nqkv.EINVAL
    assert _quant(nqkv, good, None) == nqkv.EINVAL
    assert _quant(nqkv, good, lvp, src=None) == nqkv.EINVAL
    assert _quant(nqkv, good, lvp, codes=None) == nqkv.EINVAL
    assert _quant(nqkv, good, lvp, scales=None) == nqkv.EINVAL
    assert _quant(nqkv, good, lvp, src=FAKE + 2) == nqkv.EINVAL          # misaligned
    assert _quant(nqkv, good, lvp, codes=FAKE + 8) == nqkv.EINVAL
    assert _quant(nqkv, good, lvp, n=-1) == nqkv.EINVAL
    assert _quant(nqkv, good, lvp, n=2, off=15) == nqkv.EINVAL           # past capacity
    assert _quant(nqkv, good, lvp, n=1, off=17) == nqkv.EINVAL
    assert _quant(nqkv, good, lvp, off=-1) == nqkv.EINVAL
    assert _quant(nqkv, good, lvp, st=60) == nqkv.EINVAL                 # rows not 16-byte aligned
    assert _quant(nqkv, good, lvp, n=2, st=32) == nqkv.EINVAL            # rows overlap
    assert _quant(nqkv, good, lvp, sb=-8) == nqkv.EINVAL
    assert _quant(nqkv, good, lvp, n=0) == nqkv.OK                       # empty: success, nothing launched
    for bad in (dict(B=0), dict(H=0), dict(cap_tokens=0), dict(flags=4), dict(flags=-1), dict(D=0)):
        d = nqkv.make_desc(2, 4, 64, 4, 64, 16)
        for f, v in bad.items():
            setattr(d, f, v)
        assert _quant(nqkv, d, lvp) == nqkv.EINVAL
    for bad in (dict(k=5), dict(k=1), dict(D=96), dict(D=256), dict(block=32), dict(B=4096, H=4097), dict(H=65536), dict(B=32768, H=1)):
        d = nqkv.make_desc(2, 4, 64, 4, 64, 16)
        for f, v in bad.items():
            setattr(d, f, v)
        assert _quant(nqkv, d, lvp) == nqkv.EUNSUPPORTED
    d = nqkv.make_desc(2, 4, 64, 4, 128, 16)                             # block does not divide D
    assert _quant(nqkv, d, lvp) == nqkv.EINVAL
    # tables must be finite and strictly ascending
    for bad in (lv[::-1].copy(), np.where(np.arange(16) == 3, np.nan, lv).astype(np.float32),
                np.where(np.arange(16) == 3, lv[2], lv).astype(np.float32)):
        assert _quant(nqkv, good, bad.ctypes.data_as(ctypes.POINTER(ctypes.c_float))) == nqkv.EINVAL


def test_quantize_pair_and_dequantize_argument_errors(nqkv):
    lv, lvp = _levels(nqkv)
    d = nqkv.make_desc(2, 4, 128, 4, 64, 16)
    f = nqkv.lib.nqkv_quantize_kv_pair
    assert f(ctypes.byref(d), lvp, FAKE, None, 0, 0, 128, 1, 0, FAKE, FAKE, FAKE, FAKE, None) == nqkv.EINVAL
    assert f(ctypes.byref(d), lvp, FAKE, FAKE, 0, 0, 128, 1, 0, FAKE, FAKE, None, FAKE, None) == nqkv.EINVAL
    assert f(ctypes.byref(d), lvp, FAKE, FAKE, 0, 0, 128, 0, 0, FAKE, FAKE, FAKE, FAKE, None) == nqkv.OK
    g = nqkv.lib.nqkv_dequantize_kv
    assert g(ctypes.byref(d), lvp, None, FAKE, 0, 1, FAKE, 0, 0, 128, None) == nqkv.EINVAL
    assert g(ctypes.byref(d), lvp, FAKE, FAKE, 16, 1, FAKE, 0, 0, 128, None) == nqkv.EINVAL
    assert g(ctypes.byref(d), lvp, FAKE, FAKE, 0, 1, FAKE + 4, 0, 0, 128, None) == nqkv.EINVAL
    assert g(ctypes.byref(d), lvp, FAKE, FAKE, 3, 0, FAKE, 0, 0, 128, None) == nqkv.OK


def test_workspace_planning(nqkv):
    d = nqkv.make_desc(1, 32, 128, 4, 64, 32768)
    nbytes, splits = nqkv.decode_workspace_bytes(d, 32768, 0)
    assert splits > 1 and nbytes == 262144 + 32 * splits * 130 * 4
    assert nqkv.decode_workspace_bytes(d, 32768, 1) == (0, 1)
    assert nqkv.decode_workspace_bytes(d, 32768, 7) == (262144 + 32 * 7 * 130 * 4, 7)
    assert nqkv.decode_workspace_bytes(d, 5, 0) == (0, 1)               # short sequence: one piece
    big = nqkv.make_desc(32, 32, 128, 4, 64, 2048)
    assert nqkv.decode_workspace_bytes(big, 2048, 0)[1] <= 2
    for seq, ns in ((0, 0), (32769, 0), (10, 11), (10, -1), (4000, 1025)):
        with pytest.raises(nqkv.NqkvError) as e:
            nqkv.decode_workspace_bytes(d, seq, ns)
        assert e.value.status == nqkv.EINVAL
    assert nqkv.lib.nqkv_decode_workspace_bytes(ctypes.byref(d), 100, 0, None, None) == nqkv.EINVAL


def test_decode_argument_errors(nqkv):
    lv, lvp = _levels(nqkv)
    d = nqkv.make_desc(1, 32, 128, 4, 64, 32768)
    f = nqkv.lib.nqkv_decode_attention

    def call(q=FAKE, kc=FAKE, ks=FAKE, vc=FAKE, vs=FAKE, seq=32768, scale=1.0, out=FAKE, ws=FAKE,
             ws_bytes=1 << 30, ns=0, desc=d, levels=lvp):
        return f(ctypes.byref(desc), levels, q, kc, ks, vc, vs, seq, scale, out, ws, ws_bytes, ns, None)

    assert call(q=None) == nqkv.EINVAL
    assert call(out=None) == nqkv.EINVAL
    assert call(vs=FAKE + 2) == nqkv.EINVAL
    assert call(seq=0) == nqkv.EINVAL
    assert call(seq=32769) == nqkv.EINVAL
    assert call(scale=float("inf")) == nqkv.EINVAL
    assert call(ns=8, ws=None) == nqkv.EINVAL                    # split-K needs a workspace
    assert call(ns=8, ws_bytes=100) == nqkv.EWORKSPACE
    assert call(ns=2000) == nqkv.EINVAL
    assert call(levels=None) == nqkv.EINVAL


def test_decode_static_argument_errors(nqkv):
    """The entry point without a workspace argument: every refusal comes before any GPU call, the
    size limit of its fixed array included."""
    lv, lvp = _levels(nqkv)
    d = nqkv.make_desc(1, 32, 128, 4, 64, 32768)
    f = nqkv.lib.nqkv_decode_attention_static

    def call(q=FAKE, kc=FAKE, ks=FAKE, vc=FAKE, vs=FAKE, seq=32768, scale=1.0, out=FAKE, ns=0, desc=d, levels=lvp):
        return f(ctypes.byref(desc), levels, q, kc, ks, vc, vs, seq, scale, out, ns, None)

    assert call(q=None) == nqkv.EINVAL
    assert call(out=FAKE + 4) == nqkv.EINVAL
    assert call(seq=0) == nqkv.EINVAL
    assert call(ns=2000) == nqkv.EINVAL
    assert call(levels=None) == nqkv.EINVAL
    assert call(desc=nqkv.make_desc(1, 32, 96, 4, 64, 32768)) == nqkv.EUNSUPPORTED
    # 32 sequences x 1024 pieces x 130 floats + counters > 2 MiB
    assert nqkv.decode_workspace_bytes(d, 32768, 1024)[0] > nqkv.STATIC_SCRATCH_BYTES
    assert call(ns=1024) == nqkv.EWORKSPACE
    big = nqkv.make_desc(64, 64, 128, 4, 64, 4096)
    assert call(desc=big, seq=4096, ns=8) == nqkv.EWORKSPACE
    header = open(os.path.join(ROOT, "include", "nqkv.h")).read()
    assert "#define NQKV_STATIC_SCRATCH_BYTES (2u << 20)" in header and nqkv.STATIC_SCRATCH_BYTES == 2 << 20


def test_workspace_init_and_check_argument_errors(nqkv):
    for f in (nqkv.lib.nqkv_decode_workspace_init, nqkv.lib.nqkv_decode_workspace_check):
        assert f(None, 1 << 20, None) == nqkv.EINVAL
        assert f(FAKE + 8, 1 << 20, None) == nqkv.EINVAL
        assert f(FAKE, 1000, None) == nqkv.EWORKSPACE             # the counters alone take 256 KiB


def test_decode_step_argument_errors(nqkv):
    lv, lvp = _levels(nqkv)
    d = nqkv.make_desc(1, 32, 128, 4, 64, 32768)
    f = nqkv.lib.nqkv_decode_step

    def call(q=FAKE, kn=FAKE, vn=FAKE, sb=4096, sh=128, kc=FAKE, ks=FAKE, vc=FAKE, vs=FAKE, pos=32767,
             scale=1.0, out=FAKE, ws=FAKE, ws_bytes=1 << 30, ns=0, desc=d, levels=lvp):
        return f(ctypes.byref(desc), levels, q, kn, vn, sb, sh, kc, ks, vc, vs, pos, scale, out, ws, ws_bytes,
                 ns, None)

    assert call(kn=None) == nqkv.EINVAL
    assert call(vn=None) == nqkv.EINVAL
    assert call(kn=FAKE + 2) == nqkv.EINVAL                      # rows are read 16 bytes at a time
    assert call(sb=4100) == nqkv.EINVAL
    assert call(sh=-128) == nqkv.EINVAL
    assert call(pos=-1) == nqkv.EINVAL
    assert call(pos=32768) == nqkv.EINVAL                        # no room for the new row
    assert call(q=None) == nqkv.EINVAL
    assert call(kc=None) == nqkv.EINVAL
    assert call(scale=float("nan")) == nqkv.EINVAL
    assert call(ns=8, ws=None) == nqkv.EINVAL
    assert call(ns=8, ws_bytes=100) == nqkv.EWORKSPACE
    assert call(pos=0, ns=2) == nqkv.EINVAL                      # nothing cached: nothing to cut
    assert call(pos=5, ns=6) == nqkv.EINVAL                      # more pieces than cached tokens
    assert call(levels=None) == nqkv.EINVAL


def test_decode_multi_argument_errors_and_planning(nqkv):
    lv, lvp = _levels(nqkv)
    d = nqkv.make_desc(1, 32, 128, 4, 64, 32768)
    f = nqkv.lib.nqkv_decode_attention_multi

    def call(q=FAKE, kc=FAKE, ks=FAKE, vc=FAKE, vs=FAKE, seq=32768, q_len=4, scale=1.0, out=FAKE, ws=FAKE,
             ws_bytes=1 << 30, ns=0, desc=d, levels=lvp):
        return f(ctypes.byref(desc), levels, q, kc, ks, vc, vs, seq, q_len, scale, out, ws, ws_bytes, ns, None)

    assert call(q=None) == nqkv.EINVAL
    assert call(out=None) == nqkv.EINVAL
    assert call(ks=FAKE + 2) == nqkv.EINVAL
    assert call(q_len=0) == nqkv.EINVAL
    assert call(q_len=17) == nqkv.EUNSUPPORTED
    assert call(seq=3) == nqkv.EINVAL                            # fewer cached tokens than queries
    assert call(seq=32769) == nqkv.EINVAL
    assert call(scale=float("nan")) == nqkv.EINVAL
    assert call(ns=8, ws=None) == nqkv.EINVAL
    assert call(ns=8, ws_bytes=100) == nqkv.EWORKSPACE
    assert call(ns=1025) == nqkv.EINVAL
    assert call(seq=100, ns=5) == nqkv.EINVAL                    # 100 tokens are four 32-token pieces
    assert call(levels=None) == nqkv.EINVAL
    fv = nqkv.lib.nqkv_decode_attention_multi_varlen
    def callv(lens=FAKE, mx=32768, q_len=4, q=FAKE):
        return fv(ctypes.byref(d), lvp, q, FAKE, FAKE, FAKE, FAKE, lens, mx, q_len, 1.0, FAKE, FAKE, 1 << 30, 0, None)
    assert callv(lens=None) == nqkv.EINVAL
    assert callv(lens=FAKE + 2) == nqkv.EINVAL
    assert callv(mx=32769) == nqkv.EINVAL
    assert callv(mx=3) == nqkv.EINVAL
    assert callv(q=None) == nqkv.EINVAL
    fp_ = nqkv.lib.nqkv_decode_attention_multi_paged
    pd = nqkv.make_desc(4, 8, 128, 4, 64, 256)                   # pages of 256 tokens
    def callp(table=FAKE, stride=16, pages=64, lens=FAKE, mx=4096, q_len=4, desc=pd, ns=0, ws=FAKE):
        return fp_(ctypes.byref(desc), lvp, FAKE, FAKE, FAKE, FAKE, FAKE, table, stride, pages, lens, mx, q_len, 1.0,
                   FAKE, ws, 1 << 30, ns, None)
    assert callp(table=None) == nqkv.EINVAL
    assert callp(table=FAKE + 2) == nqkv.EINVAL
    assert callp(lens=None) == nqkv.EINVAL
    assert callp(stride=0) == nqkv.EINVAL
    assert callp(pages=0) == nqkv.EINVAL
    assert callp(mx=4097) == nqkv.EINVAL                         # more tokens than the table row has pages for
    assert callp(mx=3) == nqkv.EINVAL
    assert callp(q_len=17) == nqkv.EUNSUPPORTED
    assert callp(desc=nqkv.make_desc(4, 8, 128, 4, 64, 200)) == nqkv.EUNSUPPORTED     # page size not a power of two
    assert callp(ns=4, ws=None) == nqkv.EINVAL
    assert nqkv.decode_multi_paged_workspace_bytes(pd, 4096, 4, 4) == (4 * 8 * 4 * 4 * 130 * 4, 4)
    assert nqkv.decode_multi_paged_workspace_bytes(pd, 100000, 4, 1) == (0, 1)       # not bound by the page size
    with pytest.raises(nqkv.NqkvError):
        nqkv.decode_multi_paged_workspace_bytes(nqkv.make_desc(4, 8, 128, 4, 64, 200), 4096, 4, 0)
    # workspace: partial results only, [B*H][splits][q_len][D+2] floats
    assert nqkv.decode_multi_workspace_bytes(d, 32768, 4, 1) == (0, 1)
    assert nqkv.decode_multi_workspace_bytes(d, 32768, 4, 7) == (32 * 7 * 4 * 130 * 4, 7)
    nbytes, splits = nqkv.decode_multi_workspace_bytes(d, 32768, 16, 0)
    assert splits > 1 and nbytes == 32 * splits * 16 * 130 * 4
    assert nqkv.decode_multi_workspace_bytes(d, 40, 8, 0) == (0, 1)
    for seq, ql, ns in ((0, 1, 0), (7, 8, 0), (32769, 1, 0), (64, 1, 3), (64, 1, -1)):
        with pytest.raises(nqkv.NqkvError) as e:
            nqkv.decode_multi_workspace_bytes(d, seq, ql, ns)
        assert e.value.status == nqkv.EINVAL
    assert nqkv.lib.nqkv_decode_multi_workspace_bytes(ctypes.byref(d), 100, 2, 0, None, None) == nqkv.EINVAL


def test_varlen_argument_errors(nqkv):
    lv, lvp = _levels(nqkv)
    d = nqkv.make_desc(4, 8, 128, 4, 64, 4096)
    fa, fs = nqkv.lib.nqkv_decode_attention_varlen, nqkv.lib.nqkv_decode_step_varlen

    def att(lens=FAKE, mx=4096, q=FAKE, ws=FAKE, ns=0, ws_bytes=1 << 30):
        return fa(ctypes.byref(d), lvp, q, FAKE, FAKE, FAKE, FAKE, lens, mx, 1.0, FAKE, ws, ws_bytes, ns, None)

    def step(pos=FAKE, mx=4095, kn=FAKE, ns=0):
        return fs(ctypes.byref(d), lvp, FAKE, kn, FAKE, 1024, 128, FAKE, FAKE, FAKE, FAKE, pos, mx, 1.0, FAKE, FAKE,
                  1 << 30, ns, None)

    assert att(lens=None) == nqkv.EINVAL
    assert att(lens=FAKE + 2) == nqkv.EINVAL                     # int32 alignment
    assert att(mx=0) == nqkv.EINVAL
    assert att(mx=4097) == nqkv.EINVAL                           # bound above the capacity
    assert att(q=None) == nqkv.EINVAL
    assert att(ns=4, ws=None) == nqkv.EINVAL
    assert att(ns=4, ws_bytes=64) == nqkv.EWORKSPACE
    assert step(pos=None) == nqkv.EINVAL
    assert step(mx=4096) == nqkv.EINVAL                          # no row left for the new token
    assert step(mx=-1) == nqkv.EINVAL
    assert step(kn=None) == nqkv.EINVAL
    assert step(mx=0, ns=2) == nqkv.EINVAL


def test_paged_argument_errors(nqkv):
    lv, lvp = _levels(nqkv)
    d = nqkv.make_desc(4, 8, 128, 4, 64, 256)                     # pages of 256 tokens
    assert nqkv.decode_paged_workspace_bytes(d, 256) == (0, 1)
    assert nqkv.decode_paged_workspace_bytes(d, 257) == (262144 + 4 * 8 * 2 * 130 * 4, 2)
    assert nqkv.decode_paged_workspace_bytes(d, 256 * 1024 + 1)[1] == 8        # 1025 pages in 8 runs of whole pages
    for bad_page in (64, 192, 1000):                               # not a power of two >= 128
        with pytest.raises(nqkv.NqkvError) as e:
            nqkv.decode_paged_workspace_bytes(nqkv.make_desc(4, 8, 128, 4, 64, bad_page), 4096)
        assert e.value.status == nqkv.EUNSUPPORTED
    fa, fs = nqkv.lib.nqkv_decode_attention_paged, nqkv.lib.nqkv_decode_step_paged

    def att(table=FAKE, stride=16, pages=100, lens=FAKE, mx=4096, ws=FAKE, ws_bytes=1 << 30, q=FAKE):
        return fa(ctypes.byref(d), lvp, q, FAKE, FAKE, FAKE, FAKE, table, stride, pages, lens, mx, 1.0, FAKE, ws,
                  ws_bytes, None)

    def step(table=FAKE, stride=17, pages=100, pos=FAKE, mx=4096, kn=FAKE):
        return fs(ctypes.byref(d), lvp, FAKE, kn, FAKE, 1024, 128, FAKE, FAKE, FAKE, FAKE, table, stride, pages, pos, mx,
                  1.0, FAKE, FAKE, 1 << 30, None)

    assert att(table=None) == nqkv.EINVAL
    assert att(table=FAKE + 2) == nqkv.EINVAL
    assert att(lens=None) == nqkv.EINVAL
    assert att(stride=15) == nqkv.EINVAL                          # 4096 tokens need 16 table columns
    assert att(pages=0) == nqkv.EINVAL
    assert att(mx=0) == nqkv.EINVAL
    assert att(ws=None) == nqkv.EINVAL
    assert att(ws_bytes=1000) == nqkv.EWORKSPACE
    assert att(q=None) == nqkv.EINVAL
    assert step(stride=16) == nqkv.EINVAL                         # row 4096 opens page 16: 17 columns
    assert step(kn=None) == nqkv.EINVAL
    assert step(pos=None) == nqkv.EINVAL
    assert step(mx=-1) == nqkv.EINVAL


def test_quantize_paged_argument_errors(nqkv):
    lv, lvp = _levels(nqkv)
    d = nqkv.make_desc(2, 8, 64, 4, 64, 256)                      # pages of 256 tokens
    f = nqkv.lib.nqkv_quantize_kv_paged

    def call(desc=d, n=300, off=0, table=FAKE, stride=4, pages=50, ks=FAKE, kc=FAKE, ksc=FAKE, vs=None, vc=None,
             vsc=None, st=64):
        return f(ctypes.byref(desc), lvp, ks, vs, 8 * 300 * 64, 300 * 64, st, n, off, table, stride, pages,
                 kc, ksc, vc, vsc, None)

    assert call(n=0) == nqkv.OK
    assert call(table=None) == nqkv.EINVAL
    assert call(table=FAKE + 1) == nqkv.EINVAL
    assert call(pages=0) == nqkv.EINVAL
    assert call(stride=1) == nqkv.EINVAL                          # 300 tokens need two table columns
    assert call(off=800) == nqkv.EINVAL                           # 800 + 300 tokens: beyond four pages
    assert call(off=-1) == nqkv.EINVAL
    assert call(ks=None) == nqkv.EINVAL
    assert call(vs=FAKE) == nqkv.EINVAL
    assert call(st=60) == nqkv.EINVAL
    assert call(desc=nqkv.make_desc(2, 8, 64, 4, 64, 100)) == nqkv.EUNSUPPORTED   # page size not a power of two


def test_quantize_varlen_argument_errors(nqkv):
    lv, lvp = _levels(nqkv)
    d = nqkv.make_desc(2, 4, 64, 4, 64, 1000)
    f = nqkv.lib.nqkv_quantize_kv_pair_varlen

    def call(offs=FAKE, mx=900, n=100, ks=FAKE, desc=d):
        return f(ctypes.byref(desc), lvp, FAKE, FAKE, 0, 0, 64, n, offs, mx, FAKE, ks, FAKE, FAKE, None)

    assert call(offs=None) == nqkv.EINVAL
    assert call(offs=FAKE + 2) == nqkv.EINVAL
    assert call(mx=901) == nqkv.EINVAL                           # max_offset + n_tokens beyond the capacity
    assert call(mx=-1) == nqkv.EINVAL
    assert call(mx=1 << 31) == nqkv.EINVAL
    assert call(ks=None) == nqkv.EINVAL
    assert call(n=0) == nqkv.OK                                  # nothing to do
    fp_ = nqkv.lib.nqkv_quantize_kv_paged_varlen
    pd = nqkv.make_desc(2, 4, 64, 4, 64, 256)

    def callp(offs=FAKE, mx=1000, n=24, table=FAKE, stride=4, pages=16, desc=pd):
        return fp_(ctypes.byref(desc), lvp, FAKE, FAKE, 0, 0, 64, n, offs, mx, table, stride, pages, FAKE, FAKE, FAKE, FAKE, None)

    assert callp(offs=None) == nqkv.EINVAL
    assert callp(offs=FAKE + 1) == nqkv.EINVAL
    assert callp(mx=1001) == nqkv.EINVAL                         # rows beyond table_stride * P
    assert callp(table=None) == nqkv.EINVAL
    assert callp(pages=0) == nqkv.EINVAL
    assert callp(desc=nqkv.make_desc(2, 4, 64, 4, 64, 100)) == nqkv.EUNSUPPORTED
    assert callp(n=0) == nqkv.OK


def test_quantize_hidden_argument_errors(nqkv):
    lv, lvp = _levels(nqkv)
    f = nqkv.lib.nqkv_quantize_kv_hidden

    def call(desc, sb=32 * 100 * 64, sh=64, st=32 * 64, n=100, off=0, blk=256, ks=FAKE, kc=FAKE, ksc=FAKE,
             vs=None, vc=None, vsc=None, levels=lvp):
        return f(ctypes.byref(desc), levels, ks, vs, sb, sh, st, n, off, blk, kc, ksc, vc, vsc, None)

    d = nqkv.make_desc(2, 32, 64, 4, 64, 128)                     # one scale per token-head
    assert call(d, n=0) == nqkv.OK                                 # nothing to do
    assert call(nqkv.make_desc(2, 32, 128, 4, 64, 128)) == nqkv.EINVAL      # two scales per token-head
    assert call(d, blk=512) == nqkv.EUNSUPPORTED
    assert call(d, blk=64, ks=None) == nqkv.EINVAL                 # one head per block: the ordinary call's checks
    assert call(nqkv.make_desc(2, 3, 64, 4, 64, 128)) == nqkv.EINVAL        # 3 heads of 64: 192 is not a multiple of 256
    assert call(nqkv.make_desc(2, 3, 128, 4, 128, 128), blk=256) == nqkv.EINVAL
    assert call(d, sh=32) == nqkv.EINVAL                           # heads would overlap
    assert call(d, st=2052) == nqkv.EINVAL                         # rows must stay 16-byte aligned
    assert call(d, ks=None) == nqkv.EINVAL
    assert call(d, kc=FAKE + 8) == nqkv.EINVAL
    assert call(d, vs=FAKE) == nqkv.EINVAL                         # half a pair
    assert call(d, n=100, off=29) == nqkv.EINVAL                   # past the capacity
    assert call(d, levels=None) == nqkv.EINVAL
    big = nqkv.make_desc(1, 32, 128, 4, 128, 1 << 20)              # 2 GiB of codes per batch row
    assert call(big, sh=128, st=32 * 128, sb=0, n=1) == nqkv.EUNSUPPORTED


def test_many_sequences_are_accepted_uncut_and_refused_cut(nqkv):
    """More than 65535 (batch row, head) pairs: fine for every call that keeps sequences whole (the
    automatic plan never cuts them at that count); cutting them needs one counter per pair and is
    refused beyond the counter table, before any GPU work."""
    d = nqkv.make_desc(1100, 64, 64, 4, 64, 4096)                  # 70400 pairs
    need, splits = nqkv.decode_workspace_bytes(d, 4096, 0)
    assert (need, splits) == (0, 1)
    need = ctypes.c_size_t(); sp = ctypes.c_int()
    f = nqkv.lib.nqkv_decode_workspace_bytes
    assert f(ctypes.byref(d), 4096, 1, ctypes.byref(need), ctypes.byref(sp)) == nqkv.OK
    assert f(ctypes.byref(d), 4096, 2, ctypes.byref(need), ctypes.byref(sp)) == nqkv.EUNSUPPORTED
    fm = nqkv.lib.nqkv_decode_multi_workspace_bytes
    assert fm(ctypes.byref(d), 4096, 4, 0, ctypes.byref(need), ctypes.byref(sp)) == nqkv.OK and sp.value == 1
    assert fm(ctypes.byref(d), 4096, 4, 2, ctypes.byref(need), ctypes.byref(sp)) == nqkv.EUNSUPPORTED
    lv, lvp = _levels(nqkv)
    fa = nqkv.lib.nqkv_decode_attention
    args = (lvp, FAKE, FAKE, FAKE, FAKE, FAKE, 4096, 1.0, FAKE)
    assert fa(ctypes.byref(d), *args, FAKE, 1 << 30, 2, None) == nqkv.EUNSUPPORTED
    assert nqkv.lib.nqkv_decode_attention_static(ctypes.byref(d), *args, 2, None) == nqkv.EUNSUPPORTED


def test_benchaux_library_exports_and_argument_errors():
    """The measurement helpers live in a library of their own; the product library exports none."""
    from paper_2505_16210_amd import benchaux
    header = open(os.path.join(ROOT, "include", "nqkv_benchaux.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    assert set(re.findall(r"\b(nqkv_aux_[a-z_0-9]+)\s*\(", header)) == set(benchaux.EXPORTS)
    f = benchaux.lib.nqkv_aux_read_stream
    assert f(None, 1024, FAKE, None) == -1
    assert f(FAKE, 1024, None, None) == -1
    assert f(FAKE + 4, 1024, FAKE, None) == -1
    assert f(FAKE, 1000, FAKE, None) == -1                       # whole 16-byte vectors only
    assert benchaux.lib.nqkv_aux_copy(FAKE, FAKE + 8, 1024, None) == -1
    assert benchaux.lib.nqkv_aux_copy(FAKE, FAKE, 0, None) == 0
    tiles = ctypes.c_size_t(7)
    m = benchaux.lib.nqkv_aux_mix_stream
    assert m(FAKE, 1 << 20, FAKE, 1 << 20, 3, 1, ctypes.byref(tiles), None) == -1     # only 4:1, 1:4, 1:1
    assert m(None, 1 << 20, FAKE, 1 << 20, 4, 1, ctypes.byref(tiles), None) == -1
    assert m(FAKE, 1 << 20, FAKE + 4, 1 << 20, 4, 1, ctypes.byref(tiles), None) == -1
    assert m(FAKE, 16383, FAKE, 1 << 20, 4, 1, ctypes.byref(tiles), None) == 0 and tiles.value == 0   # no whole tile: nothing launched


def test_per_call_flags(nqkv):
    """Options travel in the descriptor (the library keeps no settings): the two defined bits are
    accepted by planning calls, anything else is refused."""
    for flags in (0, nqkv.FLAG_SCAN_QUANTIZER, nqkv.FLAG_WORKGROUP_PER_ITEM, 3):
        d = nqkv.make_desc(2, 4, 128, 4, 64, 4096, flags=flags)
        assert nqkv.decode_workspace_bytes(d, 4096, 4)[1] == 4
    for flags in (4, 8, 1 << 30, -1):
        with pytest.raises(nqkv.NqkvError) as e:
            nqkv.decode_workspace_bytes(nqkv.make_desc(2, 4, 128, 4, 64, 4096, flags=flags), 4096, 4)
        assert e.value.status == nqkv.EINVAL
    assert not any("tuning" in name or "probe" in name for name in nqkv.EXPORTS)
