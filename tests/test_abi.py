"""The C-ABI library loads without a GPU, exports every symbol include/sirllm.h declares, and
rejects bad arguments on the host before anything is launched.  CPU only: no compute calls."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def b():
    from paper_2405_12528_amd import build
    if not os.path.exists(build.LIB):
        build.build()
    from paper_2405_12528_amd import binding
    return binding


def declared_functions():
    text = open(os.path.join(ROOT, "include", "sirllm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sirllm_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(b):
    names = declared_functions()
    assert set(names) >= {"sirllm_score", "sirllm_decay_select", "sirllm_compact_kv", "sirllm_step"}
    for n in names:
        assert hasattr(b.raw(), n), f"{n} is declared in sirllm.h but not exported by libsirllm.so"
    assert set(b.EXPORTS) == set(names)


def test_status_strings_and_version(b):
    assert b.sirllm_status_string(0) == "ok"
    for code in (-1, -2, -3, -4):
        assert len(b.sirllm_status_string(code)) > 5
    assert re.fullmatch(r"\d+\.\d+\.\d+", b.sirllm_version())
    assert b.sirllm_workspace_bytes(32, 2304, 8192, 32000) % 256 == 0


def test_struct_sizes_match_the_header(b):
    # int32 x3 + float; int32 x4 + int64 x4
    assert C.sizeof(b.sirllm_policy) == 16
    assert C.sizeof(b.sirllm_kv_layout) == 48


FAKE = 0x1000  # a non-null, 16-byte aligned "pointer"; validation never dereferences it


def test_score_argument_errors(b):
    L = b.raw()
    assert L.sirllm_score(FAKE, 7, 4, 10, 10, FAKE, FAKE, None, 0, None) == b.SIRLLM_ERR_UNSUPPORTED   # dtype
    assert L.sirllm_score(FAKE, 0, -1, 10, 10, FAKE, FAKE, None, 0, None) == b.SIRLLM_ERR_INVALID_ARG
    assert L.sirllm_score(FAKE, 0, 4, 0, 10, FAKE, FAKE, None, 0, None) == b.SIRLLM_ERR_INVALID_ARG    # vocab < 1
    assert L.sirllm_score(FAKE, 0, 4, 10, 9, FAKE, FAKE, None, 0, None) == b.SIRLLM_ERR_INVALID_ARG    # ld < vocab
    assert L.sirllm_score(None, 0, 4, 10, 10, FAKE, FAKE, None, 0, None) == b.SIRLLM_ERR_INVALID_ARG
    assert L.sirllm_score(FAKE, 0, 4, 10, 10, None, FAKE, None, 0, None) == b.SIRLLM_ERR_INVALID_ARG
    assert L.sirllm_score(FAKE, 0, 4, 10, 10, FAKE, None, None, 0, None) == b.SIRLLM_ERR_INVALID_ARG
    assert L.sirllm_score(FAKE + 2, 0, 4, 10, 10, FAKE, FAKE, None, 0, None) == b.SIRLLM_ERR_INVALID_ARG  # f32 at +2
    assert L.sirllm_score(FAKE, 0, 2**31, 10, 10, FAKE, FAKE, None, 0, None) == b.SIRLLM_ERR_UNSUPPORTED
    assert L.sirllm_score(None, 0, 0, 10, 10, None, None, None, 0, None) == b.SIRLLM_OK                 # empty


def test_decay_select_static_rejects_on_the_host(b):
    """The entry point without a workspace validates like sirllm_decay_select and refuses, before anything is
    launched, sizes whose scratch exceeds its static array."""
    L = b.raw()
    p = b.sirllm_policy(4, 20000, 512, 0.9)

    def call(n_streams, n_held, n_new, scores=FAKE):
        n_cand = n_held + n_new
        return L.sirllm_decay_select_static(scores, n_cand, n_streams, n_held, n_new, C.byref(p), FAKE + (1 << 40), 20516,
                                            FAKE + (1 << 41), 20516, None)
    assert call(300, 39000, 1000) == b.SIRLLM_ERR_UNSUPPORTED          # 300 x 4352 bytes > 1 MiB
    assert call(52, 16777216 - 4096, 4096) == b.SIRLLM_ERR_UNSUPPORTED  # 52 x 20480 bytes > 1 MiB
    assert call(1, 16777216, 1) == b.SIRLLM_ERR_UNSUPPORTED             # above SIRLLM_MAX_CAND
    assert call(1, -1, 5) == b.SIRLLM_ERR_INVALID_ARG
    assert call(1, 39000, 1000, scores=None) == b.SIRLLM_ERR_INVALID_ARG
    assert call(0, 39000, 1000) == b.SIRLLM_OK                          # no streams: nothing to do
    assert b.SIRLLM_STATIC_SCRATCH_BYTES == 1048576
    text = open(os.path.join(ROOT, "include", "sirllm.h")).read()
    assert re.search(r"#define\s+SIRLLM_STATIC_SCRATCH_BYTES\s+1048576\b", text)


def test_decay_select_argument_errors(b):
    L = b.raw()
    p = b.sirllm_policy(4, 20, 8, 0.9)
    def call(scores=FAKE, stride=100, n_streams=1, n_held=60, n_new=40, pol=p, idx=FAKE + 0x10000, istr=32,
             out=FAKE + 0x20000, ostr=32):
        return L.sirllm_decay_select(scores, stride, n_streams, n_held, n_new, C.byref(pol) if pol else None,
                                     idx, istr, out, ostr, None, 0, None)
    assert call(n_held=-1) == b.SIRLLM_ERR_INVALID_ARG
    assert call(n_streams=-1) == b.SIRLLM_ERR_INVALID_ARG
    assert call(pol=None) == b.SIRLLM_ERR_INVALID_ARG
    assert call(pol=b.sirllm_policy(-1, 20, 8, 0.9)) == b.SIRLLM_ERR_INVALID_ARG
    assert call(pol=b.sirllm_policy(4, 20, 8, float("nan"))) == b.SIRLLM_ERR_INVALID_ARG
    assert call(pol=b.sirllm_policy(4, 20, 8, -0.5)) == b.SIRLLM_ERR_INVALID_ARG
    assert call(pol=b.sirllm_policy(4, 20, 8, float("inf"))) == b.SIRLLM_ERR_INVALID_ARG
    assert call(scores=None) == b.SIRLLM_ERR_INVALID_ARG
    assert call(idx=None) == b.SIRLLM_ERR_INVALID_ARG
    assert call(out=None) == b.SIRLLM_ERR_INVALID_ARG
    assert call(stride=99) == b.SIRLLM_ERR_INVALID_ARG          # stride < n_cand
    assert call(istr=31) == b.SIRLLM_ERR_INVALID_ARG            # idx_stride < n_keep
    assert call(ostr=31) == b.SIRLLM_ERR_INVALID_ARG
    assert call(out=FAKE + 16) == b.SIRLLM_ERR_INVALID_ARG      # scores_out overlaps scores
    assert call(n_held=b.SIRLLM_MAX_CAND, n_new=1, stride=40000) == b.SIRLLM_ERR_UNSUPPORTED
    assert call(n_streams=0) == b.SIRLLM_OK
    assert call(n_held=0, n_new=0) == b.SIRLLM_OK
    # budget sums that overflow int32 are fine: the sum is taken in 64 bits and n_cand <= budget keeps all
    assert call(pol=b.sirllm_policy(2**31 - 1, 2**31 - 1, 2**31 - 1, 1.0), n_streams=0) == b.SIRLLM_OK


def test_compact_kv_argument_errors(b):
    L = b.raw()
    lay = lambda **kw: b.sirllm_kv_layout(**{**dict(n_layers=2, n_kv_heads=2, head_dim=16, elem_bytes=4,
                                                    stride_stream=2 * 2 * 64 * 16, stride_layer=2 * 64 * 16,
                                                    stride_head=64 * 16, stride_pos=16), **kw})
    S, D = lay(), lay()
    src, dst, idx = 0x100000, 0x900000, 0x50000
    def call(ks=src, vs=None, s=S, n_src=64, kd=dst, vd=None, d=D, ix=idx, istr=32, n_streams=1, n_keep=32):
        return L.sirllm_compact_kv(ks, vs, C.byref(s) if s else None, n_src, kd, vd, C.byref(d) if d else None,
                                   ix, istr, n_streams, n_keep, None)
    assert call(s=None) == b.SIRLLM_ERR_INVALID_ARG
    assert call(d=lay(head_dim=8)) == b.SIRLLM_ERR_INVALID_ARG           # layouts disagree
    assert call(d=lay(elem_bytes=2)) == b.SIRLLM_ERR_INVALID_ARG
    assert call(s=lay(elem_bytes=3), d=lay(elem_bytes=3)) == b.SIRLLM_ERR_INVALID_ARG
    assert call(s=lay(stride_pos=8)) == b.SIRLLM_ERR_INVALID_ARG         # rows would overlap
    assert call(s=lay(stride_head=-1)) == b.SIRLLM_ERR_INVALID_ARG
    assert call(ks=None) == b.SIRLLM_ERR_INVALID_ARG
    assert call(kd=None) == b.SIRLLM_ERR_INVALID_ARG
    assert call(ix=None) == b.SIRLLM_ERR_INVALID_ARG
    assert call(vs=src + 0x400000) == b.SIRLLM_ERR_INVALID_ARG           # V source without V destination
    assert call(n_keep=-1) == b.SIRLLM_ERR_INVALID_ARG
    assert call(istr=31) == b.SIRLLM_ERR_INVALID_ARG
    assert call(kd=src + 64) == b.SIRLLM_ERR_INVALID_ARG                 # destination overlaps source
    assert call(ks=src + 2) == b.SIRLLM_ERR_INVALID_ARG                  # 4-byte elements at an odd address
    assert call(n_keep=0) == b.SIRLLM_OK
    assert call(n_streams=0) == b.SIRLLM_OK


def test_compact_kv_layers_argument_errors(b):
    L = b.raw()
    lay = lambda **kw: b.sirllm_kv_layout(**{**dict(n_layers=3, n_kv_heads=2, head_dim=16, elem_bytes=4,
                                                    stride_stream=2 * 64 * 16, stride_layer=12345, stride_head=64 * 16,
                                                    stride_pos=16), **kw})
    one = 2 * 64 * 16 * 4                                # bytes of one layer's buffer (one stream)
    arr = lambda *ptrs: (C.c_void_p * len(ptrs))(*ptrs)
    ksrc, kdst = arr(0x100000, 0x200000, 0x300000), arr(0x900000, 0xa00000, 0xb00000)
    vsrc, vdst = arr(0x400000, 0x500000, 0x600000), arr(0xc00000, 0xd00000, 0xe00000)
    def call(ks=ksrc, vs=None, s=lay(), n_src=64, kd=kdst, vd=None, d=lay(), ix=0x50000, istr=32, n_streams=1, n_keep=32):
        return L.sirllm_compact_kv_layers(ks, vs, C.byref(s) if s else None, n_src, kd, vd, C.byref(d) if d else None,
                                          ix, istr, n_streams, n_keep, None)
    assert call(s=None) == b.SIRLLM_ERR_INVALID_ARG
    assert call(d=lay(n_layers=2)) == b.SIRLLM_ERR_INVALID_ARG                     # layer counts disagree
    assert call(d=lay(head_dim=8)) == b.SIRLLM_ERR_INVALID_ARG
    assert call(ks=None) == b.SIRLLM_ERR_INVALID_ARG
    assert call(kd=None) == b.SIRLLM_ERR_INVALID_ARG
    assert call(ix=None) == b.SIRLLM_ERR_INVALID_ARG
    assert call(istr=31) == b.SIRLLM_ERR_INVALID_ARG
    assert call(vs=vsrc) == b.SIRLLM_ERR_INVALID_ARG                               # V source without V destination
    assert call(ks=arr(0x100000, 0, 0x300000)) == b.SIRLLM_ERR_INVALID_ARG         # a layer without a buffer
    assert call(ks=arr(0x100000, 0x200002, 0x300000)) == b.SIRLLM_ERR_INVALID_ARG  # 4-byte elements at an odd address
    assert call(kd=arr(0x900000, 0x200000 + 64, 0xb00000)) == b.SIRLLM_ERR_INVALID_ARG   # a destination inside a source
    assert call(kd=arr(0x900000, 0x900000 + one // 2, 0xb00000)) == b.SIRLLM_ERR_INVALID_ARG   # two destinations overlap
    assert call(vs=vsrc, vd=arr(0xc00000, 0xd00000, 0x900000)) == b.SIRLLM_ERR_INVALID_ARG    # V destination on a K destination
    assert call(n_keep=-1) == b.SIRLLM_ERR_INVALID_ARG
    assert call(n_keep=0) == b.SIRLLM_OK and call(n_streams=0) == b.SIRLLM_OK
    assert call(s=lay(n_layers=0), d=lay(n_layers=0)) == b.SIRLLM_OK
    # stride_layer is ignored: adjacent one-layer buffers are fine whatever it says
    assert one == 0x2000


def test_compact_kv_inplace_layers_argument_errors(b):
    L = b.raw()
    lay = lambda **kw: b.sirllm_kv_layout(**{**dict(n_layers=3, n_kv_heads=2, head_dim=16, elem_bytes=4,
                                                    stride_stream=2 * 64 * 16, stride_layer=999, stride_head=64 * 16,
                                                    stride_pos=16), **kw})
    arr = lambda *ptrs: (C.c_void_p * len(ptrs))(*ptrs)
    ks = arr(0x100000, 0x200000, 0x300000)
    def call(k=ks, v=None, l=lay(), n_src=64, ix=0x50000, istr=32, n_streams=1, n_keep=32, ws=None, ws_bytes=0):
        return L.sirllm_compact_kv_inplace_layers(k, v, C.byref(l) if l else None, n_src, ix, istr, n_streams, n_keep,
                                                  ws, ws_bytes, None)
    assert call(l=None) == b.SIRLLM_ERR_INVALID_ARG
    assert call(k=None) == b.SIRLLM_ERR_INVALID_ARG
    assert call(ix=None) == b.SIRLLM_ERR_INVALID_ARG
    assert call(n_keep=65) == b.SIRLLM_ERR_INVALID_ARG                             # cannot keep more than there is
    assert call(istr=31) == b.SIRLLM_ERR_INVALID_ARG
    assert call(k=arr(0x100000, 0, 0x300000)) == b.SIRLLM_ERR_INVALID_ARG          # a layer without a buffer
    assert call(k=arr(0x100000, 0x200002, 0x300000)) == b.SIRLLM_ERR_INVALID_ARG
    assert call(k=arr(0x100000, 0x100000 + 64, 0x300000)) == b.SIRLLM_ERR_INVALID_ARG   # two layers overlap
    assert call(v=arr(0x400000, 0x300000, 0x600000)) == b.SIRLLM_ERR_INVALID_ARG        # a V buffer on a K buffer
    assert call(ws=0x30000001, ws_bytes=1 << 20) == b.SIRLLM_ERR_WORKSPACE
    assert call(n_keep=0) == b.SIRLLM_OK and call(n_streams=0) == b.SIRLLM_OK
    assert call(l=lay(n_layers=0)) == b.SIRLLM_OK


def test_score_select_argument_errors(b):
    L = b.raw()
    p = b.sirllm_policy(4, 20, 8, 0.9)
    def call(logits=0x1000, dt=0, vocab=1000, ld=1000, tok=0x2000000, scores=0x3000000, sstr=128, n_streams=1, n_held=32,
             n_new=64, pol=p, idx=0x5000000, istr=32, out=0x6000000, ostr=32, ws=None, ws_bytes=0):
        return L.sirllm_score_select(logits, dt, vocab, ld, tok, scores, sstr, n_streams, n_held, n_new,
                                     C.byref(pol) if pol else None, idx, istr, out, ostr, ws, ws_bytes, None)
    assert call(dt=7) == b.SIRLLM_ERR_UNSUPPORTED
    assert call(logits=None) == b.SIRLLM_ERR_INVALID_ARG
    assert call(tok=None) == b.SIRLLM_ERR_INVALID_ARG
    assert call(ld=999) == b.SIRLLM_ERR_INVALID_ARG
    assert call(pol=None) == b.SIRLLM_ERR_INVALID_ARG
    assert call(scores=None) == b.SIRLLM_ERR_INVALID_ARG
    assert call(sstr=95) == b.SIRLLM_ERR_INVALID_ARG                    # scores_stride < n_cand
    assert call(idx=None) == b.SIRLLM_ERR_INVALID_ARG
    assert call(istr=31) == b.SIRLLM_ERR_INVALID_ARG
    assert call(out=None) == b.SIRLLM_ERR_INVALID_ARG
    assert call(n_new=-1) == b.SIRLLM_ERR_INVALID_ARG
    assert call(n_held=40000, n_new=64, sstr=40064) == b.SIRLLM_ERR_WORKSPACE   # above 32768 slots the selection needs scratch
    assert call(n_streams=0) == b.SIRLLM_OK
    assert call(n_held=0, n_new=0, logits=None, tok=None) == b.SIRLLM_OK


def test_step_argument_errors(b):
    L = b.raw()
    p = b.sirllm_policy(4, 20, 8, 0.9)
    lay = b.sirllm_kv_layout(2, 2, 16, 4, 2 * 2 * 128 * 16, 2 * 128 * 16, 128 * 16, 16)
    def call(logits=0x1000, dt=0, vocab=1000, ld=1000, tok=0x2000000, scores=0x3000000, sstr=128, n_streams=1,
             n_held=32, n_new=64, ksrc=0x10000000, vsrc=0x20000000, kdst=0x30000000, vdst=0x40000000,
             idx=0x5000000, istr=32, out=0x6000000, ostr=32):
        return L.sirllm_step(logits, dt, vocab, ld, tok, scores, sstr, n_streams, n_held, n_new, C.byref(p),
                             ksrc, vsrc, C.byref(lay), kdst, vdst, C.byref(lay), idx, istr, out, ostr, None, 0, None)
    assert call(dt=5) == b.SIRLLM_ERR_UNSUPPORTED
    assert call(logits=None) == b.SIRLLM_ERR_INVALID_ARG
    assert call(ld=999) == b.SIRLLM_ERR_INVALID_ARG
    assert call(scores=None) == b.SIRLLM_ERR_INVALID_ARG
    assert call(n_new=-1) == b.SIRLLM_ERR_INVALID_ARG
    assert call(kdst=None) == b.SIRLLM_ERR_INVALID_ARG              # eviction needs a destination
    assert call(kdst=0x10000000 + 4096) == b.SIRLLM_ERR_INVALID_ARG  # ... that does not overlap the source
    assert call(n_held=b.SIRLLM_MAX_CAND) == b.SIRLLM_ERR_UNSUPPORTED
    assert call(n_streams=0, logits=None, tok=None) == b.SIRLLM_OK


def test_baseline_select_argument_errors(b):
    L = b.raw()
    p = b.sirllm_policy(4, 20, 8, 0.0)
    n_keep = C.c_int32(-5)
    def call(kind=1, n_streams=1, n_cand=100, pol=p, idx=FAKE, istr=32, out=n_keep, ws=None, ws_bytes=0):
        return L.sirllm_baseline_select(kind, n_streams, n_cand, C.byref(pol) if pol else None, 1, 2, idx, istr,
                                        C.byref(out) if out is not None else None, ws, ws_bytes, None)
    assert call(kind=3) == b.SIRLLM_ERR_UNSUPPORTED
    assert call(pol=None) == b.SIRLLM_ERR_INVALID_ARG
    assert call(pol=b.sirllm_policy(4, -1, 8, 0.0)) == b.SIRLLM_ERR_INVALID_ARG
    assert call(n_cand=-1) == b.SIRLLM_ERR_INVALID_ARG
    assert call(n_cand=b.SIRLLM_MAX_CAND + 1) == b.SIRLLM_ERR_UNSUPPORTED
    # random subsets of more slots than one workgroup holds need the selection's scratch
    need = b.sirllm_workspace_bytes(1, 40000, 0, 0)
    assert need > 0
    assert call(kind=2, n_cand=40000, istr=40000) == b.SIRLLM_ERR_WORKSPACE
    assert call(kind=2, n_cand=40000, istr=40000, ws=0x30000000, ws_bytes=need - 1) == b.SIRLLM_ERR_WORKSPACE
    assert call(kind=2, n_cand=40000, istr=40000, ws=0x30000010, ws_bytes=need) == b.SIRLLM_ERR_WORKSPACE
    assert call(idx=None) == b.SIRLLM_ERR_INVALID_ARG
    assert call(istr=31) == b.SIRLLM_ERR_INVALID_ARG
    assert call(n_streams=0) == b.SIRLLM_OK and n_keep.value == 32       # the kept count is host arithmetic
    assert call(kind=0, n_streams=0) == b.SIRLLM_OK and n_keep.value == 12
    assert call(n_streams=0, n_cand=10) == b.SIRLLM_OK and n_keep.value == 10
    assert call(n_streams=0, out=None) == b.SIRLLM_OK


def test_inplace_and_ragged_argument_errors(b):
    L = b.raw()
    lay = b.sirllm_kv_layout(2, 2, 16, 4, 2 * 2 * 128 * 16, 2 * 128 * 16, 128 * 16, 16)
    def inplace(k=0x10000000, v=None, l=lay, n_src=100, idx=0x5000000, istr=32, n_streams=1, n_keep=32, ws=None, ws_bytes=0):
        return L.sirllm_compact_kv_inplace(k, v, C.byref(l) if l else None, n_src, idx, istr, n_streams, n_keep, ws, ws_bytes, None)
    assert inplace(l=None) == b.SIRLLM_ERR_INVALID_ARG
    assert inplace(k=None) == b.SIRLLM_ERR_INVALID_ARG
    assert inplace(idx=None) == b.SIRLLM_ERR_INVALID_ARG
    assert inplace(n_keep=101) == b.SIRLLM_ERR_INVALID_ARG            # cannot keep more than there is
    assert inplace(istr=31) == b.SIRLLM_ERR_INVALID_ARG
    assert inplace(v=0x10000000 + 64) == b.SIRLLM_ERR_INVALID_ARG     # K and V overlap
    assert inplace(k=0x10000002) == b.SIRLLM_ERR_INVALID_ARG
    assert inplace(n_keep=0) == b.SIRLLM_OK and inplace(n_streams=0) == b.SIRLLM_OK
    assert inplace(ws=0x30000001, ws_bytes=1 << 20) == b.SIRLLM_ERR_WORKSPACE      # not 256-byte aligned
    text = open(os.path.join(ROOT, "include", "sirllm.h")).read()
    assert re.search(r"#define\s+SIRLLM_INPLACE_WORKSPACE_BYTES\s+256\b", text) and b.SIRLLM_INPLACE_WORKSPACE_BYTES == 256
    p = b.sirllm_policy(4, 20, 8, 0.9)
    def ragged(logits=0x1000, dt=0, vocab=1000, ld=1000, tok=0x2000000, scores=0x3000000, sstr=128, n_streams=2,
               held=0x7000000, cu=0x7100000, total=64, max_cand=100, max_new=64, pol=p, k=0x10000000, v=0x20000000,
               l=lay, idx=0x5000000, istr=32, out=0x6000000, ostr=32, keep=0x7200000, ws=None, ws_bytes=0):
        return L.sirllm_step_ragged(logits, dt, vocab, ld, tok, scores, sstr, n_streams, held, cu, total, max_cand,
                                    max_new, C.byref(pol) if pol else None, k, v, C.byref(l) if l else None, idx, istr, out,
                                    ostr, keep, ws, ws_bytes, None)
    assert ragged(dt=9) == b.SIRLLM_ERR_UNSUPPORTED
    assert ragged(total=-1) == b.SIRLLM_ERR_INVALID_ARG
    assert ragged(logits=None) == b.SIRLLM_ERR_INVALID_ARG
    assert ragged(pol=None) == b.SIRLLM_ERR_INVALID_ARG
    assert ragged(max_cand=b.SIRLLM_MAX_CAND + 1, sstr=1 << 25) == b.SIRLLM_ERR_UNSUPPORTED
    # above 32768 slots per stream the selection needs its scratch
    assert ragged(max_cand=40000, sstr=40000) == b.SIRLLM_ERR_WORKSPACE
    assert ragged(max_cand=40000, sstr=40000, ws=0x30000000, ws_bytes=b.sirllm_workspace_bytes(2, 40000, 0, 0) - 1) == b.SIRLLM_ERR_WORKSPACE
    assert ragged(ws=0x30000001, ws_bytes=4096) == b.SIRLLM_ERR_WORKSPACE          # optional, but aligned when given
    assert ragged(max_new=-1) == b.SIRLLM_ERR_INVALID_ARG
    assert ragged(max_new=101) == b.SIRLLM_ERR_INVALID_ARG              # more new tokens than candidates
    assert ragged(held=None) == b.SIRLLM_ERR_INVALID_ARG
    assert ragged(cu=None) == b.SIRLLM_ERR_INVALID_ARG
    assert ragged(keep=None) == b.SIRLLM_ERR_INVALID_ARG
    assert ragged(sstr=99) == b.SIRLLM_ERR_INVALID_ARG                 # scores_stride < max_cand
    assert ragged(istr=31) == b.SIRLLM_ERR_INVALID_ARG
    assert ragged(k=None) == b.SIRLLM_ERR_INVALID_ARG                  # max_cand > budget: a cache is needed
    assert ragged(l=None) == b.SIRLLM_ERR_INVALID_ARG
    assert ragged(n_streams=0) == b.SIRLLM_OK

    lay_dst = b.sirllm_kv_layout(2, 2, 16, 4, 2 * 2 * 32 * 16, 2 * 32 * 16, 32 * 16, 16)
    def ragged_oop(logits=0x1000, dt=0, vocab=1000, ld=1000, tok=0x2000000, scores=0x3000000, sstr=128, n_streams=2,
                   held=0x7000000, cu=0x7100000, total=64, max_cand=100, max_new=64, pol=p, k=0x10000000, v=0x20000000,
                   l=lay, kd=0x40000000, vd=0x48000000, ld_=lay_dst, idx=0x5000000, istr=32, out=0x6000000, ostr=32,
                   keep=0x7200000, ws=None, ws_bytes=0):
        return L.sirllm_step_ragged_out_of_place(logits, dt, vocab, ld, tok, scores, sstr, n_streams, held, cu, total,
                                                 max_cand, max_new, C.byref(pol) if pol else None, k, v,
                                                 C.byref(l) if l else None, kd, vd, C.byref(ld_) if ld_ else None, idx, istr,
                                                 out, ostr, keep, ws, ws_bytes, None)
    assert ragged_oop(kd=None) == b.SIRLLM_ERR_INVALID_ARG              # max_cand > budget: somewhere to compact to is needed
    assert ragged_oop(ld_=None) == b.SIRLLM_ERR_INVALID_ARG
    assert ragged_oop(vd=None) == b.SIRLLM_ERR_INVALID_ARG              # V on one side only
    assert ragged_oop(kd=0x10000000 + 4096) == b.SIRLLM_ERR_INVALID_ARG  # destination inside the source
    assert ragged_oop(vd=0x40000000 + 64) == b.SIRLLM_ERR_INVALID_ARG   # the two destinations overlap
    other = b.sirllm_kv_layout(2, 2, 32, 4, 2 * 2 * 32 * 32, 2 * 32 * 32, 32 * 32, 32)
    assert ragged_oop(ld_=other) == b.SIRLLM_ERR_INVALID_ARG            # head_dim differs between the two sides
    assert ragged_oop(k=None) == b.SIRLLM_ERR_INVALID_ARG
    assert ragged_oop(pol=None) == b.SIRLLM_ERR_INVALID_ARG
    assert ragged_oop(dt=9) == b.SIRLLM_ERR_UNSUPPORTED
    assert ragged_oop(max_new=101) == b.SIRLLM_ERR_INVALID_ARG
    assert ragged_oop(istr=31) == b.SIRLLM_ERR_INVALID_ARG
    assert ragged_oop(max_cand=40000, sstr=40000) in (b.SIRLLM_ERR_WORKSPACE, b.SIRLLM_ERR_INVALID_ARG)
    assert ragged_oop(n_streams=0) == b.SIRLLM_OK

    def lm_ragged(hidden=0x1000, ld_h=64, weight=0x8000000, ld_w=64, dt=1, d_model=64, vocab=1000, tok=0x2000000,
                  scores=0x3000000, sstr=128, n_streams=2, held=0x7000000, cu=0x7100000, total=64, max_cand=100,
                  max_new=64, pol=p, k=0x10000000, v=0x20000000, l=lay, idx=0x5000000, istr=32, out=0x6000000, ostr=32,
                  keep=0x7200000, ws=0x30000000, ws_bytes=1 << 30):
        return L.sirllm_step_lmhead_ragged(hidden, ld_h, weight, ld_w, dt, d_model, vocab, tok, scores, sstr, n_streams,
                                           held, cu, total, max_cand, max_new, C.byref(pol) if pol else None, k, v,
                                           C.byref(l) if l else None, idx, istr, out, ostr, keep, ws, ws_bytes, None)
    need = b.sirllm_step_lmhead_ragged_workspace_bytes(2, 100, 64, 1000)
    assert need == b.sirllm_lmhead_workspace_bytes(64, 1000) + b.SIRLLM_INPLACE_WORKSPACE_BYTES
    assert b.sirllm_step_lmhead_ragged_workspace_bytes(2, 40000, 64, 1000) == \
        b.sirllm_lmhead_workspace_bytes(64, 1000) + b.sirllm_workspace_bytes(2, 40000, 0, 0)
    assert lm_ragged(dt=0) == b.SIRLLM_ERR_UNSUPPORTED                   # f32 operands
    assert lm_ragged(d_model=60) == b.SIRLLM_ERR_UNSUPPORTED
    assert lm_ragged(hidden=None) == b.SIRLLM_ERR_INVALID_ARG
    assert lm_ragged(total=-1) == b.SIRLLM_ERR_INVALID_ARG
    assert lm_ragged(pol=None) == b.SIRLLM_ERR_INVALID_ARG
    assert lm_ragged(max_new=101) == b.SIRLLM_ERR_INVALID_ARG
    assert lm_ragged(held=None) == b.SIRLLM_ERR_INVALID_ARG
    assert lm_ragged(keep=None) == b.SIRLLM_ERR_INVALID_ARG
    assert lm_ragged(sstr=99) == b.SIRLLM_ERR_INVALID_ARG
    assert lm_ragged(k=None) == b.SIRLLM_ERR_INVALID_ARG
    assert lm_ragged(ws=None) == b.SIRLLM_ERR_WORKSPACE
    assert lm_ragged(ws_bytes=need - 1) == b.SIRLLM_ERR_WORKSPACE
    assert lm_ragged(ws=0x30000010) == b.SIRLLM_ERR_WORKSPACE
    assert lm_ragged(n_streams=0) == b.SIRLLM_OK

    def lm_ragged_oop(hidden=0x1000, ld_h=64, weight=0x8000000, ld_w=64, dt=1, d_model=64, vocab=1000, tok=0x2000000,
                      scores=0x3000000, sstr=128, n_streams=2, held=0x7000000, cu=0x7100000, total=64, max_cand=100,
                      max_new=64, pol=p, k=0x10000000, v=0x20000000, l=lay, kd=0x40000000, vd=0x48000000, ld_=lay_dst,
                      idx=0x5000000, istr=32, out=0x6000000, ostr=32, keep=0x7200000, ws=0x30000000, ws_bytes=1 << 30):
        return L.sirllm_step_lmhead_ragged_out_of_place(hidden, ld_h, weight, ld_w, dt, d_model, vocab, tok, scores, sstr,
                                                        n_streams, held, cu, total, max_cand, max_new,
                                                        C.byref(pol) if pol else None, k, v, C.byref(l) if l else None, kd, vd,
                                                        C.byref(ld_) if ld_ else None, idx, istr, out, ostr, keep, ws,
                                                        ws_bytes, None)
    assert lm_ragged_oop(kd=None) == b.SIRLLM_ERR_INVALID_ARG
    assert lm_ragged_oop(ld_=None) == b.SIRLLM_ERR_INVALID_ARG
    assert lm_ragged_oop(vd=None) == b.SIRLLM_ERR_INVALID_ARG
    assert lm_ragged_oop(kd=0x10000000 + 4096) == b.SIRLLM_ERR_INVALID_ARG   # destination inside the source
    assert lm_ragged_oop(ld_=other) == b.SIRLLM_ERR_INVALID_ARG
    assert lm_ragged_oop(dt=0) == b.SIRLLM_ERR_UNSUPPORTED
    assert lm_ragged_oop(hidden=None) == b.SIRLLM_ERR_INVALID_ARG
    assert lm_ragged_oop(pol=None) == b.SIRLLM_ERR_INVALID_ARG
    assert lm_ragged_oop(k=None) == b.SIRLLM_ERR_INVALID_ARG
    assert lm_ragged_oop(ws=None) == b.SIRLLM_ERR_WORKSPACE
    assert lm_ragged_oop(ws_bytes=need - 1) == b.SIRLLM_ERR_WORKSPACE
    assert lm_ragged_oop(n_streams=0) == b.SIRLLM_OK


def test_score_chunk_argument_errors(b):
    L = b.raw()
    assert L.sirllm_score_partial(FAKE, 0, 4, 10, 10, -1, FAKE, FAKE, None) == b.SIRLLM_ERR_INVALID_ARG   # v_begin < 0
    assert L.sirllm_score_partial(FAKE, 0, 4, 10, 9, 0, FAKE, FAKE, None) == b.SIRLLM_ERR_INVALID_ARG    # ld < n_cols
    assert L.sirllm_score_partial(FAKE, 3, 4, 10, 10, 0, FAKE, FAKE, None) == b.SIRLLM_ERR_UNSUPPORTED
    assert L.sirllm_score_partial(FAKE, 0, 4, 10, 10, 0, FAKE, None, None) == b.SIRLLM_ERR_INVALID_ARG
    assert L.sirllm_score_partial(None, 0, 0, 10, 10, 0, None, None, None) == b.SIRLLM_OK
    assert L.sirllm_score_merge(FAKE, 0, 100, 4, FAKE, None) == b.SIRLLM_ERR_INVALID_ARG                 # no parts
    assert L.sirllm_score_merge(FAKE, 2, 11, 4, FAKE, None) == b.SIRLLM_ERR_INVALID_ARG                  # parts overlap
    assert L.sirllm_score_merge(None, 2, 12, 4, FAKE, None) == b.SIRLLM_ERR_INVALID_ARG
    assert L.sirllm_score_merge(FAKE, 2, 12, 4, None, None) == b.SIRLLM_ERR_INVALID_ARG
    assert L.sirllm_score_merge(None, 2, 12, 0, None, None) == b.SIRLLM_OK


def test_large_caches_need_the_workspace(b):
    L = b.raw()
    p = b.sirllm_policy(4, 20000, 512, 0.9)
    need = b.sirllm_workspace_bytes(2, 40000, 0, 0)
    assert need > 0 and need % 256 == 0
    assert b.sirllm_workspace_bytes(2, 32768, 0, 0) == 0
    def call(ws, ws_bytes):
        return L.sirllm_decay_select(FAKE, 40000, 2, 39000, 1000, C.byref(p), FAKE + 0x100000, 20516,
                                     FAKE + 0x200000, 20516, ws, ws_bytes, None)
    assert call(None, 0) == b.SIRLLM_ERR_WORKSPACE
    assert call(0x40000, need - 1) == b.SIRLLM_ERR_WORKSPACE
    assert call(0x40010, need) == b.SIRLLM_ERR_WORKSPACE                  # not 256-byte aligned


def test_binding_refuses_host_tensors(b):
    import torch
    z = torch.zeros(2, 8)
    with pytest.raises(ValueError):
        b.sirllm_score(z, torch.zeros(2, dtype=torch.int32), torch.zeros(2))


def test_product_path_never_touches_the_oracle():
    pkg = os.path.join(ROOT, "paper_2405_12528_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b", text, flags=re.M), f"{f} imports the oracle"
                assert "sirllm_ref" not in text, f"{f} names the oracle's library"


def test_lmhead_argument_errors(b):
    L = b.raw()
    BF, F16, F32 = 1, 2, 0
    ws = b.sirllm_lmhead_workspace_bytes(4, 1000)
    assert ws % 256 == 0 and ws >= 4 * 3 * 4 * 4                                   # 4 vocabulary tiles of 256
    assert b.sirllm_lmhead_workspace_bytes(0, 1000) == 0
    ok = lambda *a: L.sirllm_lmhead_score(*a)
    assert ok(FAKE, 64, FAKE, 64, BF, 64, 0, 1000, None, None, None, 0, None) == b.SIRLLM_OK          # no rows
    assert ok(FAKE, 64, FAKE, 64, BF, 64, -1, 1000, FAKE, FAKE, FAKE, ws, None) == b.SIRLLM_ERR_INVALID_ARG
    assert ok(FAKE, 64, FAKE, 64, BF, 64, 4, 0, FAKE, FAKE, FAKE, ws, None) == b.SIRLLM_ERR_INVALID_ARG
    assert ok(FAKE, 56, FAKE, 64, BF, 64, 4, 1000, FAKE, FAKE, FAKE, ws, None) == b.SIRLLM_ERR_INVALID_ARG   # ld_h < d_model
    assert ok(FAKE, 64, FAKE, 56, BF, 64, 4, 1000, FAKE, FAKE, FAKE, ws, None) == b.SIRLLM_ERR_INVALID_ARG
    assert ok(None, 64, FAKE, 64, BF, 64, 4, 1000, FAKE, FAKE, FAKE, ws, None) == b.SIRLLM_ERR_INVALID_ARG
    assert ok(FAKE, 64, None, 64, BF, 64, 4, 1000, FAKE, FAKE, FAKE, ws, None) == b.SIRLLM_ERR_INVALID_ARG
    assert ok(FAKE, 64, FAKE, 64, BF, 64, 4, 1000, None, FAKE, FAKE, ws, None) == b.SIRLLM_ERR_INVALID_ARG
    assert ok(FAKE, 64, FAKE, 64, BF, 64, 4, 1000, FAKE, None, FAKE, ws, None) == b.SIRLLM_ERR_INVALID_ARG
    assert ok(FAKE, 64, FAKE, 64, 9, 64, 4, 1000, FAKE, FAKE, FAKE, ws, None) == b.SIRLLM_ERR_INVALID_ARG    # no such dtype
    assert ok(FAKE, 64, FAKE, 64, F32, 64, 4, 1000, FAKE, FAKE, FAKE, ws, None) == b.SIRLLM_ERR_UNSUPPORTED  # no f32 MFMA path
    assert ok(FAKE, 64, FAKE, 64, F16, 60, 4, 1000, FAKE, FAKE, FAKE, ws, None) == b.SIRLLM_ERR_UNSUPPORTED  # d_model % 8
    assert ok(FAKE, 68, FAKE, 64, BF, 64, 4, 1000, FAKE, FAKE, FAKE, ws, None) == b.SIRLLM_ERR_UNSUPPORTED   # ld_h % 8
    assert ok(FAKE + 2, 64, FAKE, 64, BF, 64, 4, 1000, FAKE, FAKE, FAKE, ws, None) == b.SIRLLM_ERR_UNSUPPORTED
    assert ok(FAKE, 64, FAKE, 1 << 21, BF, 64, 4, 1000, FAKE, FAKE, FAKE, ws, None) == b.SIRLLM_ERR_UNSUPPORTED
    assert ok(FAKE, 64, FAKE, 64, BF, 64, 4, 1000, FAKE, FAKE, None, 0, None) == b.SIRLLM_ERR_WORKSPACE
    assert ok(FAKE, 64, FAKE, 64, BF, 64, 4, 1000, FAKE, FAKE, FAKE, ws - 1, None) == b.SIRLLM_ERR_WORKSPACE
    assert ok(FAKE, 64, FAKE, 64, BF, 64, 4, 1000, FAKE, FAKE, FAKE + 16, ws, None) == b.SIRLLM_ERR_WORKSPACE  # alignment


def test_step_lmhead_argument_errors(b):
    L = b.raw()
    pol = b.sirllm_policy(4, 20, 8, 0.9)
    lay = b.sirllm_kv_layout(2, 2, 16, 4, 2 * 2 * 96 * 16, 2 * 96 * 16, 96 * 16, 16)
    dst = b.sirllm_kv_layout(2, 2, 16, 4, 2 * 2 * 32 * 16, 2 * 32 * 16, 32 * 16, 16)
    ws = b.sirllm_step_lmhead_workspace_bytes(1, 96, 64, 1000)
    assert ws == b.sirllm_lmhead_workspace_bytes(64, 1000) + b.sirllm_workspace_bytes(1, 96, 0, 0)
    K1, K2, V1, V2 = 0x100000, 0x200000, 0x300000, 0x400000

    def call(hidden=FAKE, ld_h=64, weight=FAKE, ld_w=64, dt=1, d=64, vocab=1000, tok=FAKE, scores=0x10000, n_held=32,
             n_new=64, work=0x20000, wsb=ws, out=0x40000):
        return L.sirllm_step_lmhead(hidden, ld_h, weight, ld_w, dt, d, vocab, tok, scores, 96, 1, n_held, n_new,
                                    C.byref(pol), K1, V1, C.byref(lay), K2, V2, C.byref(dst), 0x30000, 32, out, 32,
                                    work, wsb, None)

    assert call(n_new=-1) == b.SIRLLM_ERR_INVALID_ARG
    assert call(hidden=None) == b.SIRLLM_ERR_INVALID_ARG
    assert call(weight=None) == b.SIRLLM_ERR_INVALID_ARG
    assert call(tok=None) == b.SIRLLM_ERR_INVALID_ARG
    assert call(dt=0) == b.SIRLLM_ERR_UNSUPPORTED            # binary32 operands
    assert call(d=60) == b.SIRLLM_ERR_UNSUPPORTED            # d_model % 8
    assert call(ld_h=56) == b.SIRLLM_ERR_INVALID_ARG         # ld_h < d_model
    assert call(scores=None) == b.SIRLLM_ERR_INVALID_ARG
    assert call(out=0x10000) == b.SIRLLM_ERR_INVALID_ARG     # scores_out overlaps scores
    assert call(work=None, wsb=0) == b.SIRLLM_ERR_WORKSPACE
    assert call(wsb=ws - 1) == b.SIRLLM_ERR_WORKSPACE
    assert call(n_held=0, n_new=0) == b.SIRLLM_OK            # nothing to do


def test_bench_refuses_more_than_one_gpu():
    # the benchmark is a one-GPU program: asked for more it must say so and stop before touching a device
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2", "--steps", "1"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and "--gpus must be 1" in r.stderr
    assert r.stdout.strip() == ""


def test_product_files_name_no_working_folder():
    # nothing that is committed may read, import or run a file under the ignored working folder
    import subprocess
    files = subprocess.run(["git", "ls-files"], cwd=ROOT, capture_output=True, text=True).stdout.split()
    for f in files:
        if f.endswith((".py", ".hip", ".h", ".c")) and not f.startswith("tests/test_abi.py"):
            text = open(os.path.join(ROOT, f), errors="ignore").read()
            assert "_work/" not in text and "_work\\" not in text, f
