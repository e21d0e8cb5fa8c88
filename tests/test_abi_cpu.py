"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every function the header declares, and rejects bad arguments before any launch."""
import ctypes
import os
import re

import pytest

import paper_2602_01053_amd as lra
from paper_2602_01053_amd.binding import LraAdapters, LraCache, LraShape, LraTuning

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(lra.binding.LIB_PATH):
        from paper_2602_01053_amd.build import build_library
        build_library()
    return lra.load_library()


def test_header_symbols_are_exported(lib):
    text = "".join(open(os.path.join(ROOT, "include", h)).read() for h in sorted(os.listdir(os.path.join(ROOT, "include"))))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(lra_[a-z0-9_]+)\s*\(", text))
    assert {"lra_attn_decode", "lra_attn_prefill", "lra_workspace_bytes"} <= declared
    for name in declared:
        assert hasattr(lib, name), f"{name} declared in include/ but not exported"
    assert declared == set(lra.binding.EXPORTS)


def test_status_strings(lib):
    seen = {lra.lra_status_string(s) for s in range(7)}
    assert len(seen) == 7 and lra.lra_status_string(0) == "ok"
    assert lra.lra_status_string(99) == "unknown status"


FAKE = 0x1000  # never dereferenced: every case below fails validation first


def _good():
    sh = LraShape(32, 8, 128, 16, 0, 0.0)
    c = LraCache(FAKE, FAKE, FAKE, 1024, 128, 0, 0, 0, 0, 1, 0, 0, None, FAKE, 8192)
    ad = LraAdapters(FAKE, FAKE, 4)
    return sh, c, ad


def _decode(lib, sh, c, ad, q=FAKE, qa=FAKE, sqs=FAKE, n_queries=4, mq=4, out=FAKE, ws=None, ws_bytes=0):
    return lib.lra_attn_decode(ctypes.byref(sh), ctypes.byref(c), ctypes.byref(ad), q, qa, sqs,
                               n_queries, mq, out, ws, ws_bytes, None, None)


def _prefill(lib, sh, c, ad, q=FAKE, seq=0, a=0, n_new=16, out=FAKE, ws=None, ws_bytes=0):
    return lib.lra_attn_prefill(ctypes.byref(sh), ctypes.byref(c), ctypes.byref(ad), q, seq, a, n_new,
                                out, ws, ws_bytes, None, None)


def test_static_workspace_entry_point_rejects_before_any_gpu_call(lib):
    """lra_attn_decode_static runs the same checks, and refuses a call whose partial states would not fit
    its fixed buffer, before it touches the GPU (there is none here)."""
    sh, c, ad = _good()
    call = lambda s, cc, a, nq=4, mq=4, q=FAKE: lib.lra_attn_decode_static(
        ctypes.byref(s), ctypes.byref(cc), ctypes.byref(a), q, FAKE, FAKE, nq, mq, FAKE, None, None)
    assert call(sh, c, ad, q=None) == 1
    assert call(sh, c, ad, nq=0) == 2
    sh.rank = 65
    assert call(sh, c, ad) == 4
    sh, c, ad = _good()
    need = lib.lra_workspace_bytes(ctypes.byref(sh), ctypes.byref(c), 4096, 4096, 0, None)
    assert need > lra.binding.STATIC_WORKSPACE_BYTES
    assert call(sh, c, ad, nq=4096, mq=4096) == 5
    text = open(os.path.join(ROOT, "include", "lra_attn.h")).read()
    assert re.search(r"#define LRA_STATIC_WORKSPACE_BYTES \(\(size_t\)(\d+) << 20\)", text).group(1) == str(
        lra.binding.STATIC_WORKSPACE_BYTES >> 20)


def test_rejects_bad_arguments_before_launch(lib):
    NULL, SHAPE, DTYPE, UNSUP, WS = 1, 2, 3, 4, 5
    sh, c, ad = _good()
    assert lib.lra_attn_decode(None, ctypes.byref(c), ctypes.byref(ad), FAKE, FAKE, FAKE, 4, 4, FAKE,
                               None, 0, None, None) == NULL
    assert _decode(lib, sh, c, ad, q=None) == NULL
    assert _decode(lib, sh, c, ad, out=None) == NULL
    assert _decode(lib, sh, c, ad, qa=None) == NULL

    def mutated(**kw):
        s, cc, a = _good()
        for k, v in kw.items():
            for obj in (s, cc, a):
                if hasattr(obj, k):
                    setattr(obj, k, v)
        return s, cc, a

    assert _decode(lib, *mutated(dtype=7)) == DTYPE
    assert _decode(lib, *mutated(n_q_heads=30)) == SHAPE          # not a multiple of Hkv
    assert _decode(lib, *mutated(head_dim=96)) == UNSUP
    assert _decode(lib, *mutated(rank=65)) == UNSUP
    assert _decode(lib, *mutated(rank=0)) == SHAPE
    assert _decode(lib, *mutated(n_q_heads=32, n_kv_heads=1)) == UNSUP   # group of 32
    assert _decode(lib, *mutated(block_size=32)) == UNSUP
    assert _decode(lib, *mutated(kv_token_stride=1023)) == SHAPE
    assert _decode(lib, *mutated(kv_head_stride=64)) == SHAPE
    assert _decode(lib, *mutated(k_base=None)) == NULL
    assert _decode(lib, *mutated(seq_lens=None)) == NULL
    assert _decode(lib, *mutated(l=FAKE + 2)) == SHAPE            # misaligned
    assert _decode(lib, *mutated(max_seq_len=0)) == SHAPE
    assert _decode(lib, *mutated(n_seqs=2)) == SHAPE              # contiguous holds one sequence
    assert _decode(lib, *mutated(n_adapters=0)) == SHAPE
    assert _decode(lib, *mutated(scale=float("nan"))) == SHAPE
    assert _decode(lib, *mutated(key_rope_theta=-1.0)) == SHAPE
    assert _decode(lib, *mutated(key_rope_theta=float("nan"))) == SHAPE
    assert _decode(lib, *mutated(key_rope_theta=float("inf"))) == SHAPE
    assert _decode(lib, *mutated(key_rope_theta=500000.0)) == WS     # valid: stops at the missing workspace
    assert _decode(lib, *mutated(block_size=16, n_seqs=2)) == NULL   # paged without a block table
    assert _decode(lib, *mutated(block_size=16, block_table=FAKE, num_blocks=600, kv_block_stride=16384,
                                 max_blocks_per_seq=8)) == SHAPE  # table row shorter than max_seq_len
    assert _decode(lib, *mutated(l_row_stride=8)) == SHAPE          # rows shorter than the rank
    assert _decode(lib, *mutated(l_row_stride=20)) == SHAPE         # not a multiple of 8 elements
    assert _decode(lib, *mutated(l_adapter_stride=-16)) == SHAPE
    assert _decode(lib, *mutated(l_adapter_stride=12)) == SHAPE
    assert _decode(lib, *mutated(l_row_stride=1 << 32)) == UNSUP
    assert _decode(lib, *mutated(l_row_stride=64, l_adapter_stride=16)) == WS     # valid per-adapter caches: only the workspace is missing
    assert _decode(lib, sh, c, ad, n_queries=0) == SHAPE
    assert _decode(lib, sh, c, ad, mq=5) == SHAPE
    # good arguments but no / small / misaligned workspace: refused, nothing launched
    assert _decode(lib, sh, c, ad) == WS
    wsb = lambda s_, n_q, mq, n_new, tune=None: lib.lra_workspace_bytes(
        ctypes.byref(s_), ctypes.byref(c), n_q, mq, n_new, None if tune is None else ctypes.byref(tune))
    need = wsb(sh, 4, 4, 0)
    assert 0 < need < (1 << 40)
    assert _decode(lib, sh, c, ad, ws=0x10000, ws_bytes=need - 1) == WS
    assert _decode(lib, sh, c, ad, ws=0x10010, ws_bytes=need) == WS

    assert _prefill(lib, sh, c, ad, seq=1) == SHAPE
    assert _prefill(lib, sh, c, ad, a=4) == SHAPE
    assert _prefill(lib, sh, c, ad, n_new=0) == SHAPE
    assert _prefill(lib, sh, c, ad, n_new=8193) == SHAPE
    assert _prefill(lib, sh, c, ad, q=None) == NULL
    bad = lib.lra_workspace_bytes(ctypes.byref(mutated(head_dim=96)[0]), ctypes.byref(c), 4, 4, 0, None)
    assert wsb(sh, 0, 0, 2048) == 0                  # bf16 prefill, enough q tiles: one kernel
    assert 0 < wsb(sh, 0, 0, 1024) < (1 << 40)       # key tiles shared: merge
    assert 0 < wsb(sh, 0, 0, 16) < (1 << 40)         # few new tokens: split-KV path
    # the tuning struct travels with the call: the library keeps none of it
    assert wsb(sh, 0, 0, 16, LraTuning()) == wsb(sh, 0, 0, 16)             # all zero = automatic
    no_short = LraTuning(short_prefill=-1)
    assert wsb(sh, 0, 0, 16, no_short) > 0           # that path off: key tiles shared instead
    assert wsb(sh, 0, 0, 16, LraTuning(short_prefill=-1, prefill_splits=1)) == 0   # one workgroup per q tile and head
    assert wsb(sh, 0, 0, 16) == wsb(sh, 0, 0, 16, LraTuning(short_prefill=32))     # nothing stuck from the calls above
    assert wsb(sh, 4, 4, 0, LraTuning(decode_split_keys=4096)) < need              # fewer key shares, fewer partial states
    sh32 = mutated(dtype=1)[0]
    assert 0 < wsb(sh32, 0, 0, 16) < (1 << 40)
    assert wsb(sh, 4, 5, 0) == ctypes.c_size_t(-1).value
    assert bad == ctypes.c_size_t(-1).value


def test_cache_append_rejects_bad_arguments_before_launch(lib):
    from paper_2602_01053_amd.binding import LraProjection
    NULL, SHAPE, UNSUP = 1, 2, 4

    def call(sh=None, c=None, proj=None, x=FAKE, seq=0, n_new=16, w=FAKE, d_model=4096, theta=500000.0, no_proj=False):
        s0, c0, _ = _good()
        sh = sh or s0
        c = c or c0
        pr = LraProjection(w, d_model, theta)
        return lib.lra_cache_append(ctypes.byref(sh), ctypes.byref(c), None if no_proj else ctypes.byref(pr), x, seq,
                                    n_new, None, 0, None, None)

    assert call(no_proj=True) == NULL
    assert call(w=None) == NULL
    assert call(x=None) == NULL
    assert call(seq=1) == SHAPE                       # one (contiguous) sequence
    assert call(n_new=0) == SHAPE
    assert call(n_new=8193) == SHAPE                  # more new tokens than the cache can hold
    assert call(d_model=0) == SHAPE
    assert call(theta=-1.0) == SHAPE
    assert call(theta=float("nan")) == SHAPE
    assert call(theta=float("inf")) == SHAPE
    assert call(x=FAKE + 8) == SHAPE                  # misaligned
    assert call(d_model=4000) == UNSUP                # not a multiple of 64
    assert call(d_model=1 << 22) == UNSUP             # weights beyond 32-bit byte offsets
    sh, c, _ = _good()
    sh.dtype = 1
    assert call(sh=sh) == UNSUP                       # fp32 caches
    sh, c, _ = _good()
    sh.rank = 12
    assert call(sh=sh) == UNSUP                       # rank not a multiple of 8
    sh, c, _ = _good()
    c.k_base = None
    assert call(c=c) == NULL


def test_tuning_helpers_of_the_binding_round_trip(lib):
    """The lra_set_* helpers edit the one struct the binding passes to every call and return the previous value."""
    old = lra.lra_set_append_skinny(7)
    assert lra.lra_set_append_skinny(old) == 7 and old == 64
    assert lra.lra_set_append_skinny(0) == 64 and lra.binding._tuning.append_skinny == -1     # 0 = off
    assert lra.lra_set_append_skinny(64) == 0
    assert lra.lra_set_append_stages(3) == 0 and lra.lra_set_append_stages(0) == 3
    assert lra.lra_set_append_tile(256) == 0 and lra.lra_set_append_tile(0) == 256
    old = lra.lra_set_decode_split_keys(512)
    assert lra.lra_set_decode_split_keys(old) == 512
    old = lra.lra_set_kernel_variant(1)
    assert lra.lra_set_kernel_variant(old) == 1
    old = lra.lra_set_short_prefill(0)
    assert old == 32 and lra.lra_set_short_prefill(old) == 0
    assert lra.lra_set_profile_mode(1) == 0 and lra.lra_set_profile_mode(0) == 1
    t = lra.binding._tuning
    assert (t.kernel_variant, t.decode_split_keys, t.prefill_splits, t.append_stages, t.append_tile,
            t.measure_main_kernel_only) == (0, 0, 0, 0, 0, 0)


def test_library_exports_no_setters(lib):
    """No process-wide tuning state in the C library: nothing but the entry points of the headers is exported
    under the lra_ prefix."""
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", lra.binding.LIB_PATH], capture_output=True, text=True).stdout
    exported = {ln.split()[-1] for ln in out.splitlines() if " T " in ln and ln.split()[-1].startswith("lra_")}
    assert exported == set(lra.binding.EXPORTS), exported ^ set(lra.binding.EXPORTS)


def test_binding_fails_loudly_without_library(monkeypatch):
    monkeypatch.setattr(lra.binding, "_lib", None)
    monkeypatch.setattr(lra.binding, "LIB_PATH", "/nonexistent/liblra_attn.so")
    with pytest.raises(RuntimeError, match="no fallback"):
        lra.binding.load_library()


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header compiles as C99 on its own, with warnings as errors."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    src = tmp_path / "use_header.c"
    src.write_text(
        '#include "lra_attn.h"\n#include "lra_attn_measure.h"\n'
        "lra_status call(const lra_shape* s, const lra_cache* c, const lra_projection* p, const void* x) {\n"
        "  lra_tuning t = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0};\n"
        "  return lra_cache_append(s, c, p, x, 0, 1, (void*)0, 0, &t, (void*)0);\n"
        "}\n"
        "size_t need(const lra_shape* s, const lra_cache* c) { return lra_workspace_bytes(s, c, 4, 4, 0, (const lra_tuning*)0); }\n")
    res = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only",
                          "-I", os.path.join(ROOT, "include"), str(src)], capture_output=True, text=True)
    assert res.returncode == 0, res.stderr


def test_probes_reject_bad_arguments(lib):
    """The two machine probes validate on the host before any launch."""
    import ctypes
    flops = ctypes.c_int64(0)
    assert lib.lra_probe_stream_read(None, 1024, None, None) != 0
    assert lib.lra_probe_stream_read(ctypes.c_void_p(4096), 8, ctypes.c_void_p(4096), None) != 0      # fewer than 16 bytes
    assert lib.lra_probe_stream_read(ctypes.c_void_p(4100), 1024, ctypes.c_void_p(4096), None) != 0   # misaligned
    assert lib.lra_probe_mfma_bf16(0, 0, ctypes.byref(flops), ctypes.c_void_p(4096), None) != 0
    assert lib.lra_probe_mfma_bf16(10, 1, ctypes.byref(flops), None, None) != 0
