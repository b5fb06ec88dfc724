"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every
symbol the header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2403_17312_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2403_17312_amd import build
        build.build()
    binding.lib()
    return binding


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "swa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(swa_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(B):
    names = _declared_functions()
    assert set(names) == set(B.EXPORTS), names
    L = ctypes.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(L, n), n


def test_params_struct_matches_header(B):
    text = open(os.path.join(ROOT, "include", "swa.h")).read()
    body = re.search(r"typedef struct \{(.*?)\} swa_params;", text, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"(int32_t|float)\s+(\w+);", body)
    assert [f[1] for f in fields] == [f[0] for f in B.SwaParams._fields_]
    assert ctypes.sizeof(B.SwaParams) == 40
    assert int(re.search(r"#define SWA_MAX_CAP (\d+)", text).group(1)) == B.SWA_MAX_CAP
    assert int(re.search(r"#define SWA_MAX_PREFILL_ROWS (\d+)", text).group(1)) == B.SWA_MAX_PREFILL_ROWS
    assert int(re.search(r"#define SWA_MAX_FUSED_SLOTS (\d+)", text).group(1)) == B.SWA_MAX_FUSED_SLOTS
    assert int(re.search(r"#define SWA_FUSE_COMPACTION (\d+)", text).group(1)) == B.SWA_FUSE_COMPACTION
    assert int(re.search(r"#define SWA_UNORDERED (\d+)", text).group(1)) == B.SWA_UNORDERED
    assert int(re.search(r"#define SWA_HEAD_SHARED (\d+)", text).group(1)) == B.SWA_HEAD_SHARED
    assert int(re.search(r"#define SWA_MAX_UNORDERED_SLOTS (\d+)", text).group(1)) == B.SWA_MAX_UNORDERED_SLOTS
    assert int(re.search(r"#define SWA_SPLIT_ROWS (\d+)", text).group(1)) == B.SWA_SPLIT_ROWS
    assert int(re.search(r"#define SWA_KV_INT8 (\d+)", text).group(1)) == B.SWA_KV_INT8


def test_strerror_covers_all_codes(B):
    for code in range(0, -11, -1):
        msg = B.strerror(code)
        assert msg and "unknown" not in msg
    assert "unknown" in B.strerror(-99)


def test_budget_helper_matches_hand_worked_values(B):
    rows = [l.split() for l in open(os.path.join(ROOT, "tests", "golden", "keep_budget.txt"))
            if l[0] != "#"]
    for n, sp, _, keep in rows:
        assert B.swa_budget(int(n), int(n), 1, int(sp) * 100)[0] == int(keep)
    assert B.swa_budget(1000, 50, 8, 8000) == (50, 8, 42)
    assert B.swa_budget(100, 5, 64, 9000) == (5, 5, 0)
    with pytest.raises(B.SwaError):
        B.swa_budget(10, 10, 1, 10000)
    rows = [l.split() for l in open(os.path.join(ROOT, "tests", "golden", "even_split.txt"))
            if l[0] != "#"]
    for n, sp, _, k in rows:
        assert B.swa_budget(int(n), int(n), B.SWA_W_EVEN_SPLIT, int(sp) * 100) == (2 * int(k), int(k), int(k))


def test_workspace_bytes(B):
    p = B.make_params(16, 32, 128, 545, 16, 8000, B.SWA_F16)
    n = B.swa_workspace_bytes(p)
    assert n >= 64 + 4 * 16 and n % 256 == 0
    assert B.swa_workspace_bytes(B.make_params(16, 32, 96, 545, 16, 8000, B.SWA_F16)) == 0
    ps = B.make_params(16, 32, 128, 576, 16, 8000, B.SWA_F16, flags=7)
    assert B.swa_workspace_bytes(ps) >= n + 4 * (2 * 16 * 32 * 576 + 16 * 32 * 128 + 16 * 576)


@pytest.mark.parametrize("kw,code", [
    (dict(d=96), "SWA_ERR_UNSUPPORTED_D"),
    (dict(dtype=7), "SWA_ERR_UNSUPPORTED_DTYPE"),
    (dict(b=0), "SWA_ERR_BAD_SHAPE"),
    (dict(w=-2), "SWA_ERR_BAD_SHAPE"),
    (dict(cap=0), "SWA_ERR_BAD_SHAPE"),
    (dict(cap=16385), "SWA_ERR_CAPACITY"),
    (dict(len_bound=-1), "SWA_ERR_BAD_SHAPE"),
    (dict(flags=2), "SWA_ERR_BAD_SHAPE"),          # SWA_UNORDERED needs SWA_FUSE_COMPACTION
    (dict(flags=4), "SWA_ERR_BAD_SHAPE"),          # SWA_HEAD_SHARED needs the other two
    (dict(flags=5), "SWA_ERR_BAD_SHAPE"),
    (dict(flags=32), "SWA_ERR_BAD_SHAPE"),         # not a flag
    (dict(flags=17), "SWA_ERR_BAD_SHAPE"),         # SWA_SPLIT_ROWS goes with the two-call form only
    (dict(flags=8), "SWA_ERR_UNSUPPORTED_DTYPE"),  # SWA_KV_INT8 goes with fp16 rows only
    (dict(sparsity_bp=10000), "SWA_ERR_BAD_SPARSITY"),
    (dict(sparsity_bp=-1), "SWA_ERR_BAD_SPARSITY"),
    (dict(scale=float("nan")), "SWA_ERR_BAD_SHAPE"),
])
def test_bad_params_are_rejected_before_any_device_work(B, kw, code):
    base = dict(b=2, h=2, d=64, cap=32, w=2, sparsity_bp=5000, dtype=B.SWA_F32, scale=0.0, len_bound=0, flags=0)
    base.update(kw)
    p = B.SwaParams(*[base[f[0]] for f in B.SwaParams._fields_])
    L = B.lib()
    fake = ctypes.c_void_p(0x1000)          # never dereferenced: validation fails first
    want = getattr(B, code)
    assert L.swa_decode_step(ctypes.byref(p), *([fake] * 15)) == want
    assert L.swa_compact_kv(ctypes.byref(p), *([fake] * 9)) == want
    assert L.swa_prefill_scores(ctypes.byref(p), fake, 4, fake, fake, fake, fake, fake) == want
    assert L.swa_workspace_init(ctypes.byref(p), fake, fake) == want


def test_null_and_misaligned_pointers_are_rejected(B):
    p = B.make_params(2, 2, 64, 32, 2, 5000, B.SWA_F32)
    L = B.lib()
    ok = ctypes.c_void_p(0x1000)
    args = [ok] * 15
    for i in [0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 13]:      # every required pointer
        a = list(args)
        a[i] = None
        assert L.swa_decode_step(ctypes.byref(p), *a) == B.SWA_ERR_NULL, i
    a = list(args)
    a[3] = ctypes.c_void_p(0x1008)
    assert L.swa_decode_step(ctypes.byref(p), *a) == B.SWA_ERR_ALIGNMENT
    assert L.swa_decode_step(None, *args) == B.SWA_ERR_NULL
    # fused compaction: kept_idx may be NULL, the two length arrays must differ, LDS bound applies
    pf = B.make_params(2, 2, 64, 32, 2, 5000, B.SWA_F32, flags=B.SWA_FUSE_COMPACTION)
    a = list(args)
    a[7] = ctypes.c_void_p(0x2000)
    a[9] = None
    a[0] = None                                               # still rejects a missing q
    assert L.swa_decode_step(ctypes.byref(pf), *a) == B.SWA_ERR_NULL
    a = list(args)                                            # cache_len == kept_cnt
    assert L.swa_decode_step(ctypes.byref(pf), *a) == B.SWA_ERR_BAD_SHAPE
    pbig = B.make_params(2, 2, 64, 12000, 2, 5000, B.SWA_F32, flags=B.SWA_FUSE_COMPACTION)
    a[7] = ctypes.c_void_p(0x2000)
    assert L.swa_decode_step(ctypes.byref(pbig), *a) == B.SWA_ERR_CAPACITY
    assert L.swa_compact_kv(ctypes.byref(p), None, *([ok] * 8)) == B.SWA_ERR_NULL
    assert L.swa_prefill_scores(ctypes.byref(p), ok, 0, ok, ok, ok, ok, ok) == B.SWA_ERR_BAD_SHAPE
    assert L.swa_prefill_scores(ctypes.byref(p), ok, 129, ok, ok, ok, ok, ok) == B.SWA_ERR_BAD_SHAPE
    assert L.swa_prefill_scores(ctypes.byref(p), None, 4, ok, ok, ok, ok, ok) == B.SWA_ERR_NULL


def test_compressed_cache_entry_points_validate_their_arguments(B):
    L = B.lib()
    ok = ctypes.c_void_p(0x1000)
    p16 = B.make_params(2, 2, 64, 32, 2, 5000, B.SWA_F16)
    pq = B.make_params(2, 2, 64, 32, 2, 5000, B.SWA_F16, flags=B.SWA_KV_INT8)
    p32 = B.make_params(2, 2, 64, 32, 2, 5000, B.SWA_F32)
    # the plain step refuses a compressed cache, the compressed step a plain one
    assert L.swa_decode_step(ctypes.byref(pq), *([ok] * 15)) == B.SWA_ERR_UNSUPPORTED_DTYPE
    assert L.swa_decode_step_q8(ctypes.byref(p16), *([ok] * 16)) == B.SWA_ERR_UNSUPPORTED_DTYPE
    a = [ok] * 16
    a[5] = None                                               # the quantisation parameters
    assert L.swa_decode_step_q8(ctypes.byref(pq), *a) == B.SWA_ERR_NULL
    a = [ok] * 16
    a[3] = ctypes.c_void_p(0x1004)
    assert L.swa_decode_step_q8(ctypes.byref(pq), *a) == B.SWA_ERR_ALIGNMENT
    assert L.swa_quantize_kv(ctypes.byref(p32), *([ok] * 7)) == B.SWA_ERR_UNSUPPORTED_DTYPE
    for i in range(6):
        a = [ok] * 7
        a[i] = None
        assert L.swa_quantize_kv(ctypes.byref(p16), *a) == B.SWA_ERR_NULL, i
    assert L.swa_quantize_kv(None, *([ok] * 7)) == B.SWA_ERR_NULL


def test_strict_window_entry_points_validate_their_arguments(B):
    L = B.lib()
    ok = ctypes.c_void_p(0x1000)
    pu = B.make_params(2, 2, 64, 32, 2, 5000, B.SWA_F16, flags=B.SWA_FUSE_COMPACTION | B.SWA_UNORDERED)
    p0 = B.make_params(2, 2, 64, 32, 2, 5000, B.SWA_F16)

    def step(p, ring=ok, R=4, row=0, cache_len=ctypes.c_void_p(0x2000)):
        return L.swa_decode_step_window(ctypes.byref(p), ok, ok, ok, ok, ok, ring, R, row, ok, ok, cache_len,
                                        ok, ok, ok, ok, ok, ok, ok)
    assert step(p0) == B.SWA_ERR_BAD_SHAPE                      # only the unordered fused form
    assert step(B.make_params(2, 2, 64, 32, 2, 5000, B.SWA_F16, flags=B.SWA_FUSE_COMPACTION)) == B.SWA_ERR_BAD_SHAPE
    # codes need their parameters: the plain call refuses a compressed cache, the q8 call a plain one
    pq = B.make_params(2, 2, 64, 32, 2, 5000, B.SWA_F16, flags=pu.flags | B.SWA_KV_INT8)
    assert step(pq) == B.SWA_ERR_UNSUPPORTED_DTYPE

    def step_q8(p, qparams=ok, ring=ok, R=4, row=0):
        return L.swa_decode_step_window_q8(ctypes.byref(p), ok, ok, ok, ok, ok, qparams, ring, R, row, ok, ok,
                                           ctypes.c_void_p(0x2000), ok, ok, ok, ok, ok, ok, ok)
    assert step_q8(pu) == B.SWA_ERR_UNSUPPORTED_DTYPE
    assert step_q8(pq, qparams=None) == B.SWA_ERR_NULL
    assert step_q8(pq, ring=None) == B.SWA_ERR_NULL
    assert step_q8(pq, R=4, row=4) == B.SWA_ERR_BAD_SHAPE
    assert step_q8(B.make_params(2, 2, 64, 32, 2, 5000, B.SWA_F16, flags=B.SWA_FUSE_COMPACTION | B.SWA_KV_INT8)) \
        == B.SWA_ERR_BAD_SHAPE
    assert step(pu, ring=None) == B.SWA_ERR_NULL
    assert step(pu, R=0) == B.SWA_ERR_BAD_SHAPE
    assert step(pu, R=B.SWA_MAX_WINDOW_ROWS + 1) == B.SWA_ERR_BAD_SHAPE
    assert step(pu, R=4, row=4) == B.SWA_ERR_BAD_SHAPE
    assert step(pu, R=4, row=-1) == B.SWA_ERR_BAD_SHAPE
    assert step(pu, cache_len=ok) == B.SWA_ERR_BAD_SHAPE        # cache_len == kept_cnt
    assert L.swa_prefill_rows(ctypes.byref(p0), ok, 0, ok, ok, ok, ok, ok) == B.SWA_ERR_BAD_SHAPE
    assert L.swa_prefill_rows(ctypes.byref(p0), ok, B.SWA_MAX_WINDOW_ROWS + 1, ok, ok, ok, ok, ok) == B.SWA_ERR_BAD_SHAPE
    assert L.swa_prefill_rows(ctypes.byref(p0), ok, 4, ok, ok, None, ok, ok) == B.SWA_ERR_NULL
    assert L.swa_prefill_rows(ctypes.byref(p0), ctypes.c_void_p(0x1004), 4, ok, ok, ok, ok, ok) == B.SWA_ERR_ALIGNMENT


def test_prefill_attention_validates_its_arguments(B):
    L = B.lib()
    ok = ctypes.c_void_p(0x1000)
    p16 = B.make_params(2, 2, 64, 32, 2, 5000, B.SWA_BF16)
    p32 = B.make_params(2, 2, 64, 32, 2, 5000, B.SWA_F32)

    def call(p, q=ok, R=4, score=ok, out=ok):
        return L.swa_prefill_attention(ctypes.byref(p), q, ok, ok, ok, out, R, score, ok, ok)
    pq = B.make_params(2, 2, 64, 32, 2, 5000, B.SWA_F16, flags=B.SWA_KV_INT8)
    assert call(pq) == B.SWA_ERR_UNSUPPORTED_DTYPE               # the prompt's cache is not compressed yet
    assert call(p32, q=None) == B.SWA_ERR_NULL
    assert call(p16, q=None) == B.SWA_ERR_NULL
    assert call(p16, out=None) == B.SWA_ERR_NULL
    assert call(p16, R=4, score=None) == B.SWA_ERR_NULL          # a seed needs somewhere to go
    assert call(p16, R=-1) == B.SWA_ERR_BAD_SHAPE
    assert call(p16, R=B.SWA_MAX_PREFILL_ROWS + 1) == B.SWA_ERR_BAD_SHAPE
    assert call(p16, q=ctypes.c_void_p(0x1008)) == B.SWA_ERR_ALIGNMENT
    assert L.swa_prefill_attention(None, ok, ok, ok, ok, ok, 4, ok, ok, ok) == B.SWA_ERR_NULL


def test_binding_fails_loudly_without_the_library(B, monkeypatch, tmp_path):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError, match="missing"):
        B.lib()


def test_offload_tier_entry_points_validate_their_arguments(B):
    L = B.lib()
    ok = ctypes.c_void_p(0x1000)
    p = B.make_params(2, 2, 64, 32, 2, 5000, B.SWA_F16)
    good = B.SwaHostStore(0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 16)

    def off(store=good, k=ok, ws=ok):
        return L.swa_offload_evicted(ctypes.byref(p), k, ok, ok, ok, ok, ok, ok, ctypes.byref(store) if store else None,
                                     ws, ok)
    assert off(store=None) == B.SWA_ERR_NULL
    assert off(store=B.SwaHostStore(0x1000, 0, 0x1000, 0x1000, 0x1000, 16)) == B.SWA_ERR_NULL
    assert off(store=B.SwaHostStore(0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 0)) == B.SWA_ERR_BAD_SHAPE
    assert off(store=B.SwaHostStore(0x1004, 0x1000, 0x1000, 0x1000, 0x1000, 16)) == B.SWA_ERR_ALIGNMENT
    assert off(k=None) == B.SWA_ERR_NULL
    assert off(ws=None) == B.SWA_ERR_NULL

    def rel(store=good, max_req=4, cache_len=ctypes.c_void_p(0x2000), new_len=ctypes.c_void_p(0x3000), req=ok):
        return L.swa_reload_tokens(ctypes.byref(p), ctypes.byref(store) if store else None, req, ok, max_req, ok, ok, ok,
                                   ok, cache_len, new_len, ok, ok)
    assert rel(store=None) == B.SWA_ERR_NULL
    assert rel(req=None) == B.SWA_ERR_NULL
    assert rel(max_req=0) == B.SWA_ERR_BAD_SHAPE
    assert rel(max_req=33) == B.SWA_ERR_BAD_SHAPE
    assert rel(cache_len=ok, new_len=ok) == B.SWA_ERR_BAD_SHAPE        # the new lengths need their own array
