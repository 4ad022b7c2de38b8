"""CPU-only checks of the C ABI: the library loads, exports what include/kb.h declares, and every
argument error that is decided on the host comes back as the documented status (no device work)."""
import ctypes
import os
import re

import pytest

from paper_2602_14293_amd import kb as kbmod

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = ctypes.c_void_p(1 << 20)          # a 256-byte aligned non-NULL "device pointer"; never dereferenced on the host


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(kbmod.LIB_PATH):
        from paper_2602_14293_amd import build

        build.build(verbose=False)
    return kbmod.lib()


def _create(L, d=128, dtype=kbmod.KB_BF16, cap=1000, scale=None, tags=None, keys=FAKE, inv=FAKE):
    h = ctypes.c_void_p()
    st = L.kb_create(ctypes.byref(h), d, dtype, cap, keys, scale, inv, tags)
    return st, h


def test_every_declared_symbol_is_exported(L):
    header = open(os.path.join(ROOT, "include", "kb.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(kb_[a-z_]+)\s*\(", header))
    assert {"kb_create", "kb_append", "kb_normalize", "kb_query_workspace_bytes", "kb_query", "kb_size",
            "kb_destroy", "kb_status_string", "kb_query_counters", "kb_set_tuning", "kb_query_sampled",
            "kb_quantize_rows", "kb_update_gain", "kb_remove", "kb_compact", "kb_compact_workspace_bytes", "kb_query_probe",
            "kb_query_probe_workspace_bytes"} <= names
    for n in names:
        assert hasattr(L, n), f"{n} is declared in kb.h but not exported by libkb.so"


def test_status_strings(L):
    seen = {L.kb_status_string(i) for i in range(9)}
    assert len(seen) == 9 and all(seen)


def test_create_argument_errors(L):
    assert L.kb_create(None, 128, 1, 10, FAKE, None, FAKE, None) == 1                 # KB_ERR_NULL
    assert _create(L, keys=None)[0] == 1
    assert _create(L, inv=None)[0] == 1
    assert _create(L, dtype=7)[0] == 3                                               # KB_ERR_DTYPE
    assert _create(L, d=0)[0] == 2 and _create(L, d=100)[0] == 2 and _create(L, d=-64)[0] == 2
    assert _create(L, d=32, dtype=kbmod.KB_F32)[0] == 0 and _create(L, d=32, dtype=kbmod.KB_BF16)[0] == 2
    assert _create(L, cap=0)[0] == 2 and _create(L, cap=1 << 31)[0] == 2
    assert _create(L, dtype=kbmod.KB_FP8_E4M3)[0] == 1                               # fp8 needs a row scale
    assert _create(L, dtype=kbmod.KB_FP8_E4M3, scale=FAKE)[0] == 0
    assert _create(L, dtype=kbmod.KB_BF16, scale=FAKE)[0] == 2                       # and the others must not have one
    assert _create(L, keys=ctypes.c_void_p((1 << 20) + 4))[0] == 2                   # misaligned keys


def test_append_and_query_argument_errors(L):
    st, h = _create(L, cap=100, tags=FAKE)
    assert st == 0 and L.kb_size(h) == 0 and L.kb_size(None) == -1
    first = ctypes.c_int64(-5)
    assert L.kb_append(None, FAKE, None, FAKE, 1, None, None) == 1
    assert L.kb_append(h, FAKE, None, FAKE, -1, None, None) == 2
    assert L.kb_append(h, FAKE, None, FAKE, 0, None, ctypes.byref(first)) == 0 and first.value == 0
    assert L.kb_append(h, None, None, FAKE, 5, None, None) == 1
    assert L.kb_append(h, FAKE, None, None, 5, None, None) == 1                      # tagged KB needs tags
    assert L.kb_append(h, FAKE, None, FAKE, 101, None, None) == 4                    # KB_ERR_CAPACITY
    assert L.kb_normalize(None, None) == 1 and L.kb_normalize(h, None) == 0          # nothing appended: no-op

    ws = L.kb_query_workspace_bytes(h, 8, 4)
    assert ws > 0 and ws % 256 == 0
    assert L.kb_query_workspace_bytes(h, 0, 4) == 0 and L.kb_query_workspace_bytes(h, 8, 129) == 0
    assert L.kb_query_workspace_bytes(None, 8, 4) == 0

    def q(handle=h, queries=FAKE, qd=kbmod.KB_BF16, Q=8, qmask=None, k=4, oi=FAKE, os_=FAKE, w=FAKE, wb=ws):
        return L.kb_query(handle, queries, qd, Q, qmask, k, oi, os_, w, wb, None)

    assert q(handle=None) == 1 and q(queries=None) == 1 and q(oi=None) == 1 and q(os_=None) == 1
    assert q(qd=kbmod.KB_F32) == 3 and q(qd=kbmod.KB_FP8_E4M3) == 3 and q(qd=9) == 3
    assert q(Q=0) == 2 and q(k=0) == 2 and q(k=129) == 2
    assert q(queries=ctypes.c_void_p((1 << 20) + 8)) == 2
    assert q(w=None) == 7 and q(w=ctypes.c_void_p((1 << 20) + 64)) == 7             # KB_ERR_WORKSPACE

    def qs(gain=FAKE, T=0.1, first=0, **kw):
        return L.kb_query_sampled(kw.get("handle", h), FAKE, kbmod.KB_BF16, kw.get("Q", 8), None, 4, gain, ctypes.c_float(T),
                                  ctypes.c_uint64(1), first, FAKE, FAKE, FAKE, ws, None)

    assert qs(gain=None) == 1                                                        # the weighted draw needs gains
    assert qs(T=0.0) == 2 and qs(T=-1.0) == 2 and qs(T=float("nan")) == 2 and qs(T=float("inf")) == 2
    assert qs(first=-1) == 2 and qs(gain=ctypes.c_void_p((1 << 20) + 2)) == 2
    assert qs(handle=None) == 1 and qs(Q=0) == 2                                     # then the checks of kb_query
    assert L.kb_destroy(h) == 0 and L.kb_destroy(None) == 1

    st, h2 = _create(L, cap=100)                                                      # untagged
    assert q(handle=h2, qmask=FAKE) == 6                                             # KB_ERR_NO_TAGS
    L.kb_destroy(h2)


def test_fp8_takes_bf16_or_fp8_queries(L):
    st, h = _create(L, dtype=kbmod.KB_FP8_E4M3, scale=FAKE)                          # d = 128
    ws = L.kb_query_workspace_bytes(h, 4, 4)
    assert L.kb_query(h, FAKE, kbmod.KB_F32, 4, None, 4, FAKE, FAKE, FAKE, ws, None) == 3
    assert L.kb_query(h, FAKE, kbmod.KB_FP8_E4M3, 4, None, 4, FAKE, FAKE, None, ws, None) == 7   # short rows too: accepted up to the workspace check
    L.kb_destroy(h)
    st, h = _create(L, d=512, dtype=kbmod.KB_FP8_E4M3, scale=FAKE)
    ws = L.kb_query_workspace_bytes(h, 4, 4)
    assert L.kb_query(h, FAKE, kbmod.KB_FP8_E4M3, 4, None, 4, FAKE, FAKE, None, ws, None) == 7   # accepted up to the workspace check
    assert L.kb_query(h, FAKE, kbmod.KB_BF16, 4, None, 4, FAKE, FAKE, None, ws, None) == 7
    assert L.kb_query_sampled(h, FAKE, kbmod.KB_FP8_E4M3, 4, None, 4, FAKE, ctypes.c_float(0.1), ctypes.c_uint64(1), 0,
                              FAKE, FAKE, None, ws, None) == 7                                  # the weighted draw takes them as well
    L.kb_destroy(h)
    st, h = _create(L, dtype=kbmod.KB_BF16)                                          # fp8 queries go with fp8 keys only
    assert L.kb_query(h, FAKE, kbmod.KB_FP8_E4M3, 4, None, 4, FAKE, FAKE, FAKE, 1 << 20, None) == 3
    L.kb_destroy(h)


def test_quantize_rows_argument_errors(L):
    def qr(rows=FAKE, dt=kbmod.KB_BF16, n=8, d=64, codes=FAKE, scale=FAKE):
        return L.kb_quantize_rows(rows, dt, n, d, codes, scale, None)

    assert qr(rows=None) == 1 and qr(codes=None) == 1
    assert qr(dt=kbmod.KB_FP8_E4M3) == 3 and qr(dt=5) == 3
    assert qr(n=-1) == 2 and qr(n=1 << 31) == 2 and qr(d=0) == 2 and qr(d=24) == 2 and qr(d=16400) == 2
    assert qr(rows=ctypes.c_void_p((1 << 20) + 8)) == 2 and qr(codes=ctypes.c_void_p((1 << 20) + 4)) == 2
    assert qr(scale=ctypes.c_void_p((1 << 20) + 2)) == 2
    assert qr(n=0) == 0 and qr(n=0, scale=None) == 0                                  # nothing to do, nothing launched


def test_maintenance_argument_errors(L):
    def ug(gain=FAKE, n=100, idx=FAKE, val=FAKE, m=4, alpha=0.5):
        return L.kb_update_gain(gain, n, idx, val, m, ctypes.c_float(alpha), None)

    assert ug(gain=None) == 1 and ug(idx=None) == 1 and ug(val=None) == 1
    assert ug(n=-1) == 2 and ug(m=-1) == 2 and ug(alpha=-0.1) == 2 and ug(alpha=1.5) == 2 and ug(alpha=float("nan")) == 2
    assert ug(idx=ctypes.c_void_p((1 << 20) + 2)) == 2 and ug(m=0) == 0

    st, a = _create(L, cap=100, tags=FAKE)
    st, b = _create(L, cap=100, tags=FAKE, keys=ctypes.c_void_p(2 << 20), inv=ctypes.c_void_p(3 << 20))
    assert L.kb_remove(None, FAKE, 1, None) == 1 and L.kb_remove(a, None, 1, None) == 1
    assert L.kb_remove(a, FAKE, -1, None) == 2 and L.kb_remove(a, FAKE, 0, None) == 0
    assert L.kb_remove(a, FAKE, 3, None) == 0                                        # empty knowledge base: nothing to mark
    ws = L.kb_compact_workspace_bytes(a)
    assert ws > 0 and ws % 256 == 0 and L.kb_compact_workspace_bytes(None) == 0
    live = ctypes.c_int64(-1)

    def cp(src=a, dst=b, gs=None, gd=None, imap=None, w=FAKE, wb=ws):
        return L.kb_compact(src, dst, gs, gd, imap, w, wb, None, ctypes.byref(live))

    assert cp(src=None) == 1 and cp(dst=None) == 1 and cp(dst=a) == 2               # a store cannot be compacted into itself
    assert cp(gs=FAKE) == 1 and cp(gd=FAKE) == 1                                     # the gain arrays come in pairs
    assert cp(w=None) == 7 and cp(wb=0) == 7 and cp(w=ctypes.c_void_p((1 << 20) + 64)) == 7
    assert cp() == 0 and live.value == 0 and L.kb_size(b) == 0                       # empty source: nothing launched
    st, c = _create(L, cap=100, keys=ctypes.c_void_p(4 << 20), inv=ctypes.c_void_p(5 << 20))           # untagged
    st, e = _create(L, d=256, cap=100, tags=FAKE, keys=ctypes.c_void_p(6 << 20), inv=ctypes.c_void_p(7 << 20))
    st, f = _create(L, dtype=kbmod.KB_F32, cap=100, tags=FAKE, keys=ctypes.c_void_p(8 << 20), inv=ctypes.c_void_p(9 << 20))
    assert cp(dst=c) == 2 and cp(dst=e) == 2 and cp(dst=f) == 3
    for h in (a, b, c, e, f):
        L.kb_destroy(h)


def test_probe_argument_errors(L):
    st, h = _create(L, cap=100, tags=FAKE)
    ws = L.kb_query_probe_workspace_bytes(h, 4, 8, 3)
    assert ws > 0 and ws % 256 == 0
    assert L.kb_query_probe_workspace_bytes(h, 0, 8, 3) == 0 and L.kb_query_probe_workspace_bytes(h, 4, 129, 3) == 0
    assert L.kb_query_probe_workspace_bytes(h, 4, 8, 0) == 0 and L.kb_query_probe_workspace_bytes(h, 4, 8, 65) == 0
    assert L.kb_query_probe_workspace_bytes(None, 4, 8, 3) == 0

    def qp(handle=h, queries=FAKE, qd=kbmod.KB_BF16, Q=4, qmask=None, k=8, off=FAKE, C=5, probe=FAKE, nprobe=3, oi=FAKE, os_=FAKE, w=FAKE, wb=ws):
        return L.kb_query_probe(handle, queries, qd, Q, qmask, k, off, C, probe, nprobe, oi, os_, w, wb, None)

    assert qp(handle=None) == 1 and qp(queries=None) == 1 and qp(off=None) == 1 and qp(probe=None) == 1 and qp(oi=None) == 1
    assert qp(qd=kbmod.KB_F32) == 3 and qp(qd=kbmod.KB_FP8_E4M3) == 3
    assert qp(Q=0) == 2 and qp(k=0) == 2 and qp(nprobe=0) == 2 and qp(nprobe=65) == 2 and qp(C=0) == 2
    assert qp(off=ctypes.c_void_p((1 << 20) + 4)) == 2 and qp(probe=ctypes.c_void_p((1 << 20) + 2)) == 2
    assert qp(w=None) == 7 and qp(wb=ws - 1) == 7
    L.kb_destroy(h)
    st, h2 = _create(L, cap=100)
    assert qp(handle=h2, qmask=FAKE) == 6
    L.kb_destroy(h2)


def test_tuning_knobs(L):
    st, h = _create(L)
    assert L.kb_set_tuning(h, b"sample_keys", 4096) == 0
    assert L.kb_set_tuning(h, b"scan_config", 3) == 0 and L.kb_set_tuning(h, b"scan_config", 99) == 2
    assert L.kb_set_tuning(h, b"wg_per_cu", 2) == 0 and L.kb_set_tuning(h, b"wg_per_cu", 64) == 2
    assert L.kb_set_tuning(h, b"small_path", 0) == 0 and L.kb_set_tuning(h, b"small_path", 1) == 0 and L.kb_set_tuning(h, b"small_path", 2) == 2
    assert L.kb_set_tuning(h, b"nonsense", 1) == 2 and L.kb_set_tuning(h, None, 1) == 1
    assert L.kb_check_draw_noise(None, None) == 1                                    # nowhere to write the result
    L.kb_destroy(h)


def test_workspace_size_covers_every_smaller_row_count(L):
    # sized at capacity; must stay sufficient while the KB grows from empty (checked via the size at smaller capacities)
    for dtype, scale in ((kbmod.KB_BF16, None), (kbmod.KB_F32, None), (kbmod.KB_FP8_E4M3, FAKE)):
        st, big = _create(L, d=256, dtype=dtype, cap=1 << 21, scale=scale)
        need_big = L.kb_query_workspace_bytes(big, 128, 16)
        for cap in (1, 100, 1000, 5000, 70000, 1 << 20, (1 << 21) - 1):
            st, small = _create(L, d=256, dtype=dtype, cap=cap, scale=scale)
            assert L.kb_query_workspace_bytes(small, 128, 16) <= need_big
            L.kb_destroy(small)
        L.kb_destroy(big)


def _dense_counts(cap, tile):
    """Row counts on both sides of every tile boundary near the small end, a stride through the rest, the counts a
    review found failing with an earlier sizing, and the capacity itself."""
    ns = set(range(0, min(cap, 70000) + 1, 61)) | {1, 2, cap - 1, cap}
    for t in range(1, min(cap // tile, 600) + 1):
        ns |= {t * tile - 1, t * tile, t * tile + 1}
    ns |= set(range(1, cap + 1, 4099))
    ns |= {(1 << 20) + j for j in (0, 1, 31, 32, 255, 256, 257)} | {131087, 1970178, (1 << 18) - 1, 1 << 18, (1 << 18) + 1}
    return sorted(n for n in ns if 0 <= n <= cap)


@pytest.mark.parametrize("dtype,d,cap,Q,k", [
    (kbmod.KB_BF16, 1024, 1 << 21, 128, 16),        # the growing knowledge base: one more row than 2^20 used to fail
    (kbmod.KB_BF16, 1024, 1 << 20, 256, 32),
    (kbmod.KB_BF16, 768, 65536, 64, 16),
    (kbmod.KB_BF16, 512, 1 << 19, 50, 24),          # 64-row tiles below 2^18 rows, the full-line kernel above
    (kbmod.KB_BF16, 256, 3_000_001, 300, 128),
    (kbmod.KB_BF16, 64, 1 << 22, 1, 1),
    (kbmod.KB_F32, 256, 4096, 8, 8),
    (kbmod.KB_F32, 64, 1 << 20, 40, 100),
    (kbmod.KB_FP8_E4M3, 768, 1 << 22, 1024, 64),
    (kbmod.KB_FP8_E4M3, 512, 1 << 19, 33, 7),
])
def test_workspace_size_bounds_the_plan_of_every_row_count(L, dtype, d, cap, Q, k):
    st, h = _create(L, d=d, dtype=dtype, cap=cap, scale=FAKE if dtype == kbmod.KB_FP8_E4M3 else None)
    assert st == 0
    need = L.kb_query_workspace_bytes(h, Q, k)
    assert need > 0 and need % 256 == 0
    worst = 0
    for kind in (0, 1, 2, 3):
        for n in _dense_counts(cap, 128):
            got = L.kb_query_plan_bytes(h, n, Q, k, kind)
            assert got <= need, f"kind {kind}: {n} rows need {got} bytes, kb_query_workspace_bytes says {need}"
            worst = max(worst, got)
    assert worst * 4 >= need, f"the bound {need} is far above the largest plan found ({worst})"
    assert L.kb_query_plan_bytes(h, cap + 1, Q, k, 0) == 0 and L.kb_query_plan_bytes(h, 5, Q, k, 4) == 0
    L.kb_destroy(h)


def test_workspace_size_follows_the_tuning_knobs(L):
    st, h = _create(L, d=1024, cap=1 << 20)
    for name, value in ((b"sample_keys", 4096), (b"scan_config", 3), (b"wg_per_cu", 2), (b"small_path", 0)):
        assert L.kb_set_tuning(h, name, value) == 0
        need = L.kb_query_workspace_bytes(h, 256, 32)
        for kind in (0, 1):
            for n in _dense_counts(1 << 20, 128)[::7]:
                assert L.kb_query_plan_bytes(h, n, 256, 32, kind) <= need, (name, n)
    L.kb_destroy(h)


def test_append_reports_the_first_index_only_on_success(L):
    st, h = _create(L, cap=10)
    first = ctypes.c_int64(-7)
    assert L.kb_append(h, FAKE, None, None, 11, None, ctypes.byref(first)) == 4 and first.value == -7     # KB_ERR_CAPACITY
    assert L.kb_append(h, None, None, None, 3, None, ctypes.byref(first)) == 1 and first.value == -7      # KB_ERR_NULL
    assert L.kb_append(h, FAKE, None, None, 0, None, ctypes.byref(first)) == 0 and first.value == 0       # a no-op reports the size
    L.kb_destroy(h)
