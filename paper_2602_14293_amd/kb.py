"""Thin binding of libkb.so (argument marshalling only; every step of retrieval runs in the HIP kernels).

PyTorch provides device memory and the stream.  The functions mirror the C ABI of ``include/kb.h``:
kb_create / kb_append / kb_normalize / kb_query_workspace_bytes / kb_query / kb_size / kb_destroy.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkb.so")

KB_F32, KB_BF16, KB_FP8_E4M3 = 0, 1, 2
KB_K_MAX = 128
STATUS_NAMES = ["KB_OK", "KB_ERR_NULL", "KB_ERR_INVALID_ARG", "KB_ERR_DTYPE", "KB_ERR_CAPACITY",
                "KB_ERR_NOT_NORMALIZED", "KB_ERR_NO_TAGS", "KB_ERR_WORKSPACE", "KB_ERR_DEVICE"]
_TORCH_DTYPE = {KB_F32: torch.float32, KB_BF16: torch.bfloat16, KB_FP8_E4M3: torch.float8_e4m3fn}
_CODE_OF = {v: k for k, v in _TORCH_DTYPE.items()}

_lib = None


class KBError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        name = STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else str(status)
        super().__init__(f"{where}: {name} ({lib().kb_status_string(status).decode()})")


def lib() -> ctypes.CDLL:
    """Load libkb.so; there is no fallback: a missing library is an error."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} has not been built: run `python -m paper_2602_14293_amd.build` "
                               "(or __graft_entry__.build())")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
        L.kb_create.restype = i32
        L.kb_create.argtypes = [ctypes.POINTER(vp), i32, i32, i64, vp, vp, vp, vp]
        L.kb_append.restype = i32
        L.kb_append.argtypes = [vp, vp, vp, vp, i64, vp, ctypes.POINTER(i64)]
        L.kb_normalize.restype = i32
        L.kb_normalize.argtypes = [vp, vp]
        L.kb_query_workspace_bytes.restype = sz
        L.kb_query_workspace_bytes.argtypes = [vp, i32, i32]
        L.kb_query_plan_bytes.restype = sz
        L.kb_query_plan_bytes.argtypes = [vp, i64, i32, i32, i32]
        L.kb_query.restype = i32
        L.kb_query.argtypes = [vp, vp, i32, i32, vp, i32, vp, vp, vp, sz, vp]
        L.kb_query_static.restype = i32
        L.kb_query_static.argtypes = [vp, vp, i32, i32, vp, i32, vp, vp, vp]
        L.kb_query_probe_workspace_bytes.restype = sz
        L.kb_query_probe_workspace_bytes.argtypes = [vp, i32, i32, i32]
        L.kb_query_probe.restype = i32
        L.kb_query_probe.argtypes = [vp, vp, i32, i32, vp, i32, vp, i32, vp, i32, vp, vp, vp, sz, vp]
        L.kb_update_gain.restype = i32
        L.kb_update_gain.argtypes = [vp, i64, vp, vp, i64, ctypes.c_float, vp]
        L.kb_remove.restype = i32
        L.kb_remove.argtypes = [vp, vp, i64, vp]
        L.kb_compact_workspace_bytes.restype = sz
        L.kb_compact_workspace_bytes.argtypes = [vp]
        L.kb_compact.restype = i32
        L.kb_compact.argtypes = [vp, vp, vp, vp, vp, vp, sz, vp, ctypes.POINTER(i64)]
        L.kb_quantize_rows.restype = i32
        L.kb_quantize_rows.argtypes = [vp, i32, i64, i32, vp, vp, vp]
        L.kb_query_sampled.restype = i32
        L.kb_query_sampled.argtypes = [vp, vp, i32, i32, vp, i32, vp, ctypes.c_float, ctypes.c_uint64, i32, vp, vp, vp, sz, vp]
        L.kb_check_draw_noise.restype = i32
        L.kb_check_draw_noise.argtypes = [vp, vp]
        L.kb_query_counters.restype = i32
        L.kb_query_counters.argtypes = [vp, vp, ctypes.POINTER(i64), vp]
        L.kb_set_tuning.restype = i32
        L.kb_set_tuning.argtypes = [vp, ctypes.c_char_p, i64]
        L.kb_profile_begin.restype = i32
        L.kb_profile_begin.argtypes = [vp, i32]
        L.kb_profile_end.restype = i32
        L.kb_profile_end.argtypes = [vp, vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i32)]
        L.kb_size.restype = i64
        L.kb_size.argtypes = [vp]
        L.kb_destroy.restype = i32
        L.kb_destroy.argtypes = [vp]
        L.kb_status_string.restype = ctypes.c_char_p
        L.kb_status_string.argtypes = [i32]
        _lib = L
    return _lib


def _check(status: int, where: str):
    if status != 0:
        raise KBError(status, where)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def quantize_rows(rows: torch.Tensor, want_scale: bool = True):
    """kb_quantize_rows: float32 / bfloat16 rows [n, d] on the GPU -> (float8_e4m3fn codes [n, d], float32 scale [n] or None)."""
    assert rows.is_cuda and rows.dim() == 2 and rows.is_contiguous()
    n, d = rows.shape
    codes = torch.empty((n, d), dtype=torch.float8_e4m3fn, device=rows.device)
    scale = torch.empty(n, dtype=torch.float32, device=rows.device) if want_scale else None
    _check(lib().kb_quantize_rows(_ptr(rows), _CODE_OF[rows.dtype], n, d, _ptr(codes), _ptr(scale), _stream()), "kb_quantize_rows")
    return codes, scale


def update_gain(gain: torch.Tensor, indices: torch.Tensor, values: torch.Tensor, alpha: float):
    """kb_update_gain: gain[indices] moves towards values by the factor alpha, in place."""
    assert gain.dtype == torch.float32 and indices.dtype == torch.int32 and values.dtype == torch.float32
    assert gain.is_contiguous() and indices.is_contiguous() and values.is_contiguous() and indices.numel() == values.numel()
    _check(lib().kb_update_gain(_ptr(gain), gain.numel(), _ptr(indices), _ptr(values), indices.numel(), ctypes.c_float(alpha),
                                _stream()), "kb_update_gain")


def check_draw_noise():
    """kb_check_draw_noise: (generator values whose noise falls below the previous value's, values looked at)."""
    out = torch.empty(2, dtype=torch.int64, device="cuda")
    _check(lib().kb_check_draw_noise(_ptr(out), _stream()), "kb_check_draw_noise")
    torch.cuda.synchronize()
    return int(out[0]), int(out[1])


class KnowledgeBase:
    """Owns the device buffers (torch tensors) and a kb_t handle over them."""

    def __init__(self, d: int, key_dtype: int, capacity: int, tagged: bool = False, device="cuda"):
        self.d, self.key_dtype, self.capacity, self.tagged = d, key_dtype, capacity, tagged
        self.device = torch.device(device)
        self.keys = torch.empty((capacity, d), dtype=_TORCH_DTYPE[key_dtype], device=self.device)
        self.scale = torch.empty(capacity, dtype=torch.float32, device=self.device) if key_dtype == KB_FP8_E4M3 else None
        self.inv_norm = torch.zeros(capacity, dtype=torch.float32, device=self.device)
        self.tags = torch.zeros(capacity, dtype=torch.int64, device=self.device) if tagged else None
        self._workspace = None
        self._probe_workspace = None
        self._workspace_need = {}      # (Q, k) -> kb_query_workspace_bytes: a function of the handle's settings only
        h = ctypes.c_void_p()
        _check(lib().kb_create(ctypes.byref(h), d, key_dtype, capacity, _ptr(self.keys), _ptr(self.scale),
                               _ptr(self.inv_norm), _ptr(self.tags)), "kb_create")
        self._h = h

    # -- C ABI, one method per entry point -------------------------------------------------------
    def append(self, rows: torch.Tensor, scale: Optional[torch.Tensor] = None, tags: Optional[torch.Tensor] = None) -> int:
        n = rows.shape[0]
        assert rows.dtype == self.keys.dtype and rows.is_contiguous() and (n == 0 or rows.shape[1] == self.d)
        first = ctypes.c_int64(-1)
        _check(lib().kb_append(self._h, _ptr(rows), _ptr(scale), _ptr(tags), n, _stream(), ctypes.byref(first)), "kb_append")
        return first.value

    def append_in_place(self, n: int) -> int:
        """Rows [size, size+n) were written into self.keys / self.scale / self.tags by the caller."""
        s = self.size
        first = ctypes.c_int64(-1)
        _check(lib().kb_append(self._h, _ptr(self.keys[s:s + n]), None if self.scale is None else _ptr(self.scale[s:s + n]),
                               None if self.tags is None else _ptr(self.tags[s:s + n]), n, _stream(), ctypes.byref(first)),
               "kb_append")
        return first.value

    def normalize(self):
        _check(lib().kb_normalize(self._h, _stream()), "kb_normalize")

    def workspace_bytes(self, Q: int, k: int) -> int:
        # (asked once per batch shape: the planner behind it walks every plan the handle can run, some tens of
        # microseconds of host time that a small query would otherwise pay on every call)
        need = self._workspace_need.get((Q, k))
        if need is None:
            need = self._workspace_need[(Q, k)] = lib().kb_query_workspace_bytes(self._h, Q, k)
        return need

    def query(self, queries: torch.Tensor, k: int, qmask: Optional[torch.Tensor] = None,
              out_index: Optional[torch.Tensor] = None, out_score: Optional[torch.Tensor] = None):
        Q = queries.shape[0]
        assert queries.is_contiguous() and queries.shape[1] == self.d
        need = self.workspace_bytes(Q, k)
        if need == 0:
            raise KBError(2, "kb_query_workspace_bytes")
        if self._workspace is None or self._workspace.numel() < need:
            self._workspace = torch.empty(need, dtype=torch.uint8, device=self.device)
        if out_index is None:
            out_index = torch.empty((Q, k), dtype=torch.int32, device=self.device)
        if out_score is None:
            out_score = torch.empty((Q, k), dtype=torch.float32, device=self.device)
        _check(lib().kb_query(self._h, _ptr(queries), _CODE_OF[queries.dtype], Q, _ptr(qmask), k, _ptr(out_index),
                              _ptr(out_score), _ptr(self._workspace), self._workspace.numel(), _stream()), "kb_query")
        return out_index, out_score

    def query_static(self, queries: torch.Tensor, k: int, qmask: Optional[torch.Tensor], out_index: torch.Tensor,
                     out_score: torch.Tensor):
        """kb_query_static: the query in the library's own scratch array; the caller passes inputs and outputs only."""
        Q = queries.shape[0]
        assert queries.is_contiguous() and queries.shape[1] == self.d
        assert out_index.shape == (Q, k) and out_index.dtype == torch.int32 and out_score.shape == (Q, k) and out_score.dtype == torch.float32
        _check(lib().kb_query_static(self._h, _ptr(queries), _CODE_OF[queries.dtype], Q, _ptr(qmask), k, _ptr(out_index),
                                     _ptr(out_score), _stream()), "kb_query_static")
        return out_index, out_score

    def query_sampled(self, queries: torch.Tensor, k: int, gain: torch.Tensor, temperature: float, seed: int,
                      qmask: Optional[torch.Tensor] = None, first_query: int = 0,
                      out_index: Optional[torch.Tensor] = None, out_key: Optional[torch.Tensor] = None):
        """Weighted random selection: k entries per query drawn without replacement, P ~ gain * exp(score / T)."""
        Q = queries.shape[0]
        assert queries.is_contiguous() and queries.shape[1] == self.d
        assert gain.dtype == torch.float32 and gain.is_contiguous() and gain.numel() >= self.size
        need = self.workspace_bytes(Q, k)
        if need == 0:
            raise KBError(2, "kb_query_workspace_bytes")
        if self._workspace is None or self._workspace.numel() < need:
            self._workspace = torch.empty(need, dtype=torch.uint8, device=self.device)
        if out_index is None:
            out_index = torch.empty((Q, k), dtype=torch.int32, device=self.device)
        if out_key is None:
            out_key = torch.empty((Q, k), dtype=torch.float32, device=self.device)
        _check(lib().kb_query_sampled(self._h, _ptr(queries), _CODE_OF[queries.dtype], Q, _ptr(qmask), k, _ptr(gain),
                                      ctypes.c_float(temperature), ctypes.c_uint64(seed & 0xFFFFFFFFFFFFFFFF), first_query,
                                      _ptr(out_index), _ptr(out_key), _ptr(self._workspace), self._workspace.numel(), _stream()),
               "kb_query_sampled")
        return out_index, out_key

    def query_probe(self, queries: torch.Tensor, k: int, cluster_offsets: torch.Tensor, probe: torch.Tensor,
                    qmask: Optional[torch.Tensor] = None):
        """kb_query_probe: exact top-k over the rows of the clusters probe[r, :] (cluster c = rows offsets[c] .. offsets[c+1])."""
        Q, nprobe = probe.shape
        assert queries.is_contiguous() and queries.shape == (Q, self.d)
        assert cluster_offsets.dtype == torch.int64 and cluster_offsets.is_contiguous() and probe.dtype == torch.int32 and probe.is_contiguous()
        need = lib().kb_query_probe_workspace_bytes(self._h, Q, k, nprobe)
        if need == 0:
            raise KBError(2, "kb_query_probe_workspace_bytes")
        if self._probe_workspace is None or self._probe_workspace.numel() < need:
            self._probe_workspace = torch.empty(need, dtype=torch.uint8, device=self.device)
        out_index = torch.empty((Q, k), dtype=torch.int32, device=self.device)
        out_score = torch.empty((Q, k), dtype=torch.float32, device=self.device)
        _check(lib().kb_query_probe(self._h, _ptr(queries), _CODE_OF[queries.dtype], Q, _ptr(qmask), k, _ptr(cluster_offsets),
                                    cluster_offsets.numel() - 1, _ptr(probe), nprobe, _ptr(out_index), _ptr(out_score),
                                    _ptr(self._probe_workspace), self._probe_workspace.numel(), _stream()), "kb_query_probe")
        return out_index, out_score

    def remove(self, indices: torch.Tensor):
        assert indices.dtype == torch.int32 and indices.is_contiguous()
        _check(lib().kb_remove(self._h, _ptr(indices), indices.numel(), _stream()), "kb_remove")

    def compact_into(self, dst: "KnowledgeBase", gain: Optional[torch.Tensor] = None, want_index_map: bool = True):
        """kb_compact: live entries of this knowledge base into the empty `dst`.  Returns (live, index_map, gain of dst)."""
        need = lib().kb_compact_workspace_bytes(self._h)
        ws = torch.empty(max(need, 256), dtype=torch.uint8, device=self.device)
        index_map = torch.empty(self.size, dtype=torch.int32, device=self.device) if want_index_map else None
        gain_dst = torch.empty(dst.capacity, dtype=torch.float32, device=self.device) if gain is not None else None
        live = ctypes.c_int64(-1)
        _check(lib().kb_compact(self._h, dst._h, _ptr(gain), _ptr(gain_dst), _ptr(index_map), _ptr(ws), ws.numel(), _stream(),
                                ctypes.byref(live)), "kb_compact")
        return live.value, index_map, None if gain_dst is None else gain_dst[:live.value]

    def counters(self) -> dict:
        out = (ctypes.c_int64 * 4)()
        _check(lib().kb_query_counters(self._h, _ptr(self._workspace), out, _stream()), "kb_query_counters")
        return {"candidates": out[0], "exhaustive_queries": out[1], "sample_keys": out[2], "scan_workgroups": out[3]}

    def profile_begin(self, max_calls: int):
        _check(lib().kb_profile_begin(self._h, max_calls), "kb_profile_begin")

    def profile_end(self):
        """(summed main-scan kernel milliseconds, number of recorded launches)"""
        ms, n = ctypes.c_double(0.0), ctypes.c_int32(0)
        _check(lib().kb_profile_end(self._h, _stream(), ctypes.byref(ms), ctypes.byref(n)), "kb_profile_end")
        return ms.value, n.value

    def set_tuning(self, name: str, value: int):
        _check(lib().kb_set_tuning(self._h, name.encode(), value), "kb_set_tuning")
        self._workspace_need.clear()        # the size depends on the knobs

    @property
    def size(self) -> int:
        return lib().kb_size(self._h)

    def close(self):
        if self._h:
            lib().kb_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
