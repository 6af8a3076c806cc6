"""ctypes binding of librpa.so: argument marshalling only.

Every step of the path (cache update, attention, split merge, and the host
work partition) runs inside the library.  There is no fallback: if the library
is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librpa.so")

RPA_OK = 0
ERR_INVALID_ARG, ERR_BAD_LENGTHS, ERR_UNSUPPORTED, ERR_HIP, ERR_WORKSPACE = -1, -2, -3, -4, -5
VARIANT_AUTO, VARIANT_DECODE, VARIANT_PREFILL, VARIANT_MIXED = 0, 1, 2, 3
VARIANT_NAMES = {0: "auto", 1: "decode", 2: "prefill", 3: "mixed"}


class Shape(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "num_q_heads", "num_kv_heads", "head_dim", "page_size", "max_tokens", "max_seqs",
        "max_pages_per_seq", "num_pages", "non_causal", "kv_fp8")] + [("k_scale", C.c_float), ("v_scale", C.c_float),
                                                                      ("kv_merged", C.c_int32)]


class WorkUnit(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "seq", "q_start", "q_pos0", "n_q", "kv_begin", "kv_end", "ctx", "seq_q0", "part_row",
        "flags", "bin", "reserved")]


class CombineItem(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("part_row", "n_splits", "rows", "q_start")]


class PlanStats(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "variant", "num_narrow_units", "num_wide_units", "num_combine_items", "max_splits",
        "kv_chunk", "num_narrow_bins", "narrow_waves")] + [("partial_rows", C.c_int64),
                                                             ("workspace_bytes", C.c_int64),
                                                             ("wide_rows", C.c_int32), ("concurrent", C.c_int32)]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


class Options(C.Structure):
    _fields_ = [("variant", C.c_int32), ("kv_chunk", C.c_int32), ("wide_kv_chunk", C.c_int32),
                ("narrow_waves", C.c_int32), ("units_per_cu", C.c_int32), ("ablate", C.c_int32),
                ("wide_rows", C.c_int32), ("wide_order", C.c_int32), ("mixed_overlap", C.c_int32),
                ("stream_ordered_upload", C.c_int32), ("wide_persistent", C.c_int32)]


class RpaError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"rpa error {code}: {msg}")
        self.code = code


_lib = None

EXPORTS = ("rpa_create", "rpa_destroy", "rpa_update_and_attend", "rpa_last_error", "rpa_plan_info",
           "rpa_set_options", "rpa_set_regime_options", "rpa_plan_host", "rpa_profile_enable", "rpa_profile_read",
           "rpa_copy_probe", "rpa_mfma_probe", "rpa_update_and_attend_noalloc", "rpa_noalloc_last_error")


ABLATE_LIB_PATH = os.path.join(_HERE, "librpa_ablate.so")   # measurement build: the same code with -DRPA_ABLATE
_loaded = {}


def lib():
    """Load librpa.so (built in-tree by paper_2604_15464_amd/build.py)."""
    global _lib
    if _lib is None:
        _lib = load_library(LIB_PATH)
    return _lib


def load_library(path):
    """Load a build of the library and declare its entry points."""
    if path in _loaded:
        return _loaded[path]
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build it with `python -m paper_2604_15464_amd.build` "
                           "(there is no fallback path)")
    l = C.CDLL(path)
    l.rpa_create.argtypes = [C.POINTER(C.c_void_p), C.POINTER(Shape), C.c_int]
    l.rpa_create.restype = C.c_int
    l.rpa_destroy.argtypes = [C.c_void_p]
    l.rpa_destroy.restype = None
    l.rpa_update_and_attend.argtypes = [C.c_void_p] + [C.c_void_p] * 7 + [C.c_void_p, C.c_void_p,
                                                                            C.c_int32, C.c_float, C.c_void_p]
    l.rpa_update_and_attend.restype = C.c_int
    l.rpa_last_error.argtypes = [C.c_void_p]
    l.rpa_last_error.restype = C.c_char_p
    l.rpa_plan_info.argtypes = [C.c_void_p, C.POINTER(PlanStats)]
    l.rpa_plan_info.restype = C.c_int
    l.rpa_set_options.argtypes = [C.c_void_p, C.POINTER(Options)]
    l.rpa_set_options.restype = C.c_int
    l.rpa_set_regime_options.argtypes = [C.c_void_p, C.c_int32, C.POINTER(Options)]
    l.rpa_set_regime_options.restype = C.c_int
    l.rpa_profile_enable.argtypes = [C.c_void_p, C.c_int]
    l.rpa_profile_enable.restype = C.c_int
    l.rpa_profile_read.argtypes = [C.c_void_p, C.POINTER(C.c_float), C.POINTER(C.c_float), C.POINTER(C.c_float),
                                   C.POINTER(C.c_int32)]
    l.rpa_profile_read.restype = C.c_int
    l.rpa_plan_host.argtypes = [C.POINTER(Shape), C.c_void_p, C.c_void_p, C.c_int32, C.POINTER(Options), C.c_int,
                                C.POINTER(WorkUnit), C.c_int32, C.POINTER(CombineItem), C.c_int32,
                                C.POINTER(PlanStats)]
    l.rpa_plan_host.restype = C.c_int
    l.rpa_copy_probe.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p, C.POINTER(C.c_float)]
    l.rpa_copy_probe.restype = C.c_int
    l.rpa_mfma_probe.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.POINTER(C.c_float), C.POINTER(C.c_double)]
    l.rpa_mfma_probe.restype = C.c_int
    l.rpa_update_and_attend_noalloc.argtypes = [C.POINTER(Shape), C.c_int] + [C.c_void_p] * 7 + [
        C.c_void_p, C.c_void_p, C.c_int32, C.c_float, C.c_void_p]
    l.rpa_update_and_attend_noalloc.restype = C.c_int
    l.rpa_noalloc_last_error.argtypes = []
    l.rpa_noalloc_last_error.restype = C.c_char_p
    _loaded[path] = l
    return l


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(C.c_void_p)


def make_shape(num_q_heads, num_kv_heads, head_dim, page_size, max_tokens, max_seqs, max_pages_per_seq,
               num_pages, causal=True, kv_scales=None, kv_merged=False) -> Shape:
    """kv_scales = (k_scale, v_scale) selects the 8-bit (E4M3) cache; kv_merged the
    one-pool layout [num_pages, page_size, Hkv, 2, D] (K and V side by side)."""
    k_scale, v_scale = kv_scales if kv_scales is not None else (0.0, 0.0)
    return Shape(num_q_heads, num_kv_heads, head_dim, page_size, max_tokens, max_seqs, max_pages_per_seq,
                 num_pages, 0 if causal else 1, 0 if kv_scales is None else 1, k_scale, v_scale,
                 1 if kv_merged else 0)


def shape_key(shape: Shape) -> str:
    """Key of a shape in a tuning table: what the launch shapes depend on."""
    return (f"hq{shape.num_q_heads}_hkv{shape.num_kv_heads}_d{shape.head_dim}_ps{shape.page_size}"
            f"_{'fp8' if shape.kv_fp8 else 'bf16'}{'_nomask' if shape.non_causal else ''}"
            f"{'_merged' if shape.kv_merged else ''}")


def plan_host(shape: Shape, cu_q_lens, kv_lens, num_cus=256, variant=VARIANT_AUTO, kv_chunk=0,
              wide_kv_chunk=0, max_units=1 << 20, narrow_waves=0, wide_rows=0, mixed_overlap=0):
    """Host-only work partition (no GPU needed).  Returns (units, items, stats)
    with units/items as numpy structured views."""
    l = lib()
    cu, cu_p = _i32(cu_q_lens)
    kv, kv_p = _i32(kv_lens)
    n = len(kv)
    units = (WorkUnit * max_units)()
    items = (CombineItem * max_units)()
    stats = PlanStats()
    opt = Options(variant, kv_chunk, wide_kv_chunk, narrow_waves, 0, 0, wide_rows, 0, mixed_overlap, 0, 0)
    rc = l.rpa_plan_host(C.byref(shape), cu_p, kv_p, n, C.byref(opt), num_cus, units, max_units, items,
                         max_units, C.byref(stats))
    if rc != RPA_OK:
        raise RpaError(rc, l.rpa_last_error(None).decode())
    nu = stats.num_narrow_units + stats.num_wide_units
    u = np.frombuffer(units, dtype=np.int32).reshape(max_units, 12)[:nu].copy()
    it = np.frombuffer(items, dtype=np.int32).reshape(max_units, 4)[:stats.num_combine_items].copy()
    return u, it, stats.as_dict()


def update_and_attend_noalloc(shape: Shape, device, out_ptr, q_ptr, k_new_ptr, v_new_ptr, k_pages_ptr, v_pages_ptr,
                              page_table_ptr, cu_q_lens, kv_lens, sm_scale, stream_ptr):
    """rpa_update_and_attend_noalloc: pointers in, status out (no context, no
    allocation in the library); cu_q_lens / kv_lens are host int32 arrays."""
    l = lib()
    cu, cu_p = _i32(cu_q_lens)
    kv, kv_p = _i32(kv_lens)
    rc = l.rpa_update_and_attend_noalloc(C.byref(shape), int(device), out_ptr, q_ptr, k_new_ptr, v_new_ptr,
                                         k_pages_ptr, v_pages_ptr, page_table_ptr, cu_p, kv_p, len(kv),
                                         float(sm_scale), stream_ptr)
    if rc != RPA_OK:
        raise RpaError(rc, l.rpa_noalloc_last_error().decode())


UNIT_FIELDS = ("seq", "q_start", "q_pos0", "n_q", "kv_begin", "kv_end", "ctx", "seq_q0", "part_row", "flags",
               "bin")


class RaggedPagedAttention:
    """One context = one static shape on one GPU."""

    def __init__(self, num_q_heads, num_kv_heads, head_dim, page_size, max_tokens, max_seqs,
                 max_pages_per_seq, num_pages, device=0, causal=True, kv_scales=None, library=None, kv_merged=False):
        self._lib = lib() if library is None else library
        self.shape = make_shape(num_q_heads, num_kv_heads, head_dim, page_size, max_tokens, max_seqs,
                                max_pages_per_seq, num_pages, causal, kv_scales, kv_merged)
        self._ctx = C.c_void_p()
        rc = self._lib.rpa_create(C.byref(self._ctx), C.byref(self.shape), int(device))
        if rc != RPA_OK:
            raise RpaError(rc, self._lib.rpa_last_error(None).decode())
        self.device = int(device)

    @classmethod
    def for_workload(cls, wl, max_tokens=None, max_seqs=None, device=0, causal=True, kv_scales=None, library=None,
                     kv_merged=False):
        return cls(wl.num_q_heads, wl.num_kv_heads, wl.head_dim, wl.page_size,
                   max(1, max_tokens or wl.num_tokens), max(1, max_seqs or wl.num_seqs),
                   wl.max_pages_per_seq, wl.num_pages, device, causal, kv_scales, library, kv_merged)

    def close(self):
        if getattr(self, "_ctx", None) is not None and self._ctx.value:
            self._lib.rpa_destroy(self._ctx)
            self._ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_options(self, variant=VARIANT_AUTO, kv_chunk=0, wide_kv_chunk=0, narrow_waves=0, units_per_cu=0,
                    ablate=0, wide_rows=0, wide_order=0, mixed_overlap=0, stream_ordered_upload=0, wide_persistent=0):
        opt = Options(variant, kv_chunk, wide_kv_chunk, narrow_waves, units_per_cu, ablate, wide_rows, wide_order,
                      mixed_overlap, stream_ordered_upload, wide_persistent)
        rc = self._lib.rpa_set_options(self._ctx, C.byref(opt))
        if rc != RPA_OK:
            raise RpaError(rc, self._lib.rpa_last_error(self._ctx).decode())

    def set_regime_options(self, regime, **knobs):
        """Knobs used for the batches of one regime (VARIANT_DECODE / _PREFILL /
        _MIXED); no knobs = that regime's defaults.  See rpa_set_regime_options."""
        names = [n for n, _ in Options._fields_]
        opt = Options(*[int(knobs.pop(n, 0)) for n in names])
        if knobs:
            raise TypeError(f"unknown knobs {sorted(knobs)}")
        rc = self._lib.rpa_set_regime_options(self._ctx, int(regime), C.byref(opt))
        if rc != RPA_OK:
            raise RpaError(rc, self._lib.rpa_last_error(self._ctx).decode())

    def load_tuning(self, table):
        """Apply a table written by `python -m paper_2604_15464_amd.tune` (a dict or a
        JSON file path): the entry for this context's shape, one set of knobs per
        regime.  Returns the entry's key, or None if the table has none."""
        import json

        if not isinstance(table, dict):
            with open(table) as f:
                table = json.load(f)
        key = shape_key(self.shape)
        entry = table.get("shapes", {}).get(key)
        if entry is None:
            return None
        for name, regime in (("decode", VARIANT_DECODE), ("prefill", VARIANT_PREFILL), ("mixed", VARIANT_MIXED)):
            if name in entry:
                self.set_regime_options(regime, **entry[name]["knobs"])
        return key

    def plan_info(self) -> dict:
        st = PlanStats()
        rc = self._lib.rpa_plan_info(self._ctx, C.byref(st))
        if rc != RPA_OK:
            raise RpaError(rc, "rpa_plan_info")
        return st.as_dict()

    def profile_enable(self, on=True):
        rc = self._lib.rpa_profile_enable(self._ctx, 1 if on else 0)
        if rc != RPA_OK:
            raise RpaError(rc, self._lib.rpa_last_error(self._ctx).decode())

    def profile_read(self) -> dict:
        """Milliseconds per kernel summed over the calls since the last read."""
        a, b, c_, n = C.c_float(), C.c_float(), C.c_float(), C.c_int32()
        rc = self._lib.rpa_profile_read(self._ctx, C.byref(a), C.byref(b), C.byref(c_), C.byref(n))
        if rc != RPA_OK:
            raise RpaError(rc, self._lib.rpa_last_error(self._ctx).decode())
        return {"narrow_ms": a.value, "wide_ms": b.value, "combine_ms": c_.value, "calls": n.value}

    def copy_probe(self, dst, src, timed=True):
        """Plain streaming copy src -> dst (contiguous cuda tensors of equal byte
        size); returns the kernel's milliseconds when timed."""
        import torch

        nbytes = src.numel() * src.element_size()
        if dst.numel() * dst.element_size() != nbytes or not (src.is_contiguous() and dst.is_contiguous()):
            raise ValueError("copy_probe: contiguous tensors of equal byte size expected")
        ms = C.c_float()
        rc = self._lib.rpa_copy_probe(self._ctx, dst.data_ptr(), src.data_ptr(), nbytes,
                                      torch.cuda.current_stream(src.device).cuda_stream,
                                      C.byref(ms) if timed else None)
        if rc != RPA_OK:
            raise RpaError(rc, self._lib.rpa_last_error(self._ctx).decode())
        return ms.value if timed else None

    def mfma_probe(self, steps, device=None):
        """A launch of bf16 MFMAs alone on every compute unit; returns (milliseconds, FLOPs)."""
        import torch

        ms, flops = C.c_float(), C.c_double()
        rc = self._lib.rpa_mfma_probe(self._ctx, int(steps), torch.cuda.current_stream(device).cuda_stream,
                                      C.byref(ms), C.byref(flops))
        if rc != RPA_OK:
            raise RpaError(rc, self._lib.rpa_last_error(self._ctx).decode())
        return ms.value, flops.value

    def update_and_attend_raw(self, out_ptr, q_ptr, k_new_ptr, v_new_ptr, k_pages_ptr, v_pages_ptr,
                              page_table_ptr, cu_q_lens, kv_lens, num_seqs, sm_scale, stream_ptr):
        """Pointers in, status out: cu_q_lens / kv_lens are contiguous int32 numpy arrays."""
        rc = self._lib.rpa_update_and_attend(
            self._ctx, out_ptr, q_ptr, k_new_ptr, v_new_ptr, k_pages_ptr, v_pages_ptr, page_table_ptr,
            cu_q_lens.ctypes.data, kv_lens.ctypes.data, num_seqs, sm_scale, stream_ptr)
        if rc != RPA_OK:
            raise RpaError(rc, self._lib.rpa_last_error(self._ctx).decode())

    def update_and_attend(self, q, k_new, v_new, k_pages, v_pages, page_table, cu_q_lens, kv_lens,
                          sm_scale, out=None, stream=None):
        """torch tensors on this context's GPU (bf16, the page pools uint8 with
        the 8-bit cache; page_table int32); cu_q_lens / kv_lens host arrays.  k_pages / v_pages are updated in
        place; returns out.  The call is asynchronous on `stream` (default:
        torch's current stream)."""
        import torch

        cu = np.ascontiguousarray(cu_q_lens, dtype=np.int32)
        kv = np.ascontiguousarray(kv_lens, dtype=np.int32)
        n = int(kv.shape[0])
        if cu.shape[0] != n + 1:
            raise ValueError("cu_q_lens must have num_seqs + 1 entries")
        sh = self.shape
        pool_dtype = torch.uint8 if sh.kv_fp8 else torch.bfloat16     # 8-bit cache: E4M3 bytes
        pool_shape = (sh.num_pages, sh.page_size, sh.num_kv_heads, sh.head_dim)
        if sh.kv_merged:                    # one pool, K and V side by side; v_pages is not used
            pool_shape = (sh.num_pages, sh.page_size, sh.num_kv_heads, 2, sh.head_dim)
        checks = [("q", q, (sh.max_tokens, sh.num_q_heads, sh.head_dim), torch.bfloat16),
                  ("k_new", k_new, (sh.max_tokens, sh.num_kv_heads, sh.head_dim), torch.bfloat16),
                  ("v_new", v_new, (sh.max_tokens, sh.num_kv_heads, sh.head_dim), torch.bfloat16),
                  ("k_pages", k_pages, pool_shape, pool_dtype)]
        if not sh.kv_merged:
            checks.append(("v_pages", v_pages, pool_shape, pool_dtype))
        for name, t, shape, dtype in checks:
            if tuple(t.shape) != shape or t.dtype != dtype or not t.is_contiguous() or not t.is_cuda:
                raise ValueError(f"{name}: expected contiguous cuda {dtype} tensor of shape {shape}, "
                                 f"got {tuple(t.shape)} {t.dtype}")
        if (tuple(page_table.shape) != (sh.max_seqs, sh.max_pages_per_seq) or page_table.dtype != torch.int32
                or not page_table.is_contiguous() or not page_table.is_cuda):
            raise ValueError("page_table: expected contiguous cuda int32 [max_seqs, max_pages_per_seq]")
        if out is None:
            out = torch.empty_like(q)
        elif tuple(out.shape) != tuple(q.shape) or out.dtype != torch.bfloat16 or not out.is_contiguous():
            raise ValueError("out: wrong shape / dtype")
        st = torch.cuda.current_stream(q.device) if stream is None else stream
        self.update_and_attend_raw(out.data_ptr(), q.data_ptr(), k_new.data_ptr(), v_new.data_ptr(),
                                   k_pages.data_ptr(), None if sh.kv_merged else v_pages.data_ptr(), page_table.data_ptr(),
                                   cu, kv, n, float(sm_scale), st.cuda_stream)
        return out
