"""ctypes marshalling for the C ABI in include/kvtc.h -- no arithmetic happens here."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence, Tuple

import numpy as np

KVTC_BF16, KVTC_F32 = 0, 1
_STATUS = {0: "KVTC_OK", 1: "KVTC_E_ARG", 2: "KVTC_E_UNSUPPORTED", 3: "KVTC_E_SMALL", 4: "KVTC_E_HIP", 5: "KVTC_E_NOMEM"}

# layout of kvtc_job: { int32 plan; int32 n_tokens; int64 x_row0; }
JOB_DTYPE = np.dtype([("plan", "<i4"), ("n_tokens", "<i4"), ("x_row0", "<i8")])


class KvtcError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{_STATUS.get(status, status)}: {message}")
        self.status = status


class _Group(C.Structure):
    _fields_ = [("n", C.c_uint16), ("bits", C.c_uint8), ("reserved", C.c_uint8)]


class KvtcSplit(C.Structure):
    _fields_ = [("n_sink", C.c_int64), ("n_coded", C.c_int64), ("n_window", C.c_int64)]


class KvtcLayout(C.Structure):
    _fields_ = [("token_stride", C.c_int64), ("block_features", C.c_int32), ("reserved", C.c_int32), ("block_stride", C.c_int64)]


def lib_path() -> str:
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libkvtc.so")


_lib = None


def lib() -> C.CDLL:
    """The loaded library; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        path = lib_path()
        if not os.path.exists(path):
            raise RuntimeError(f"{path} is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'`")
        L = C.CDLL(path)
        vp, i64, sz = C.c_void_p, C.c_int64, C.c_size_t
        L.kvtc_plan_create.argtypes = [C.POINTER(vp), C.c_int, C.c_int, vp, vp, C.c_int, vp, vp]
        L.kvtc_plan_create.restype = C.c_int
        L.kvtc_plan_destroy.argtypes = [vp]
        L.kvtc_plan_destroy.restype = None
        L.kvtc_record_bytes.argtypes = [vp]
        L.kvtc_record_bytes.restype = sz
        L.kvtc_encoded_bytes.argtypes = [vp, i64]
        L.kvtc_encoded_bytes.restype = sz
        L.kvtc_encode.argtypes = [vp, vp, C.c_int, i64, i64, vp, sz, vp]
        L.kvtc_encode.restype = C.c_int
        L.kvtc_decode.argtypes = [vp, vp, sz, i64, vp, C.c_int, i64, vp]
        L.kvtc_decode.restype = C.c_int
        L.kvtc_batch_create.argtypes = [C.POINTER(vp), C.POINTER(vp), C.c_int, vp]
        L.kvtc_batch_create.restype = C.c_int
        L.kvtc_batch_destroy.argtypes = [vp]
        L.kvtc_batch_destroy.restype = None
        L.kvtc_offsets.argtypes = [vp, vp, C.c_int, vp, vp]
        L.kvtc_offsets.restype = C.c_int
        L.kvtc_encode_batch.argtypes = [vp, vp, C.c_int, vp, C.c_int, i64, vp, vp, sz, vp, vp]
        L.kvtc_encode_batch.restype = C.c_int
        L.kvtc_encode_batch_static.argtypes = [C.POINTER(vp), C.c_int, vp, C.c_int, vp, C.c_int, i64, vp, sz, vp, vp, vp]
        L.kvtc_encode_batch_static.restype = C.c_int
        L.kvtc_decode_batch.argtypes = [vp, vp, C.c_int, vp, sz, vp, vp, C.c_int, i64, vp, vp]
        L.kvtc_decode_batch.restype = C.c_int
        L.kvtc_window_split.argtypes = [i64, C.c_int, C.c_int, C.c_int, C.POINTER(KvtcSplit)]
        L.kvtc_cr_with_window.argtypes = [C.c_double, C.c_double, C.c_double, C.c_double]
        L.kvtc_cr_with_window.restype = C.c_double
        L.kvtc_fp8_pack.argtypes = [vp, C.c_int, i64, C.c_int, i64, vp, sz, vp]
        L.kvtc_fp8_unpack.argtypes = [vp, sz, i64, C.c_int, vp, C.c_int, i64, vp]
        L.kvtc_offsets_append.argtypes = [vp, vp, C.c_int, vp, vp, vp, vp]
        lp = C.POINTER(KvtcLayout)
        L.kvtc_encode_blocked.argtypes = [vp, vp, C.c_int, i64, lp, vp, sz, vp]
        L.kvtc_decode_blocked.argtypes = [vp, vp, sz, i64, vp, C.c_int, lp, vp]
        L.kvtc_encode_batch_blocked.argtypes = [vp, vp, C.c_int, vp, C.c_int, lp, vp, vp, sz, vp, vp]
        L.kvtc_decode_batch_blocked.argtypes = [vp, vp, C.c_int, vp, sz, vp, vp, C.c_int, lp, vp, vp]
        for f in (L.kvtc_encode_blocked, L.kvtc_decode_blocked, L.kvtc_encode_batch_blocked, L.kvtc_decode_batch_blocked):
            f.restype = C.c_int
        L.kvtc_wide_create.argtypes = [C.POINTER(vp), C.c_int, C.c_int, vp, vp, C.c_int, vp, vp]
        L.kvtc_wide_destroy.argtypes = [vp]
        L.kvtc_wide_destroy.restype = None
        L.kvtc_wide_sections.argtypes = [vp]
        L.kvtc_wide_sections.restype = C.c_int
        L.kvtc_wide_section_record_bytes.argtypes = [vp, C.c_int]
        L.kvtc_wide_section_record_bytes.restype = sz
        L.kvtc_wide_record_bytes.argtypes = [vp]
        L.kvtc_wide_record_bytes.restype = sz
        L.kvtc_wide_encoded_bytes.argtypes = [vp, i64]
        L.kvtc_wide_encoded_bytes.restype = sz
        L.kvtc_wide_encode.argtypes = [vp, vp, C.c_int, i64, lp, vp, sz, vp]
        L.kvtc_wide_decode.argtypes = [vp, vp, sz, i64, vp, C.c_int, lp, vp, vp]
        for f in (L.kvtc_wide_create, L.kvtc_wide_encode, L.kvtc_wide_decode):
            f.restype = C.c_int
        L.kvtc_entropy_create.argtypes = [C.POINTER(vp), C.c_int, C.c_int, vp, vp]
        L.kvtc_entropy_destroy.argtypes = [vp]
        L.kvtc_entropy_destroy.restype = None
        L.kvtc_entropy_bound.argtypes = [vp, i64]
        L.kvtc_entropy_bound.restype = sz
        L.kvtc_entropy_encode.argtypes = [vp, C.c_int, vp, i64, vp, sz, vp, vp]
        L.kvtc_entropy_decode.argtypes = [vp, C.c_int, vp, sz, i64, vp, sz, vp]
        L.kvtc_entropy_encode_batch.argtypes = [vp, vp, C.c_int, i64, vp, sz, vp, sz, vp, vp]
        L.kvtc_entropy_decode_batch.argtypes = [vp, vp, C.c_int, i64, vp, sz, vp, sz, vp]
        for f in (L.kvtc_entropy_create, L.kvtc_entropy_encode, L.kvtc_entropy_decode, L.kvtc_entropy_encode_batch, L.kvtc_entropy_decode_batch):
            f.restype = C.c_int
        L.kvtc_calib_block_errors.argtypes = [vp, i64, i64, vp, C.c_int, C.c_int, vp, vp]
        L.kvtc_calib_block_errors.restype = C.c_int
        L.kvtc_calib_moments.argtypes = [vp, C.c_int, i64, C.c_int, lp, vp, vp, vp]
        L.kvtc_calib_moments.restype = C.c_int
        L.kvtc_rope.argtypes = [vp, C.c_int, i64, C.c_int, C.c_int, i64, i64, vp, i64, C.c_double, C.c_int, C.c_int, vp]
        L.kvtc_rope.restype = C.c_int
        L.kvtc_last_error.argtypes = []
        L.kvtc_last_error.restype = C.c_char_p
        L.kvtc_host_f16_round_down.argtypes = [C.c_float]
        L.kvtc_host_f16_round_down.restype = C.c_uint16
        L.kvtc_host_f16_round_up.argtypes = [C.c_float]
        L.kvtc_host_f16_round_up.restype = C.c_uint16
        L.kvtc_host_group_header.argtypes = [C.c_float, C.c_float, C.c_int, C.POINTER(C.c_uint16), C.POINTER(C.c_uint16)]
        L.kvtc_host_group_header.restype = None
        L.kvtc_host_code.argtypes = [C.c_float, C.c_uint16, C.c_uint16, C.c_int]
        L.kvtc_host_code.restype = C.c_uint32
        L.kvtc_probe_stream.argtypes = [C.c_int, vp, vp, sz, vp]
        L.kvtc_probe_mfma_bf16.argtypes = [C.c_int, C.c_int, vp, C.POINTER(C.c_double), vp]
        _lib = L
    return _lib


def kvtc_last_error() -> str:
    return lib().kvtc_last_error().decode()


def _check(status: int) -> None:
    if status != 0:
        raise KvtcError(status, kvtc_last_error())


def _ptr(t) -> Optional[int]:
    """Device/host address of a torch tensor, numpy array, int or None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if isinstance(t, np.ndarray):
        return t.ctypes.data
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


# ---- plain wrappers, one per C entry point ---------------------------------------------------

def kvtc_plan_create(p: int, r: int, mu_host: np.ndarray, v_kept_host: np.ndarray,
                     groups: Sequence[Sequence[int]], stream=None) -> int:
    mu = np.ascontiguousarray(mu_host, dtype=np.float32)
    v = np.ascontiguousarray(v_kept_host, dtype=np.uint16)
    assert mu.shape == (p,) and v.shape == (p, r), (mu.shape, v.shape)
    arr = (_Group * len(groups))(*[_Group(int(n), int(b), 0) for n, b in groups])
    out = C.c_void_p()
    _check(lib().kvtc_plan_create(C.byref(out), p, r, mu.ctypes.data, v.ctypes.data, len(groups),
                                  C.cast(arr, C.c_void_p), _stream(stream)))
    return out.value


def kvtc_plan_destroy(plan: int) -> None:
    lib().kvtc_plan_destroy(plan)


def kvtc_record_bytes(plan: int) -> int:
    return lib().kvtc_record_bytes(plan)


def kvtc_encoded_bytes(plan: int, n_tokens: int) -> int:
    return lib().kvtc_encoded_bytes(plan, n_tokens)


def kvtc_encode(plan: int, x_dev, dtype: int, n_tokens: int, ld_x: int, out_dev, out_cap: int, stream=None) -> None:
    _check(lib().kvtc_encode(plan, _ptr(x_dev), dtype, n_tokens, ld_x, _ptr(out_dev), out_cap, _stream(stream)))


def kvtc_decode(plan: int, in_dev, in_bytes: int, n_tokens: int, x_out_dev, dtype: int, ld_x: int, stream=None) -> None:
    _check(lib().kvtc_decode(plan, _ptr(in_dev), in_bytes, n_tokens, _ptr(x_out_dev), dtype, ld_x, _stream(stream)))


def kvtc_batch_create(plans: Sequence[int], stream=None) -> int:
    arr = (C.c_void_p * len(plans))(*plans)
    out = C.c_void_p()
    _check(lib().kvtc_batch_create(C.byref(out), arr, len(plans), _stream(stream)))
    return out.value


def kvtc_batch_destroy(batch: int) -> None:
    lib().kvtc_batch_destroy(batch)


def kvtc_offsets(batch: int, jobs_dev, n_jobs: int, offsets_dev, stream=None) -> None:
    _check(lib().kvtc_offsets(batch, _ptr(jobs_dev), n_jobs, _ptr(offsets_dev), _stream(stream)))


def kvtc_encode_batch(batch: int, jobs_dev, n_jobs: int, x_base_dev, dtype: int, ld_x: int, offsets_dev,
                      out_base_dev, out_cap: int, status_dev, stream=None) -> None:
    _check(lib().kvtc_encode_batch(batch, _ptr(jobs_dev), n_jobs, _ptr(x_base_dev), dtype, ld_x, _ptr(offsets_dev),
                                   _ptr(out_base_dev), out_cap, _ptr(status_dev), _stream(stream)))


def kvtc_encode_batch_static(plans: Sequence[int], jobs_dev, n_jobs: int, x_base_dev, dtype: int, ld_x: int,
                             out_base_dev, out_cap: int, offsets_out_dev, status_dev, stream=None) -> None:
    arr = (C.c_void_p * len(plans))(*plans)
    _check(lib().kvtc_encode_batch_static(arr, len(plans), _ptr(jobs_dev), n_jobs, _ptr(x_base_dev), dtype, ld_x,
                                          _ptr(out_base_dev), out_cap, _ptr(offsets_out_dev), _ptr(status_dev), _stream(stream)))


def kvtc_decode_batch(batch: int, jobs_dev, n_jobs: int, in_base_dev, in_bytes: int, offsets_dev, x_out_base_dev,
                      dtype: int, ld_x: int, status_dev, stream=None) -> None:
    _check(lib().kvtc_decode_batch(batch, _ptr(jobs_dev), n_jobs, _ptr(in_base_dev), in_bytes, _ptr(offsets_dev),
                                   _ptr(x_out_base_dev), dtype, ld_x, _ptr(status_dev), _stream(stream)))


def kvtc_window_split(ctx: int, s: int = 4, w: int = 128, c: int = 16) -> Tuple[int, int, int]:
    out = KvtcSplit()
    _check(lib().kvtc_window_split(ctx, s, w, c, C.byref(out)))
    return out.n_sink, out.n_coded, out.n_window


def kvtc_cr_with_window(ctx: float, w: float, s: float, cr: float) -> float:
    return lib().kvtc_cr_with_window(ctx, w, s, cr)


def kvtc_fp8_pack(x_dev, dtype: int, n_tokens: int, p: int, ld_x: int, out_dev, out_cap: int, stream=None) -> None:
    _check(lib().kvtc_fp8_pack(_ptr(x_dev), dtype, n_tokens, p, ld_x, _ptr(out_dev), out_cap, _stream(stream)))


def kvtc_fp8_unpack(in_dev, in_bytes: int, n_tokens: int, p: int, x_out_dev, dtype: int, ld_x: int, stream=None) -> None:
    _check(lib().kvtc_fp8_unpack(_ptr(in_dev), in_bytes, n_tokens, p, _ptr(x_out_dev), dtype, ld_x, _stream(stream)))


def kvtc_offsets_append(batch: int, jobs_dev, n_jobs: int, region_dev, n_coded_dev, offsets_dev, stream=None) -> None:
    _check(lib().kvtc_offsets_append(batch, _ptr(jobs_dev), n_jobs, _ptr(region_dev), _ptr(n_coded_dev), _ptr(offsets_dev),
                                     _stream(stream)))


PROBE_READ, PROBE_WRITE, PROBE_COPY = 0, 1, 2


ROPE_HALF, ROPE_INTERLEAVED = 0, 1


def layout(token_stride: int, block_features: int = 0, block_stride: int = 0) -> "KvtcLayout":
    """A kvtc_layout: feature f of token t at t * token_stride + (f // block_features) * block_stride + f % block_features."""
    return KvtcLayout(token_stride, block_features, 0, block_stride)


def kvtc_encode_blocked(plan, x_dev, dtype: int, n_tokens: int, lay, out_dev, out_cap: int, stream=None) -> None:
    _check(lib().kvtc_encode_blocked(plan, _ptr(x_dev), dtype, n_tokens, C.byref(lay), _ptr(out_dev), out_cap, _stream(stream)))


def kvtc_decode_blocked(plan, in_dev, in_bytes: int, n_tokens: int, x_out_dev, dtype: int, lay, stream=None) -> None:
    _check(lib().kvtc_decode_blocked(plan, _ptr(in_dev), in_bytes, n_tokens, _ptr(x_out_dev), dtype, C.byref(lay), _stream(stream)))


def kvtc_encode_batch_blocked(batch, jobs_dev, n_jobs: int, x_base_dev, dtype: int, lay, offsets_dev, out_base_dev,
                              out_cap: int, status_dev, stream=None) -> None:
    _check(lib().kvtc_encode_batch_blocked(batch, _ptr(jobs_dev), n_jobs, _ptr(x_base_dev), dtype, C.byref(lay), _ptr(offsets_dev),
                                           _ptr(out_base_dev), out_cap, _ptr(status_dev), _stream(stream)))


def kvtc_decode_batch_blocked(batch, jobs_dev, n_jobs: int, in_base_dev, in_bytes: int, offsets_dev, x_out_base_dev,
                              dtype: int, lay, status_dev, stream=None) -> None:
    _check(lib().kvtc_decode_batch_blocked(batch, _ptr(jobs_dev), n_jobs, _ptr(in_base_dev), in_bytes, _ptr(offsets_dev),
                                           _ptr(x_out_base_dev), dtype, C.byref(lay), _ptr(status_dev), _stream(stream)))


def kvtc_rope(x_dev, dtype: int, n_tokens: int, n_heads: int, d_head: int, token_stride: int, head_stride: int,
              positions_dev, position0: int, base: float, pairing: int, inverse: bool, stream=None) -> None:
    _check(lib().kvtc_rope(_ptr(x_dev), dtype, n_tokens, n_heads, d_head, token_stride, head_stride,
                           _ptr(positions_dev) if positions_dev is not None else None, position0, float(base), pairing,
                           1 if inverse else 0, _stream(stream)))


def kvtc_probe_stream(mode: int, src_dev, dst_dev, nbytes: int, stream=None) -> None:
    _check(lib().kvtc_probe_stream(mode, _ptr(src_dev), _ptr(dst_dev), nbytes, _stream(stream)))


def kvtc_probe_mfma_bf16(iters: int, random_operands: int, sink_dev, stream=None) -> float:
    """Launches the matrix-core loop; returns the floating-point operations of the launch."""
    flops = C.c_double()
    _check(lib().kvtc_probe_mfma_bf16(iters, random_operands, _ptr(sink_dev), C.byref(flops), _stream(stream)))
    return flops.value


def make_jobs(plan_idx: Sequence[int], n_tokens: Sequence[int], x_row0: Sequence[int]) -> np.ndarray:
    """Host image of a kvtc_job array (copy it to the device as raw bytes)."""
    jobs = np.zeros(len(plan_idx), dtype=JOB_DTYPE)
    jobs["plan"], jobs["n_tokens"], jobs["x_row0"] = plan_idx, n_tokens, x_row0
    return jobs


# ---- small owners so handles are released --------------------------------------------------------

class Plan:
    """Owns a kvtc_plan handle."""

    def __init__(self, p: int, r: int, mu_host, v_kept_host, groups, stream=None):
        self.p, self.r, self.groups = p, r, [(int(n), int(b)) for n, b in groups]
        self.handle = kvtc_plan_create(p, r, mu_host, v_kept_host, self.groups, stream)
        self.record_bytes = kvtc_record_bytes(self.handle)

    def close(self):
        if getattr(self, "handle", None):
            kvtc_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def kvtc_wide_create(p: int, r: int, mu_host: np.ndarray, v_kept_host: np.ndarray,
                     groups: Sequence[Sequence[int]], stream=None) -> int:
    mu = np.ascontiguousarray(mu_host, dtype=np.float32)
    v = np.ascontiguousarray(v_kept_host, dtype=np.uint16)
    assert mu.shape == (p,) and v.shape == (p, r), (mu.shape, v.shape)
    arr = (_Group * len(groups))(*[_Group(int(n), int(b), 0) for n, b in groups])
    out = C.c_void_p()
    _check(lib().kvtc_wide_create(C.byref(out), p, r, mu.ctypes.data, v.ctypes.data, len(groups),
                                  C.cast(arr, C.c_void_p), _stream(stream)))
    return out.value


def kvtc_wide_destroy(w: int) -> None:
    lib().kvtc_wide_destroy(w)


def kvtc_wide_sections(w: int) -> int:
    return lib().kvtc_wide_sections(w)


def kvtc_wide_section_record_bytes(w: int, section: int) -> int:
    return lib().kvtc_wide_section_record_bytes(w, section)


def kvtc_wide_record_bytes(w: int) -> int:
    return lib().kvtc_wide_record_bytes(w)


def kvtc_wide_encoded_bytes(w: int, n_tokens: int) -> int:
    return lib().kvtc_wide_encoded_bytes(w, n_tokens)


def kvtc_wide_encode(w, x_dev, dtype: int, n_tokens: int, lay, out_dev, out_cap: int, stream=None) -> None:
    _check(lib().kvtc_wide_encode(w, _ptr(x_dev), dtype, n_tokens, C.byref(lay), _ptr(out_dev), out_cap, _stream(stream)))


def kvtc_wide_decode(w, in_dev, in_bytes: int, n_tokens: int, x_out_dev, dtype: int, lay, sum_dev=None, stream=None) -> None:
    _check(lib().kvtc_wide_decode(w, _ptr(in_dev), in_bytes, n_tokens, _ptr(x_out_dev), dtype, C.byref(lay),
                                  _ptr(sum_dev) if sum_dev is not None else None, _stream(stream)))


class WidePlan:
    """Owns a kvtc_wide handle."""

    def __init__(self, p: int, r: int, mu_host, v_kept_host, groups, stream=None):
        self.p, self.r = p, r
        self.handle = kvtc_wide_create(p, r, mu_host, v_kept_host, groups, stream)
        self.record_bytes = kvtc_wide_record_bytes(self.handle)
        self.n_sections = kvtc_wide_sections(self.handle)

    def close(self):
        if getattr(self, "handle", None):
            kvtc_wide_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# layout of kvtc_entropy_job: { int32 table; int32 n_tokens; uint64 records_off; uint64 coded_off; uint64 coded_cap; }
ENTROPY_JOB_DTYPE = np.dtype([("table", "<i4"), ("n_tokens", "<i4"), ("records_off", "<u8"), ("coded_off", "<u8"), ("coded_cap", "<u8")])


def make_entropy_jobs(tables, n_tokens, records_off, coded_off, coded_cap) -> np.ndarray:
    """A host kvtc_entropy_job table (copy it to the device yourself)."""
    jobs = np.zeros(len(tables), dtype=ENTROPY_JOB_DTYPE)
    jobs["table"], jobs["n_tokens"], jobs["records_off"] = tables, n_tokens, records_off
    jobs["coded_off"], jobs["coded_cap"] = coded_off, coded_cap
    return jobs


def kvtc_entropy_create(record_bytes: int, code_len_host: np.ndarray, stream=None) -> int:
    """code_len_host: [record_bytes][256] (one table set) or [n_tables][record_bytes][256]."""
    L = np.ascontiguousarray(code_len_host, dtype=np.uint8)
    if L.ndim == 2:
        L = L[None]
    assert L.shape[1:] == (record_bytes, 256), L.shape
    out = C.c_void_p()
    _check(lib().kvtc_entropy_create(C.byref(out), record_bytes, L.shape[0], L.ctypes.data, _stream(stream)))
    return out.value


def kvtc_entropy_destroy(e: int) -> None:
    lib().kvtc_entropy_destroy(e)


def kvtc_entropy_bound(e: int, n_tokens: int) -> int:
    return lib().kvtc_entropy_bound(e, n_tokens)


def kvtc_entropy_encode(e, records_dev, n_tokens: int, out_dev, out_cap: int, out_bytes_dev, table: int = 0, stream=None) -> None:
    _check(lib().kvtc_entropy_encode(e, table, _ptr(records_dev), n_tokens, _ptr(out_dev), out_cap, _ptr(out_bytes_dev), _stream(stream)))


def kvtc_entropy_decode(e, in_dev, in_bytes: int, n_tokens: int, records_out_dev, out_cap: int, table: int = 0, stream=None) -> None:
    _check(lib().kvtc_entropy_decode(e, table, _ptr(in_dev), in_bytes, n_tokens, _ptr(records_out_dev), out_cap, _stream(stream)))


def kvtc_entropy_encode_batch(e, jobs_dev, n_jobs: int, max_tokens: int, records_base_dev, records_bytes: int, coded_base_dev,
                              coded_cap: int, coded_bytes_dev, stream=None) -> None:
    _check(lib().kvtc_entropy_encode_batch(e, _ptr(jobs_dev), n_jobs, max_tokens, _ptr(records_base_dev), records_bytes,
                                           _ptr(coded_base_dev), coded_cap, _ptr(coded_bytes_dev), _stream(stream)))


def kvtc_entropy_decode_batch(e, jobs_dev, n_jobs: int, max_tokens: int, coded_base_dev, coded_bytes: int, records_base_dev,
                              records_cap: int, stream=None) -> None:
    _check(lib().kvtc_entropy_decode_batch(e, _ptr(jobs_dev), n_jobs, max_tokens, _ptr(coded_base_dev), coded_bytes,
                                           _ptr(records_base_dev), records_cap, _stream(stream)))


class EntropyTables:
    """Owns a kvtc_entropy handle (one or several table sets for records of one size)."""

    def __init__(self, record_bytes: int, code_len_host, stream=None):
        self.record_bytes = record_bytes
        self.handle = kvtc_entropy_create(record_bytes, code_len_host, stream)

    def close(self):
        if getattr(self, "handle", None):
            kvtc_entropy_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def kvtc_calib_block_errors(coef_dev, n_tokens: int, ld: int, blocks_dev, n_blocks: int, max_bits: int, change_dev, stream=None) -> None:
    """blocks_dev: device array of int32 pairs (start, n); change_dev: [n_blocks][max_bits] float64 on the device."""
    _check(lib().kvtc_calib_block_errors(_ptr(coef_dev), n_tokens, ld, _ptr(blocks_dev), n_blocks, max_bits, _ptr(change_dev), _stream(stream)))


def kvtc_calib_moments(x_dev, dtype: int, n_tokens: int, p: int, lay, sum_dev, gram_dev, stream=None) -> None:
    _check(lib().kvtc_calib_moments(_ptr(x_dev), dtype, n_tokens, p, C.byref(lay), _ptr(sum_dev), _ptr(gram_dev), _stream(stream)))


class Batch:
    """Owns a kvtc_batch handle (and keeps its plans alive)."""

    def __init__(self, plans: Sequence[Plan], stream=None):
        self.plans = list(plans)
        self.handle = kvtc_batch_create([p.handle for p in self.plans], stream)

    def close(self):
        if getattr(self, "handle", None):
            kvtc_batch_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
