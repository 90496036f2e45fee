"""MI355X-native KV-cache transform coder (encode/decode hot path of KVTC).

Thin ctypes binding over libkvtc.so (HIP kernels for gfx950 behind a C ABI, see
include/kvtc.h).  PyTorch is only used by callers for device memory and streams.
Importing the package never needs the GPU; calling into it without a built
library raises.
"""
from .binding import (  # noqa: F401
    KVTC_BF16, KVTC_F32, KvtcError, Plan, Batch, lib, lib_path,
    kvtc_plan_create, kvtc_plan_destroy, kvtc_record_bytes, kvtc_encoded_bytes,
    kvtc_encode, kvtc_decode, kvtc_batch_create, kvtc_batch_destroy, kvtc_offsets,
    kvtc_encode_batch, kvtc_decode_batch, kvtc_encode_batch_static, kvtc_last_error, JOB_DTYPE, make_jobs,
    kvtc_window_split, kvtc_cr_with_window, kvtc_fp8_pack, kvtc_fp8_unpack, kvtc_offsets_append,
    kvtc_probe_stream, kvtc_probe_mfma_bf16, PROBE_READ, PROBE_WRITE, PROBE_COPY,
    kvtc_rope, ROPE_HALF, ROPE_INTERLEAVED,
    WidePlan, kvtc_wide_create, kvtc_wide_destroy, kvtc_wide_sections, kvtc_wide_section_record_bytes, kvtc_wide_record_bytes,
    kvtc_wide_encoded_bytes, kvtc_wide_encode, kvtc_wide_decode,
    EntropyTables, kvtc_entropy_create, kvtc_entropy_destroy, kvtc_entropy_bound, kvtc_entropy_encode, kvtc_entropy_decode,
    kvtc_entropy_encode_batch, kvtc_entropy_decode_batch, make_entropy_jobs, ENTROPY_JOB_DTYPE,
    kvtc_calib_block_errors, kvtc_calib_moments,
    KvtcLayout, layout, kvtc_encode_blocked, kvtc_decode_blocked, kvtc_encode_batch_blocked, kvtc_decode_batch_blocked,
)
from . import bundles  # noqa: F401
