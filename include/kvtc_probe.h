/*
 * kvtc_probe.h -- what this GPU achieves on the two resources the coder is bound by, measured by
 * plain hand-written kernels of the same library, for quoting beside the published peaks:
 * a streaming read, a streaming write and a copy of a device buffer (the memory side; the coder's
 * encode is almost all reads, its decode almost all writes), and a loop of independent bf16
 * 32x32x16 matrix-core operations with no memory traffic (the compute side, which binds the
 * full-rank projection of the paper's eq. 3).  Not part of the coder's path.
 *
 * Same conventions as kvtc.h: *_dev are device pointers, `stream` is a hipStream_t; calls are
 * ordered on the stream, allocate nothing and do not synchronise; the caller times them.
 */
#ifndef KVTC_PROBE_H
#define KVTC_PROBE_H

#include "kvtc.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { KVTC_PROBE_READ = 0, KVTC_PROBE_WRITE = 1, KVTC_PROBE_COPY = 2 } kvtc_probe_mode;

/* Streams `bytes` (a multiple of 16; both pointers 16-byte aligned) once: READ reads src_dev and
 * writes nothing (dst_dev receives one dword only if the data xor to a value they never have),
 * WRITE fills dst_dev with a constant, COPY does dst_dev[i] = src_dev[i].  KVTC_E_ARG on null or
 * misaligned arguments. */
kvtc_status kvtc_probe_stream(kvtc_probe_mode mode, const void* src_dev, void* dst_dev, size_t bytes,
                              kvtc_stream stream);

/* Every wavefront of a grid that fills the device runs `iters` rounds of eight independent
 * v_mfma_f32_32x32x16_bf16 on register operands.  random_operands = 0: the operands take eight small
 * values; 1: pseudo-random bf16 values of both signs, different from one instruction to the next, as
 * the coder's operands are -- the rate the matrix cores sustain depends on it (the chip lowers its
 * clock under the higher switching activity), so both are reported.  *flops_host receives the
 * floating-point operations of the launch (2 * 32 * 32 * 16 per instruction).  sink_dev (>= 4 bytes)
 * is written only if a result is NaN.  KVTC_E_ARG on iters < 1, a flag outside 0..1 or a null pointer. */
kvtc_status kvtc_probe_mfma_bf16(int iters, int random_operands, void* sink_dev, double* flops_host, kvtc_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* KVTC_PROBE_H */
