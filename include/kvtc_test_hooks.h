/*
 * kvtc_test_hooks.h -- internal: host-only exports of the library that let CPU tests run the
 * kernels' scalar quantiser numerics without a GPU.  They are compiled from the very functions
 * the kernels call (csrc/kvtc_numeric.h: the directed fp32 -> fp16 roundings of the shared shift
 * (down) and scale (up), paper Section "Quantization", the group header, and the code decision
 * for one value).  Not part of the coder's API; applications include kvtc.h only.
 */
#ifndef KVTC_TEST_HOOKS_H
#define KVTC_TEST_HOOKS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

uint16_t kvtc_host_f16_round_down(float x);
uint16_t kvtc_host_f16_round_up(float x);
void kvtc_host_group_header(float lo, float hi, int bits, uint16_t* shift16, uint16_t* scale16);
uint32_t kvtc_host_code(float d, uint16_t shift16, uint16_t scale16, int bits);

#ifdef __cplusplus
}
#endif
#endif /* KVTC_TEST_HOOKS_H */
