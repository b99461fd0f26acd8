// fp32 operands on the bf16 matrix cores: the hi / lo split and the LDS layout of bf16 operand
// tiles that the dense GEMM kernels and the heavy-row product share.
#pragma once

#include <stdint.h>
#include <hip/hip_runtime.h>

namespace mst {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// An LDS row is 64 k of bf16 = 128 bytes = eight 16-byte units; unit u of row m is kept at
// position u ^ ((m >> 1) & 7): the MFMA operand reads of 16 consecutive rows then cover all
// banks once.
__device__ inline uint32_t bf_unit(int m, int u) { return (uint32_t)(m * 128 + ((u ^ ((m >> 1) & 7)) << 4)); }

__device__ inline uint32_t cvt_pk_bf16(float a, float b) {       // {bf16(a), bf16(b)}, round to nearest even
    uint32_t r;
    asm("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
// x = hi + lo + (at most 2^-16 |x|): hi = bf16(x), lo = bf16(x - hi); x - hi is exact in fp32
__device__ inline void split_pair(float x0, float x1, uint32_t& hi, uint32_t& lo) {
    hi = cvt_pk_bf16(x0, x1);
    lo = cvt_pk_bf16(x0 - __uint_as_float(hi << 16), x1 - __uint_as_float(hi & 0xFFFF0000u));
}

}  // namespace mst
