// bf16 MFMA operand helpers shared by the dense-tile kernels for batches of small graphs.
#pragma once
#include "layer_device.hpp"

namespace dfgnn {

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

// two floats -> packed bf16 pair, round to nearest even (v_cvt_pk_bf16_f32)
__device__ inline uint32_t cvt_pk_bf16(float lo, float hi) {
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
__device__ inline uint16_t to_bf16(float f) { return (uint16_t)(cvt_pk_bf16(f, 0.f) & 0xffffu); }
// A tile of fp32 weights (attention weights or their gradients) as MFMA A operand.  The weights are
// split into a bf16 head and a bf16 remainder and multiplied in two MFMAs, so the second products keep
// ~16 bits of the weights instead of 8 (MFMA time is negligible here; the inputs K, V, Q, dO are exact).
struct SplitFrag {
    s16x4 hi, lo;
};
__device__ inline SplitFrag split_bf16x4(float a, float b, float c, float d) {
    const uint32_t h01 = cvt_pk_bf16(a, b), h23 = cvt_pk_bf16(c, d);
    const float ha = __builtin_bit_cast(float, h01 << 16), hb = __builtin_bit_cast(float, h01 & 0xffff0000u);
    const float hc = __builtin_bit_cast(float, h23 << 16), hd = __builtin_bit_cast(float, h23 & 0xffff0000u);
    const uint32_t l01 = cvt_pk_bf16(a - ha, b - hb), l23 = cvt_pk_bf16(c - hc, d - hd);
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    SplitFrag f;
    f.hi = __builtin_bit_cast(s16x4, u32x2{h01, h23});
    f.lo = __builtin_bit_cast(s16x4, u32x2{l01, l23});
    return f;
}
__device__ inline f32x4 mfma_split(const SplitFrag& a, s16x4 b, f32x4 acc) {
    acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a.hi, b, acc, 0, 0, 0);
    return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a.lo, b, acc, 0, 0, 0);
}

}  // namespace dfgnn
