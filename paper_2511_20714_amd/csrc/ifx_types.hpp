// Vector types shared by the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint16_t u16x8 __attribute__((ext_vector_type(8)));

// Private cache layout (per layer).
//   K  : [heads][k_tokens][head_dim]                 one key = one contiguous row
//   V  : fp32: same as K.
//        bf16: [heads][v_tokens / 8][head_dim][8]    "granules" of 8 consecutive tokens,
//              stored dimension-major so that 8 keys of one dimension are 16 contiguous
//              bytes: exactly one lane's share of the A operand of the P*V MFMA.
// Token t of physical slot s sits at token index s * block_tokens + t.
struct ifx_layer_view {
    void *k;           // K region of the layer
    void *v;           // V region of the layer
    int64_t k_tokens;  // tokens allocated per head in K
    int64_t v_tokens;  // tokens allocated per head in V (bf16: multiple of 64, includes staging room)
};

// A key range cut into up to four runs of physical tokens: key j (0 <= j < total) is physical
// token j + delta[k] of a head's region, k = number of end[] entries <= j.  Unused end[] entries
// hold INT_MAX.
struct ifx_key_runs {
    int end[3];
    int delta[4];
};
