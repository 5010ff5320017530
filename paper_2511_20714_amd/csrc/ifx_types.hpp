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
//        fp8 (E4M3 codes): both layouts with one byte per element.
// Token t of physical slot s sits at token index s * block_tokens + t.

// A selection of cached blocks as a key set: `count` whole blocks of block_tokens tokens each, entry
// e starting at physical token first_token(e) of a head's region.  Up to IFX_MAX_KEY_BLOCKS
// entries travel in the kernel arguments (`first`); a longer list lies in device memory (`list`,
// count entries) and the bf16 kernel then works through it IFX_MAX_KEY_BLOCKS entries at a time.
// magic = floor(2^32 / block_tokens) + 1, so that the high word of j * magic is j / block_tokens
// (the host checks this for every j the kernel can form).  The bf16 kernel keeps the entries it is
// working on in one register, a lane per entry, with one lane left for "past the end".
constexpr int IFX_MAX_KEY_BLOCKS = 63;
struct ifx_key_blocks {
    int first[IFX_MAX_KEY_BLOCKS + 1];
    const int *list;  // nullptr: the entries are in `first`
    int count;
    unsigned magic;   // 0: no selection, the cached keys are the region's tokens [0, C)
    __host__ __device__ int first_token(int e) const { return list ? list[e] : first[e]; }
};
