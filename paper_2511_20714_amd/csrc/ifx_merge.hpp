// Merge of two partial attention results over disjoint key sets (paper, Parallelism section:
// ring attention circulates queries or keys/values between devices and combines the partial
// results; KV Management section: chunked access to the cache).  With L_x = ln sum_j exp(s_ij)
// over key set x and out_x the attention output normalised over x,
//   out = (e^{L_a} out_a + e^{L_b} out_b) / (e^{L_a} + e^{L_b}),   L = ln(e^{L_a} + e^{L_b}).
#pragma once
#include "ifx_types.hpp"

namespace ifx {

// One thread per (row, 8 elements); rows = tokens * heads, D % 8 == 0.  T is float or __bf16.
// out may alias out_a or out_b, lse may alias lse_a or lse_b (each thread reads before it writes;
// the D/8 threads of a row all read lse_a/lse_b and only the first writes lse, after a wave-wide
// read: rows never straddle a wave because 64 % (D/8) == 0 is required by the launcher).
template <typename T>
__global__ __launch_bounds__(256) void merge_kernel(const T *__restrict__ out_a, const float *__restrict__ lse_a,
                                                   const T *__restrict__ out_b, const float *__restrict__ lse_b,
                                                   T *out, float *lse, int64_t rows, int D)
{
    const int chunks = D >> 3;
    const int64_t total = rows * chunks;
    const int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= total) return;
    const int64_t row = g / chunks;
    const int c = (int)(g - row * chunks);
    const float la = lse_a[row], lb = lse_b[row];
    const float mx = fmaxf(la, lb);
    // weights relative to the larger one: no overflow; an empty side (-inf) gets weight 0
    const float wa = mx == -INFINITY ? 0.5f : expf(la - mx), wb = mx == -INFINITY ? 0.5f : expf(lb - mx);
    const float inv = 1.0f / (wa + wb);
    const T *pa = out_a + row * D + c * 8, *pb = out_b + row * D + c * 8;
    float r[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) r[e] = (wa * (float)pa[e] + wb * (float)pb[e]) * inv;
    T *po = out + row * D + c * 8;
#pragma unroll
    for (int e = 0; e < 8; ++e) po[e] = (T)r[e];
    if (lse != nullptr && c == 0) lse[row] = mx + logf(wa + wb);
}

}  // namespace ifx
