// Cache commit, V staging and cache read-back kernels (gfx950).
// Commit moves a block's K/V from the caller's [tokens, heads, head_dim]
// tensors into the private per-head layout (paper, Introduction, framework
// paragraph: the finished block's KV updates the cache).  Pure data movement:
// every element is copied bit for bit, 16 bytes per lane per access.
#pragma once
#include "ifx_types.hpp"

namespace ifx {

// Row copy: src [n, H, row_bytes] -> dst [H][dst_tokens][row_bytes] at token offset tok0.
// One 16-byte chunk per thread-iteration; consecutive threads read consecutive
// source chunks and write whole rows.
__global__ __launch_bounds__(256) void rows_to_heads_kernel(const u32x4 *__restrict__ src,
                                                           u32x4 *__restrict__ dst, int64_t n, int H,
                                                           int chunks_per_row, int64_t dst_tokens,
                                                           int64_t tok0)
{
    const int64_t total = n * H * chunks_per_row;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < total; g += stride) {
        const int c = (int)(g % chunks_per_row);
        const int64_t th = g / chunks_per_row;
        const int h = (int)(th % H);
        const int64_t t = th / H;
        dst[((int64_t)h * dst_tokens + tok0 + t) * chunks_per_row + c] = src[g];
    }
}

// bf16 V: src [n, H, D] -> granules [H][v_tokens/8][D][8] at token offset tok0
// (tok0, n and pad_tokens multiples of 8); the pad_tokens tokens behind the block are
// zero-filled (attention pads its last key tile with them).  A thread takes 8 tokens x 8 dimensions:
// eight coalesced 16-byte reads, an 8x8 transpose of 16-bit values in
// registers, eight 16-byte writes covering 128 contiguous bytes.
__global__ __launch_bounds__(256) void v_to_granules_kernel(const u16x8 *__restrict__ src,
                                                           u16x8 *__restrict__ dst, int64_t n, int H, int D,
                                                           int64_t v_tokens, int64_t tok0, int64_t pad_tokens)
{
    const int dchunks = D >> 3;
    const int64_t real = (n >> 3) * H * dchunks;
    const int64_t total = ((n + pad_tokens) >> 3) * H * dchunks;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t gran_per_head = v_tokens >> 3;
    const int64_t g0 = tok0 >> 3;
    for (int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; w < total; w += stride) {
        const int c = (int)(w % dchunks);
        const int64_t gh = w / dchunks;
        const int h = (int)(gh % H);
        const int64_t g = gh / H;
        u16x8 *o = dst + (((int64_t)h * gran_per_head + g0 + g) * D + (c << 3));
        if (w >= real) {  // zero fill behind the block (granule order is token-major, so these are the last items)
            const u16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int i = 0; i < 8; ++i) o[i] = z;
            continue;
        }
        u16x8 in[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) in[e] = src[(((g << 3) + e) * H + h) * dchunks + c];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            u16x8 r;
#pragma unroll
            for (int e = 0; e < 8; ++e) r[e] = in[e][i];
            o[i] = r;
        }
    }
}

// Read-back of resident tokens into [C, H, row] order for inspection.
// logical != 0: oldest block first (slot = (oldest + b) mod cap_blocks), else slot order.
__global__ __launch_bounds__(256) void heads_to_rows_kernel(const u32x4 *__restrict__ src,
                                                           u32x4 *__restrict__ dst, int64_t C, int64_t n,
                                                           int H, int chunks_per_row, int64_t src_tokens,
                                                           int64_t oldest, int64_t cap_blocks, int logical)
{
    const int64_t total = C * H * chunks_per_row;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < total; g += stride) {
        const int c = (int)(g % chunks_per_row);
        const int64_t th = g / chunks_per_row;
        const int h = (int)(th % H);
        const int64_t l = th / H;
        const int64_t b = l / n, t = l % n;
        const int64_t slot = logical ? (oldest + b) % cap_blocks : b;
        dst[g] = src[((int64_t)h * src_tokens + slot * n + t) * chunks_per_row + c];
    }
}

__global__ __launch_bounds__(256) void granules_to_rows_kernel(const uint16_t *__restrict__ src,
                                                              u16x8 *__restrict__ dst, int64_t C, int64_t n,
                                                              int H, int D, int64_t v_tokens, int64_t oldest,
                                                              int64_t cap_blocks, int logical)
{
    const int dchunks = D >> 3;
    const int64_t total = C * H * dchunks;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t gran_per_head = v_tokens >> 3;
    for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < total; g += stride) {
        const int c = (int)(g % dchunks);
        const int64_t th = g / dchunks;
        const int h = (int)(th % H);
        const int64_t l = th / H;
        const int64_t b = l / n, t = l % n;
        const int64_t slot = logical ? (oldest + b) % cap_blocks : b;
        const int64_t p = slot * n + t;
        const uint16_t *s = src + (((int64_t)h * gran_per_head + (p >> 3)) * D + (c << 3)) * 8 + (p & 7);
        u16x8 r;
#pragma unroll
        for (int i = 0; i < 8; ++i) r[i] = s[i * 8];
        dst[g] = r;
    }
}

}  // namespace ifx
