// Cache commit and cache read-back kernels (gfx950).
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

// Largest squared key norm per head, tagged with an epoch: entry = (epoch << 32) | float bits of
// max_j |k_j|^2 (non-negative floats order like their bit patterns).  A newer epoch always wins an
// atomic max, so an entry needs no clearing when its slot is rewritten.  The epoch lives on the
// device, tag[0], next to a count of finished workgroups, tag[1]: every store launch writes under
// epoch tag[0] + 1, and its last workgroup to finish publishes that value and clears the count.
// Launches on one layer are ordered by the caller's stream, so a launch sees a settled pair.
__device__ __forceinline__ float bf16x2_sumsq(uint32_t w)
{
    const float lo = __builtin_bit_cast(float, w << 16), hi = __builtin_bit_cast(float, w & 0xffff0000u);
    return lo * lo + hi * hi;
}

// Sum over the 16 lanes of a DPP row; the total lands in lane 15 of the row.
__device__ __forceinline__ float row16_sum_to_lane15(float x)
{
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x111, 0xf, 0xf, true));  // row_shr:1
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x112, 0xf, 0xf, true));  // row_shr:2
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x114, 0xf, 0xf, true));  // row_shr:4
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x118, 0xf, 0xf, true));  // row_shr:8
    return x;
}

// bf16 K with head_dim 128 (16 chunks of 16 bytes per row, one row per 16-lane DPP row): copy
// src [n, H, 128] -> dst [H][dst_tokens][128] at token offset tok0 and
// knorm[h] = max(knorm[h], epoch : max_t |k[t,h,:]|^2).
// Runs as workgroup `bid` of `nblocks`, nblocks a multiple of H: a workgroup serves one head
// (bid % H) and 16 tokens per round, one per 16-lane group, so it writes 4 KiB contiguous per
// round and ends with ONE global atomic (many workgroups updating the same few words serialise
// in the L2: with a workgroup meeting every head that tail was half the kernel's time).
__device__ __forceinline__ void k_rows_norm_body(int bid, int nblocks, uint32_t *group_max, const u32x4 *__restrict__ src,
                                                 u32x4 *__restrict__ dst, int64_t n, int H, int64_t dst_tokens,
                                                 int64_t tok0, unsigned long long *__restrict__ knorm, uint32_t *__restrict__ tag)
{
    const int c = threadIdx.x & 15;
    const int g = threadIdx.x >> 4;                 // 16-lane group
    const int h = bid % H;
    const int tok_stride = (nblocks / H) * 16;      // tokens advanced per round
    // (read first, used last: the load's latency hides behind the copy)
    const uint32_t epoch = threadIdx.x == 0 ? __hip_atomic_load(&tag[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1u : 0u;
    int tok = (bid / H) * 16 + g;
    const int ntok = (int)n;
    const u32x4 *srow = src + (int64_t)h * 16 + c;  // + tok * H * 16
    u32x4 *drow = dst + ((int64_t)h * dst_tokens + tok0) * 16 + c;
    // The largest norm as an integer maximum over the bit patterns with the sign cleared: finite
    // norms order like their bits, +inf (an overflowed norm) lies above them and every NaN above
    // that, so a norm that is not finite sticks whatever the compiler assumes about NaNs.
    uint32_t best = 0u;
    auto take = [&](const u32x4 &v) {
        const float ss = bf16x2_sumsq(v[0]) + bf16x2_sumsq(v[1]) + bf16x2_sumsq(v[2]) + bf16x2_sumsq(v[3]);
        const uint32_t tot = __builtin_bit_cast(uint32_t, row16_sum_to_lane15(ss)) & 0x7fffffffu;
        best = tot > best ? tot : best;
    };
    // four rows in flight per 16-lane group
    for (; tok + 3 * tok_stride < ntok; tok += 4 * tok_stride) {
        u32x4 v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] = srow[(int64_t)(tok + k * tok_stride) * H * 16];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            drow[(int64_t)(tok + k * tok_stride) * 16] = v[k];
            take(v[k]);
        }
    }
    for (; tok < ntok; tok += tok_stride) {
        const u32x4 v = srow[(int64_t)tok * H * 16];
        drow[(int64_t)tok * 16] = v;
        take(v);
    }
    if (c == 15) group_max[g] = best;
    __syncthreads();
    if (threadIdx.x == 0) {
        // every workgroup has read the epoch before it counts itself done, so the last one may
        // advance it (the count is asked for first: its round trip overlaps the rest)
        uint32_t epoch_read = epoch;
        asm volatile("" : "+v"(epoch_read));  // the epoch has arrived in its register before the count goes out
        const uint32_t done_before = atomicAdd(&tag[1], 1u);
        uint32_t m = 0u;
        for (int k = 0; k < 16; ++k) m = group_max[k] > m ? group_max[k] : m;
        const unsigned long long mine = ((unsigned long long)epoch_read << 32) | m;
        if (m != 0u && mine > knorm[h]) atomicMax(&knorm[h], mine);  // the plain read only skips work
        if (done_before == (uint32_t)nblocks - 1u) {
            atomicExch(&tag[1], 0u);
            atomicExch(&tag[0], epoch_read);
        }
    }
}

// bf16 V: src [n, H, D] -> granules [H][v_tokens/8][D][8] at token offset tok0
// (tok0 and n multiples of 8).  A thread takes 8 tokens x 8 dimensions:
// eight coalesced 16-byte reads, an 8x8 transpose of 16-bit values in
// registers, eight 16-byte writes covering 128 contiguous bytes.
// Runs as workgroup `bid` of `nblocks`.
__device__ __forceinline__ void v_to_granules_body(int bid, int nblocks, const u16x8 *__restrict__ src,
                                                   u16x8 *__restrict__ dst, int64_t n, int H, int D, int64_t v_tokens,
                                                   int64_t tok0)
{
    const int dchunks = D >> 3;
    const int64_t total = (n >> 3) * H * dchunks;
    const int64_t stride = (int64_t)nblocks * blockDim.x;
    const int64_t gran_per_head = v_tokens >> 3;
    const int64_t g0 = tok0 >> 3;
    for (int64_t w = (int64_t)bid * blockDim.x + threadIdx.x; w < total; w += stride) {
        const int c = (int)(w % dchunks);
        const int64_t gh = w / dchunks;
        const int h = (int)(gh % H);
        const int64_t g = gh / H;
        u16x8 *o = dst + (((int64_t)h * gran_per_head + g0 + g) * D + (c << 3));
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

// What one layer's share of a commit launch needs: the caller's block and where it goes.
struct commit_layer {
    const void *k_src, *v_src;  // [n, H, 128] bf16
    void *k_dst, *v_dst;        // the layer's K region and V region
    unsigned long long *knorm;  // the slot's key-norm row [H]
    uint32_t *tag;              // the layer's {epoch, finished workgroups}
    int64_t tok0;               // first token of the slot
};
constexpr int COMMIT_MAX_LAYERS = 64;  // 64 * 56 bytes of kernel arguments
struct commit_layers {
    commit_layer l[COMMIT_MAX_LAYERS];
};

// One launch for the bf16 blocks of up to COMMIT_MAX_LAYERS layers: grid (x, layers); of a layer's
// workgroups the first k_blocks copy K and take the key norms, the rest turn V into granules.
// k_blocks must be a multiple of H.
__global__ __launch_bounds__(256) void store_block_bf16_kernel(const commit_layers layers, int64_t n, int H, int64_t k_tokens,
                                                              int64_t v_tokens, int k_blocks)
{
    __shared__ uint32_t group_max[16];  // float bits
    const commit_layer &L = layers.l[blockIdx.y];
    if ((int)blockIdx.x < k_blocks)
        k_rows_norm_body((int)blockIdx.x, k_blocks, group_max, (const u32x4 *)L.k_src, (u32x4 *)L.k_dst, n, H, k_tokens, L.tok0,
                         L.knorm, L.tag);
    else
        v_to_granules_body((int)blockIdx.x - k_blocks, (int)gridDim.x - k_blocks, (const u16x8 *)L.v_src, (u16x8 *)L.v_dst, n, H,
                           128, v_tokens, L.tok0);
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
