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
    float best = 0.f;
    auto take = [&](const u32x4 &v) {
        const float ss = bf16x2_sumsq(v[0]) + bf16x2_sumsq(v[1]) + bf16x2_sumsq(v[2]) + bf16x2_sumsq(v[3]);
        const float tot = row16_sum_to_lane15(ss);
        best = tot > best || tot != tot ? tot : best;  // a NaN sticks
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
    if (c == 15) group_max[g] = __builtin_bit_cast(uint32_t, best);  // NaN bits order above all finite
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
// (tok0, n and pad_tokens multiples of 8); the pad_tokens tokens behind the block are
// zero-filled (attention pads its last key tile with them).  A thread takes 8 tokens x 8 dimensions:
// eight coalesced 16-byte reads, an 8x8 transpose of 16-bit values in
// registers, eight 16-byte writes covering 128 contiguous bytes.
// Runs as workgroup `bid` of `nblocks`.
__device__ __forceinline__ void v_to_granules_body(int bid, int nblocks, const u16x8 *__restrict__ src,
                                                   u16x8 *__restrict__ dst, int64_t n, int H, int D, int64_t v_tokens,
                                                   int64_t tok0, int64_t pad_tokens)
{
    const int dchunks = D >> 3;
    const int64_t real = (n >> 3) * H * dchunks;
    const int64_t total = ((n + pad_tokens) >> 3) * H * dchunks;
    const int64_t stride = (int64_t)nblocks * blockDim.x;
    const int64_t gran_per_head = v_tokens >> 3;
    const int64_t g0 = tok0 >> 3;
    for (int64_t w = (int64_t)bid * blockDim.x + threadIdx.x; w < total; w += stride) {
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

// One launch for a bf16 block: workgroups [0, k_blocks) copy K and take the key norms, the rest
// turn V into granules.  Used by the commit and by the staging in front of every attention call.
// k_blocks must be a multiple of H.
__global__ __launch_bounds__(256) void store_block_bf16_kernel(const u32x4 *__restrict__ k_src, u32x4 *__restrict__ k_dst,
                                                              const u16x8 *__restrict__ v_src, u16x8 *__restrict__ v_dst,
                                                              int64_t n, int H, int64_t k_tokens, int64_t v_tokens,
                                                              int64_t tok0, int64_t pad_tokens,
                                                              unsigned long long *__restrict__ knorm,
                                                              uint32_t *__restrict__ tag, int k_blocks)
{
    __shared__ uint32_t group_max[16];  // float bits
    if ((int)blockIdx.x < k_blocks)
        k_rows_norm_body((int)blockIdx.x, k_blocks, group_max, k_src, k_dst, n, H, k_tokens, tok0, knorm, tag);
    else
        v_to_granules_body((int)blockIdx.x - k_blocks, (int)gridDim.x - k_blocks, v_src, v_dst, n, H, 128, v_tokens, tok0,
                           pad_tokens);
}

// bf16: move a block inside the cache's own layouts from token offset src_tok to dst_tok of every
// head (K rows and V granules are contiguous per head there), and copy its key norms from knorm
// row src to row dst under a new epoch.  Used to commit the block that the last attention call
// staged behind the resident tokens without reading the caller's tensors again.
// chunks_per_head = n * 256 / 16 (K) = n / 8 * 2048 / 16 (V).
__global__ __launch_bounds__(256) void move_block_bf16_kernel(u32x4 *__restrict__ k_region, u32x4 *__restrict__ v_region,
                                                             int64_t n, int H, int64_t k_tokens, int64_t v_tokens,
                                                             int64_t src_tok, int64_t dst_tok,
                                                             const unsigned long long *__restrict__ knorm_src,
                                                             unsigned long long *__restrict__ knorm_dst, uint32_t *__restrict__ tag)
{
    const int64_t per_head = n * 16;  // 16-byte chunks of one head's K rows (and of its V granules)
    const int64_t total = 2 * per_head * H;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < total; g += stride) {
        const int64_t which = g / (per_head * H);  // 0: K, 1: V
        const int64_t r = g - which * per_head * H;
        const int64_t h = r / per_head, c = r - h * per_head;
        u32x4 *base = which ? v_region : k_region;
        const int64_t tokens = which ? v_tokens : k_tokens;
        base[(h * tokens + dst_tok) * 16 + c] = base[(h * tokens + src_tok) * 16 + c];
    }
    if (blockIdx.x == 0) {  // the one workgroup that touches the epoch
        const uint32_t epoch = __hip_atomic_load(&tag[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1u;
        for (int h = threadIdx.x; h < H; h += blockDim.x)
            knorm_dst[h] = ((unsigned long long)epoch << 32) | (knorm_src[h] & 0xffffffffull);
        __syncthreads();
        if (threadIdx.x == 0) atomicExch(&tag[0], epoch);
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
