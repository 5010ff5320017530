// Cache commit and cache read-back kernels (gfx950), for bf16, fp32 and fp8 (E4M3) caches.
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

// Largest squared key norms: knorm[head][slot][part] = float bits of max_t |k[t,head,:]|^2 over
// the tokens of the block in `slot` that workgroup `part` of the head copied (non-negative floats
// order like their bit patterns).  Every commit rewrites all parts of its slot's entries with
// plain stores, so nothing is ever stale and no atomic is needed (device-wide atomics on a few
// words cost about 100 ns apiece, one after the other: a counter met by every workgroup was most
// of an earlier version's run time).  The attention kernel takes the maximum over the resident
// slots' entries of its head.
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

// ---- fp8 (OCP E4M3) cache variant: a block is rounded to E4M3 as it is committed (paper, KV
// Management section and Challenges section: a compressed / quantised KV store; the format and the
// rule are this library's: nearest code, ties to the even code, magnitudes beyond 448 and
// infinities to +-448, NaN stays NaN).  The hardware conversion rounds the same way but turns
// everything beyond 464 into NaN, so magnitudes are clamped to 448 first.
typedef __bf16 commit_bf16x2 __attribute__((ext_vector_type(2)));
typedef short commit_s16x2 __attribute__((ext_vector_type(2)));
typedef unsigned short commit_u16x2 __attribute__((ext_vector_type(2)));
typedef float commit_f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// two bf16 in a word: magnitudes in (448, inf] become 448, NaN and everything else stay
__device__ __forceinline__ uint32_t clamp448_bf16x2(uint32_t w)
{
    const commit_u16x2 mag = __builtin_bit_cast(commit_u16x2, w & 0x7fff7fffu);
    const commit_u16x2 lim = {0x43E0, 0x43E0}, inf = {0x7F80, 0x7F80}, one = {1, 1}, all = {0x7FFF, 0x7FFF};
    const commit_u16x2 clamped = __builtin_elementwise_min(mag, lim);
    const commit_u16x2 is_nan = __builtin_elementwise_min(__builtin_elementwise_sub_sat(mag, inf), one);  // 1 where NaN
    const commit_u16x2 nan_bits = is_nan * all;
    return (w & 0x80008000u) | __builtin_bit_cast(uint32_t, clamped) | __builtin_bit_cast(uint32_t, nan_bits);
}

// 8 bf16 (16 bytes) -> 8 E4M3 codes (8 bytes)
__device__ __forceinline__ u32x2 bf16x8_to_e4m3(const u32x4 &v)
{
    u32x2 r;
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        commit_s16x2 acc = {0, 0};
        acc = __builtin_amdgcn_cvt_scalef32_pk_fp8_bf16(acc, __builtin_bit_cast(commit_bf16x2, clamp448_bf16x2(v[2 * k])), 1.0f, false);
        acc = __builtin_amdgcn_cvt_scalef32_pk_fp8_bf16(acc, __builtin_bit_cast(commit_bf16x2, clamp448_bf16x2(v[2 * k + 1])), 1.0f, true);
        r[k] = __builtin_bit_cast(uint32_t, acc);
    }
    return r;
}

// sum of squares of the 8 values 8 E4M3 codes stand for
__device__ __forceinline__ float e4m3x8_sumsq(const u32x2 &c)
{
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const commit_f32x2 lo = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(c[k], 1.0f, false);
        const commit_f32x2 hi = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(c[k], 1.0f, true);
        s += lo[0] * lo[0] + lo[1] * lo[1] + hi[0] * hi[0] + hi[1] * hi[1];
    }
    return s;
}

// K with head_dim 128 (16 chunks of 16 bytes per source row, one row per 16-lane DPP row): copy
// src [n, H, 128] bf16 -> dst [H][dst_tokens][128] (bf16 rows, or FP8: rows of E4M3 codes) at token
// offset tok0 and record the largest squared key norm of the rows as stored in *knorm_entry.
// Runs as workgroup (head h, part p) of H * parts: the tokens [p * chunk, (p + 1) * chunk) of head
// h, chunk = ceil(n / parts); 16 tokens per round, one per 16-lane group, U rounds in flight.  The
// workgroup writes one contiguous piece of the head's region; the H workgroups of a part read
// neighbouring rows of the source at about the same time.
template <int U, bool FP8>
__device__ __forceinline__ void k_rows_norm_body(int h, int p, int parts, uint32_t *group_max, const u32x4 *__restrict__ src,
                                                 void *__restrict__ dst, int64_t n, int H, int64_t dst_tokens,
                                                 int64_t tok0, uint32_t *__restrict__ knorm_entry)
{
    const int c = threadIdx.x & 15;
    const int g = threadIdx.x >> 4;  // 16-lane group
    const int chunk = ((int)n + parts - 1) / parts;
    const int t_end = (p + 1) * chunk < (int)n ? (p + 1) * chunk : (int)n;
    int t = p * chunk + g;
    const u32x4 *srow = src + (int64_t)h * 16 + c;  // + t * H * 16
    u32x4 *drow = static_cast<u32x4 *>(dst) + ((int64_t)h * dst_tokens + tok0) * 16 + c;  // + t * 16
    u32x2 *drow8 = static_cast<u32x2 *>(dst) + ((int64_t)h * dst_tokens + tok0) * 16 + c;
    // The largest norm as an integer maximum over the bit patterns with the sign cleared: finite
    // norms order like their bits, +inf (an overflowed norm) lies above them and every NaN above
    // that, so a norm that is not finite sticks whatever the compiler assumes about NaNs.
    uint32_t best = 0u;
    auto put = [&](int tok, const u32x4 &v) {
        float ss;
        if constexpr (FP8) {
            const u32x2 codes = bf16x8_to_e4m3(v);
            drow8[(int64_t)tok * 16] = codes;
            ss = e4m3x8_sumsq(codes);
        } else {
            drow[(int64_t)tok * 16] = v;
            ss = bf16x2_sumsq(v[0]) + bf16x2_sumsq(v[1]) + bf16x2_sumsq(v[2]) + bf16x2_sumsq(v[3]);
        }
        const uint32_t tot = __builtin_bit_cast(uint32_t, row16_sum_to_lane15(ss)) & 0x7fffffffu;
        best = tot > best ? tot : best;
    };
    for (; t + (U - 1) * 16 < t_end; t += U * 16) {
        u32x4 v[U];
#pragma unroll
        for (int k = 0; k < U; ++k) v[k] = srow[(int64_t)(t + k * 16) * H * 16];
#pragma unroll
        for (int k = 0; k < U; ++k) put(t + k * 16, v[k]);
    }
    for (; t < t_end; t += 16) put(t, srow[(int64_t)t * H * 16]);
    if (c == 15) group_max[g] = best;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t m = 0u;
        for (int k = 0; k < 16; ++k) m = group_max[k] > m ? group_max[k] : m;
        *knorm_entry = m;  // every part of the slot's entries is rewritten by every commit
    }
}

// bf16 V with head_dim 128: src [n, H, 128] -> granules [H][v_tokens/8][128][8] at token offset
// tok0 (tok0 and n multiples of 8).  The unit of work of a wavefront is half a granule of one
// head: 8 tokens x 64 dimensions.  Its lanes read the 8 rows' 128-byte pieces with one 16-byte
// load each, put them into LDS row by row (rows 144 bytes apart, so the four rows a transposing
// read gathers lie in different banks), get them back with two transposing reads
// (ds_read_b64_tr_b16: lane l receives dimension l of 4 tokens) and write 16 bytes each, 1 KiB
// contiguous per wavefront.  U units are in flight per wavefront.  Runs as workgroup `bid` of
// `nblocks`, 4 wavefronts each; LDS: 4 * U * V_UNIT_LDS bytes.
constexpr int V_UNIT_LDS = 8 * 144;
typedef short commit_s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) commit_s16x4 *commit_lds_s16x4_ptr;
// FP8: the 16 bytes become 8 E4M3 codes, granules [H][v_tokens/8][128][8] of one byte each.
template <int U, bool FP8>
__device__ __forceinline__ void v_to_granules_body(int bid, int nblocks, unsigned char *lds, const u32x4 *__restrict__ src,
                                                   void *__restrict__ dst, int64_t n, int H, int64_t v_tokens, int64_t tok0)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int units = (int)(n >> 3) * H * 2;          // (granule, head, half), half fastest
    const int stride = nblocks * 4;                   // wavefronts of the launch's V part
    unsigned char *my = lds + wave * (U * V_UNIT_LDS);
    const int wr = (lane >> 3) * 144 + (lane & 7) * 16;  // row lane / 8, 16-byte chunk lane % 8
    const int rd = ((lane & 15) >> 2) * 144 + (lane >> 4) * 32 + (lane & 3) * 8;
    const int64_t gran_per_head = v_tokens >> 3, g0 = tok0 >> 3;
    for (int u0 = bid * 4 + wave; u0 < units; u0 += U * stride) {
        u32x4 v[U];
#pragma unroll
        for (int k = 0; k < U; ++k) {
            const int u = u0 + k * stride;
            if (u < units) {
                const int half = u & 1, h = (u >> 1) % H, g = (u >> 1) / H;
                v[k] = src[(((int64_t)g * 8 + (lane >> 3)) * H + h) * 16 + half * 8 + (lane & 7)];
            }
        }
#pragma unroll
        for (int k = 0; k < U; ++k) {
            const int u = u0 + k * stride;
            if (u < units) {
                const int half = u & 1, h = (u >> 1) % H, g = (u >> 1) / H;
                unsigned char *unit = my + k * V_UNIT_LDS;
                *reinterpret_cast<u32x4 *>(unit + wr) = v[k];
                typedef __attribute__((address_space(3))) unsigned char *lds_bytes;
                const commit_s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((commit_lds_s16x4_ptr)((lds_bytes)unit + rd));
                const commit_s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((commit_lds_s16x4_ptr)((lds_bytes)unit + rd + 4 * 144));
                typedef short s16x8 __attribute__((ext_vector_type(8)));
                const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                const int64_t at = ((int64_t)h * gran_per_head + g0 + g) * 128 + half * 64 + lane;
                if constexpr (FP8)
                    static_cast<u32x2 *>(dst)[at] = bf16x8_to_e4m3(__builtin_bit_cast(u32x4, both));
                else
                    static_cast<u32x4 *>(dst)[at] = __builtin_bit_cast(u32x4, both);
            }
        }
    }
}

// What one layer's share of a commit launch needs: the caller's block and where it goes.
struct commit_layer {
    const void *k_src, *v_src;  // [n, H, 128] bf16
    void *k_dst, *v_dst;        // the layer's K region and V region
    uint32_t *knorm;            // the layer's key-norm table [H][cap_blocks][parts]
    int64_t tok0;               // first token of the slot
    int slot;
};
constexpr int COMMIT_MAX_LAYERS = 64;  // 64 * 56 bytes of kernel arguments
struct commit_layers {
    commit_layer l[COMMIT_MAX_LAYERS];
};

// One launch for the bf16 blocks of up to COMMIT_MAX_LAYERS layers: grid (x, layers); of a layer's
// workgroups the first H * parts copy K (workgroup p * H + h: head h, part p) and take the key
// norms, the rest turn V into granules.
// FP8: the cache holds E4M3 codes (the source blocks are bf16 either way).
template <int U, bool FP8>
__global__ __launch_bounds__(256) void store_block_bf16_kernel(const commit_layers layers, int64_t n, int H, int64_t k_tokens,
                                                              int64_t v_tokens, int parts, int cap_blocks)
{
    __shared__ uint32_t group_max[16];  // float bits
    __shared__ __attribute__((aligned(16))) unsigned char v_lds[4 * U * V_UNIT_LDS];
    const commit_layer &L = layers.l[blockIdx.y];
    const int k_blocks = H * parts;
    if ((int)blockIdx.x < k_blocks) {
        const int h = (int)blockIdx.x % H, p = (int)blockIdx.x / H;
        k_rows_norm_body<U, FP8>(h, p, parts, group_max, (const u32x4 *)L.k_src, L.k_dst, n, H, k_tokens, L.tok0,
                                 L.knorm + ((int64_t)h * cap_blocks + L.slot) * parts + p);
    } else {
        v_to_granules_body<U, FP8>((int)blockIdx.x - k_blocks, (int)gridDim.x - k_blocks, v_lds, (const u32x4 *)L.v_src, L.v_dst, n, H,
                                   v_tokens, L.tok0);
    }
}

// Read-back of one block for inspection: the n tokens of physical slot `slot` of every head go to
// dst [n, H, row] (the caller's buffer at the block's place in the order it asked for).
__global__ __launch_bounds__(256) void heads_to_rows_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, int64_t n,
                                                           int H, int chunks_per_row, int64_t src_tokens, int64_t slot)
{
    const int64_t total = n * H * chunks_per_row;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < total; g += stride) {
        const int c = (int)(g % chunks_per_row);
        const int64_t th = g / chunks_per_row;
        const int h = (int)(th % H);
        const int64_t t = th / H;
        dst[g] = src[((int64_t)h * src_tokens + slot * n + t) * chunks_per_row + c];
    }
}

__global__ __launch_bounds__(256) void granules_to_rows_kernel(const uint16_t *__restrict__ src, u16x8 *__restrict__ dst, int64_t n,
                                                              int H, int D, int64_t v_tokens, int64_t slot)
{
    const int dchunks = D >> 3;
    const int64_t total = n * H * dchunks;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t gran_per_head = v_tokens >> 3;
    for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < total; g += stride) {
        const int c = (int)(g % dchunks);
        const int64_t th = g / dchunks;
        const int h = (int)(th % H);
        const int64_t t = th / H;
        const int64_t p = slot * n + t;
        const uint16_t *s = src + (((int64_t)h * gran_per_head + (p >> 3)) * D + (c << 3)) * 8 + (p & 7);
        u16x8 r;
#pragma unroll
        for (int i = 0; i < 8; ++i) r[i] = s[i * 8];
        dst[g] = r;
    }
}

// Read-back of one block of an fp8 cache, widened (exactly) to bf16: dst [n, H, 128].
// One thread per 8 dimensions of one (token, head).
__global__ __launch_bounds__(256) void e4m3_block_to_rows_kernel(const unsigned char *__restrict__ k_region,
                                                                const unsigned char *__restrict__ v_region, u32x4 *__restrict__ k_dst,
                                                                u32x4 *__restrict__ v_dst, int64_t n, int H, int64_t k_tokens,
                                                                int64_t v_tokens, int64_t slot)
{
    const int64_t total = n * H * 16;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    auto widen8 = [](const u32x2 &c) {
        u32x4 r;
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            r[2 * k] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((int)c[k], 1.0f, false));
            r[2 * k + 1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((int)c[k], 1.0f, true));
        }
        return r;
    };
    for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < total; g += stride) {
        const int c = (int)(g & 15);  // dimensions 8 c .. 8 c + 7
        const int64_t th = g >> 4;
        const int h = (int)(th % H);
        const int64_t t = th / H, p = slot * n + t;
        k_dst[g] = widen8(*reinterpret_cast<const u32x2 *>(k_region + ((int64_t)h * k_tokens + p) * 128 + c * 8));
        const unsigned char *vs = v_region + (((int64_t)h * (v_tokens >> 3) + (p >> 3)) * 128 + c * 8) * 8 + (p & 7);
        u32x2 codes = {0u, 0u};
#pragma unroll
        for (int i = 0; i < 8; ++i) codes[i >> 2] |= (uint32_t)vs[i * 8] << (8 * (i & 3));
        v_dst[g] = widen8(codes);
    }
}

}  // namespace ifx
