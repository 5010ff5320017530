// fp32 block attention (gfx950): fp32 loads, fp32 FMA, accurate expf, online
// softmax per query row.  A small, simple kernel for the fp32 cache dtype; the
// bf16 MFMA kernel is the fast path.
//
// Operation (paper, Introduction, framework paragraph + abstract): every query
// of the block attends to all resident cached tokens and all tokens of its own
// block; softmax over that whole key set; no other mask.
#pragma once
#include "ifx_types.hpp"

namespace ifx {

constexpr int F32_BM = 32;   // query rows per workgroup
constexpr int F32_BN = 64;   // keys per tile
constexpr int F32_MAXD = 128;

// LDS rows are padded by 4 floats: 16-byte alignment for the vector reads, and consecutive rows
// start 4 banks apart, so the 8 key rows a wavefront reads at once do not collide.
inline size_t attn_f32_lds_bytes(int D)
{
    return sizeof(float) * ((size_t)F32_BM * (D + 4) + (size_t)F32_BN * (D + 4) + (size_t)F32_BN * D +
                            (size_t)F32_BM * (F32_BN + 4));
}

// grid (ceil(n / 32), H), 256 threads.  Thread t serves query row t/8; the 8 threads of a row
// split the tile's keys (scores: keys sub, sub+8, ...) and the head dimensions (PV: 4-float chunks
// sub, sub+8, ...).  All LDS traffic is 16-byte reads: per 4 head dimensions one Q read (the same
// address for the 8 threads of a row) and 8 K reads feed 32 FMAs; per 4 keys one P read and up to
// 4 V reads feed 16 FMAs per chunk.  D % 4 == 0, D <= 128.
__global__ __launch_bounds__(256) void attn_f32_kernel(const float *__restrict__ q,
                                                      const float *__restrict__ kc,
                                                      const float *__restrict__ vc,
                                                      const float *__restrict__ kb,
                                                      const float *__restrict__ vb, float *__restrict__ out,
                                                      float *__restrict__ lse, int n, int C, int n_blk, int H, int D,
                                                      int64_t cache_tokens, float scale, const ifx_key_blocks blocks)
{
    // Keys: C cached tokens (logical order of the caller's selection, whole blocks of n tokens, mapped to physical
    // tokens by `blocks`), then the n_blk tokens of the current block (n_blk is n or 0).
    extern __shared__ __attribute__((aligned(16))) float smem[];
    const int ldq = D + 4;
    float *Qs = smem;                        // [32][D+4]
    float *Ks = Qs + F32_BM * ldq;           // [64][D+4]
    float *Vs = Ks + F32_BN * ldq;           // [64][D]
    float *Ps = Vs + F32_BN * D;             // [32][68]
    const int ldp = F32_BN + 4;

    const int tid = threadIdx.x;
    const int h = blockIdx.y;
    const int row0 = blockIdx.x * F32_BM;
    const int r = tid >> 3;    // row within tile
    const int sub = tid & 7;   // position among the row's 8 threads
    const int Lk = C + n_blk;
    const int d4n = D >> 2;    // 4-float chunks per row

    for (int e = tid; e < F32_BM * d4n; e += 256) {
        const int rr = e / d4n, c = e - rr * d4n;
        const int i = row0 + rr;
        f32x4 v = {0.f, 0.f, 0.f, 0.f};
        if (i < n) v = *reinterpret_cast<const f32x4 *>(q + ((int64_t)i * H + h) * D + 4 * c);
        *reinterpret_cast<f32x4 *>(Qs + rr * ldq + 4 * c) = v;
    }

    constexpr int MAXC = F32_MAXD / 32;  // 4-float output chunks per thread
    f32x4 acc[MAXC];
#pragma unroll
    for (int w = 0; w < MAXC; ++w) acc[w] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m = -INFINITY, l = 0.0f;

    for (int j0 = 0; j0 < Lk; j0 += F32_BN) {
        __syncthreads();  // previous tile fully consumed (also orders the Q fill)
        for (int e = tid; e < F32_BN * d4n; e += 256) {
            const int jj = e / d4n, c = e - jj * d4n;
            const int j = j0 + jj;
            f32x4 kv = {0.f, 0.f, 0.f, 0.f}, vv = {0.f, 0.f, 0.f, 0.f};
            if (j < C) {
                const int jp = blocks.magic ? blocks.first_token(j / n) + j % n : j;  // key j of the selection is physical token jp
                const int64_t off = ((int64_t)h * cache_tokens + jp) * D + 4 * c;
                kv = *reinterpret_cast<const f32x4 *>(kc + off);
                vv = *reinterpret_cast<const f32x4 *>(vc + off);
            } else if (j < Lk) {
                const int64_t off = ((int64_t)(j - C) * H + h) * D + 4 * c;
                kv = *reinterpret_cast<const f32x4 *>(kb + off);
                vv = *reinterpret_cast<const f32x4 *>(vb + off);
            }
            *reinterpret_cast<f32x4 *>(Ks + jj * ldq + 4 * c) = kv;
            *reinterpret_cast<f32x4 *>(Vs + jj * D + 4 * c) = vv;
        }
        __syncthreads();

        // scores of row r against keys sub, sub+8, ...
        float s[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) s[u] = 0.0f;
        for (int c = 0; c < d4n; ++c) {
            const f32x4 qv = *reinterpret_cast<const f32x4 *>(Qs + r * ldq + 4 * c);
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const f32x4 kv = *reinterpret_cast<const f32x4 *>(Ks + (sub + 8 * u) * ldq + 4 * c);
                s[u] = fmaf(qv[0], kv[0], s[u]);
                s[u] = fmaf(qv[1], kv[1], s[u]);
                s[u] = fmaf(qv[2], kv[2], s[u]);
                s[u] = fmaf(qv[3], kv[3], s[u]);
            }
        }
        float tmax = -INFINITY;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            s[u] = (j0 + sub + 8 * u < Lk) ? s[u] * scale : -INFINITY;
            tmax = fmaxf(tmax, s[u]);
        }
        tmax = fmaxf(tmax, __shfl_xor(tmax, 1));
        tmax = fmaxf(tmax, __shfl_xor(tmax, 2));
        tmax = fmaxf(tmax, __shfl_xor(tmax, 4));
        const float m_new = fmaxf(m, tmax);  // finite: each tile holds at least one valid key
        const float alpha = expf(m - m_new);  // 0 on the first tile
        float psum = 0.0f;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const float p = expf(s[u] - m_new);
            psum += p;
            Ps[r * ldp + sub + 8 * u] = p;
        }
        psum += __shfl_xor(psum, 1);
        psum += __shfl_xor(psum, 2);
        psum += __shfl_xor(psum, 4);
        l = l * alpha + psum;
        m = m_new;
        __syncthreads();

        // out[r][4 (sub + 8w) .. + 3] += sum_j P[r][j] * V[j][same]
#pragma unroll
        for (int w = 0; w < MAXC; ++w) acc[w] *= alpha;
        for (int j4 = 0; j4 < F32_BN; j4 += 4) {
            const f32x4 p = *reinterpret_cast<const f32x4 *>(Ps + r * ldp + j4);
#pragma unroll
            for (int w = 0; w < MAXC; ++w) {
                const int c = sub + 8 * w;
                if (c < d4n) {
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        const f32x4 v = *reinterpret_cast<const f32x4 *>(Vs + (j4 + t) * D + 4 * c);
                        acc[w] += p[t] * v;
                    }
                }
            }
        }
    }

    const int i = row0 + r;
    if (i < n) {
        if (lse != nullptr && sub == 0) lse[(int64_t)i * H + h] = m + logf(l);
        const float inv = 1.0f / l;
#pragma unroll
        for (int w = 0; w < MAXC; ++w) {
            const int c = sub + 8 * w;
            if (c < d4n) *reinterpret_cast<f32x4 *>(out + ((int64_t)i * H + h) * D + 4 * c) = acc[w] * inv;
        }
    }
}

}  // namespace ifx
