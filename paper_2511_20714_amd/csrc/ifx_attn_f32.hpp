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

inline size_t attn_f32_lds_bytes(int D)
{
    return sizeof(float) * ((size_t)F32_BM * (D + 1) + (size_t)F32_BN * (D + 1) + (size_t)F32_BN * D +
                            (size_t)F32_BM * (F32_BN + 1));
}

// grid (ceil(n / 32), H), 256 threads.  Thread t serves query row t/8; the 8
// threads of a row split the tile's keys (scores) and the head dimensions (PV).
__global__ __launch_bounds__(256) void attn_f32_kernel(const float *__restrict__ q,
                                                      const float *__restrict__ kc,
                                                      const float *__restrict__ vc,
                                                      const float *__restrict__ kb,
                                                      const float *__restrict__ vb, float *__restrict__ out,
                                                      float *__restrict__ lse, int n, int C, int n_blk, int H, int D,
                                                      int64_t cache_tokens, float scale, const ifx_key_runs runs)
{
    // Keys: C cached tokens (logical order of the caller's selection, mapped to physical tokens by
    // `runs`), then the n_blk tokens of the current block (n_blk is n or 0).
    extern __shared__ float smem[];
    const int ldq = D + 1;
    float *Qs = smem;                        // [32][D+1]
    float *Ks = Qs + F32_BM * ldq;           // [64][D+1]
    float *Vs = Ks + F32_BN * ldq;           // [64][D]
    float *Ps = Vs + F32_BN * D;             // [32][65]
    const int ldp = F32_BN + 1;

    const int tid = threadIdx.x;
    const int h = blockIdx.y;
    const int row0 = blockIdx.x * F32_BM;
    const int r = tid >> 3;    // row within tile
    const int sub = tid & 7;   // position among the row's 8 threads
    const int Lk = C + n_blk;

    for (int e = tid; e < F32_BM * D; e += 256) {
        const int rr = e / D, d = e - rr * D;
        const int i = row0 + rr;
        Qs[rr * ldq + d] = (i < n) ? q[((int64_t)i * H + h) * D + d] : 0.0f;
    }

    float acc[F32_MAXD / 8];
#pragma unroll
    for (int w = 0; w < F32_MAXD / 8; ++w) acc[w] = 0.0f;
    float m = -INFINITY, l = 0.0f;
    const int nd = D >> 3;

    for (int j0 = 0; j0 < Lk; j0 += F32_BN) {
        __syncthreads();  // previous tile fully consumed (also orders the Q fill)
        for (int e = tid; e < F32_BN * D; e += 256) {
            const int jj = e / D, d = e - jj * D;
            const int j = j0 + jj;
            float kv = 0.0f, vv = 0.0f;
            if (j < C) {
                int dl = runs.delta[0];
                dl = j >= runs.end[0] ? runs.delta[1] : dl;
                dl = j >= runs.end[1] ? runs.delta[2] : dl;
                dl = j >= runs.end[2] ? runs.delta[3] : dl;
                const int64_t off = ((int64_t)h * cache_tokens + j + dl) * D + d;
                kv = kc[off];
                vv = vc[off];
            } else if (j < Lk) {
                const int64_t off = ((int64_t)(j - C) * H + h) * D + d;
                kv = kb[off];
                vv = vb[off];
            }
            Ks[jj * ldq + d] = kv;
            Vs[jj * D + d] = vv;
        }
        __syncthreads();

        // scores of row r against keys sub, sub+8, ...
        float s[8];
        float tmax = -INFINITY;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int jj = sub + 8 * u;
            float a = 0.0f;
            for (int d = 0; d < D; ++d) a = fmaf(Qs[r * ldq + d], Ks[jj * ldq + d], a);
            a *= scale;
            s[u] = (j0 + jj < Lk) ? a : -INFINITY;
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

        // out[r][sub + 8w] += sum_j P[r][j] * V[j][sub + 8w]
#pragma unroll
        for (int w = 0; w < F32_MAXD / 8; ++w) acc[w] *= alpha;
        for (int jj = 0; jj < F32_BN; ++jj) {
            const float p = Ps[r * ldp + jj];
#pragma unroll
            for (int w = 0; w < F32_MAXD / 8; ++w)
                if (w < nd) acc[w] = fmaf(p, Vs[jj * D + sub + 8 * w], acc[w]);
        }
    }

    const int i = row0 + r;
    if (i < n) {
        if (lse != nullptr && sub == 0) lse[(int64_t)i * H + h] = m + logf(l);
        const float inv = 1.0f / l;
#pragma unroll
        for (int w = 0; w < F32_MAXD / 8; ++w)
            if (w < nd) out[((int64_t)i * H + h) * D + sub + 8 * w] = acc[w] * inv;
    }
}

}  // namespace ifx
