// bf16 block attention for gfx950: flash-style fused forward.
//
// Operation (paper, Introduction, framework paragraph + abstract): every query
// of the current block attends to all resident cached tokens of the layer and
// to all tokens of its own block; one softmax over that key set.
//
// Shape of the computation
//   A workgroup = 4 wavefronts = 128 query rows of one head; a wavefront owns
//   32 query rows.  Keys are visited in tiles of 64.  The contractions run
//   transposed so that a lane owns one query:
//     S^T (keys x queries) = K (keys x d) * Q^T (d x queries)   v_mfma_f32_32x32x16_bf16
//     O^T (d x queries)   += V^T (d x keys) * P^T (keys x queries)
//   In the 32x32 accumulator layout a lane holds column (lane % 32) and rows
//   8*(r/4) + 4*(lane/32) + r%4 for r = 0..15.  With queries as columns the
//   softmax statistics of a query live in one lane (plus its partner lane^32):
//   row max and row sum are in-register reductions and one cross-lane exchange
//   per tile.  The K rows fed to MFMA row rho are permuted (swap of two index
//   bits) so that registers 8t..8t+7 of the S^T accumulator hold 8 consecutive
//   keys: converted to bf16 they are, unchanged, the lane's B operand of the PV
//   MFMA, and the matching A operand is one 16-byte read of the V granule
//   layout (8 keys of one dimension contiguous).
//   Softmax is online in fp32 in the exp2 domain; the running maximum is only
//   raised when some query's tile maximum exceeds it by more than 2^8 (the
//   result is identical, P stays <= 256), which removes most accumulator
//   rescales.
//   K/V tiles go global -> registers -> LDS, double buffered, one barrier per
//   tile.  The K tile is XOR-swizzled at 16-byte granularity so that the 16
//   lanes of one ds_read_b128 phase hit 16 different bank groups.
#pragma once
#include "ifx_types.hpp"

namespace ifx {

constexpr int BF_D = 128;
constexpr int BF_BM = 128;
constexpr int BF_BN = 64;
constexpr int BF_THREADS = 256;
constexpr int BF_KTILE_BYTES = BF_BN * BF_D * 2;  // 16 KiB
constexpr int BF_VTILE_BYTES = BF_BN * BF_D * 2;  // 16 KiB
constexpr int BF_STAGE_BYTES = BF_KTILE_BYTES + BF_VTILE_BYTES;
constexpr int BF_LDS_BYTES = 2 * BF_STAGE_BYTES;  // 64 KiB
constexpr float BF_RESCALE_THRESHOLD = 8.0f;      // log2 units

struct attn_bf16_args {
    const __bf16 *q;    // [n, H, 128]
    const __bf16 *kc;   // layer K region [H][k_tokens][128]
    const __bf16 *vt;   // layer V region, granules [H][v_tokens/8][128][8]; holds cache then staged block
    const __bf16 *kb;   // [n, H, 128]
    __bf16 *out;        // [n, H, 128]
    int n, C, H;
    int64_t k_tokens, v_tokens;
    float scale_log2;   // softmax scale * log2(e)
    int q_tiles;        // ceil(n / 128)
    int total;          // q_tiles * H
    int per_xcd;        // ceil(total / 8)
};

__device__ __forceinline__ u32x4 ld16(const void *p) { return *reinterpret_cast<const u32x4 *>(p); }

__global__ __launch_bounds__(BF_THREADS, 2) void attn_bf16_kernel(const attn_bf16_args a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous
    // range of (head, q-tile) so the workgroups sharing an L2 stream the same heads.
    const int xcd = blockIdx.x & 7;
    const int idx = blockIdx.x >> 3;
    const int logical = xcd * a.per_xcd + idx;
    if (logical >= a.total) return;
    const int head = logical / a.q_tiles;
    const int qt = logical - head * a.q_tiles;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int lq = lane & 31, lh = lane >> 5;
    const int n = a.n, C = a.C, H = a.H;
    const int Lk = C + n;

    // ---- Q: B operand of S^T = K Q^T; lane = query lq, d = 16 s + 8 lh + [0,8)
    const int qi = qt * BF_BM + wave * 32 + lq;
    const int qi_c = qi < n ? qi : n - 1;
    bf16x8 Q[8];
    {
        const bf16x8 *qp = reinterpret_cast<const bf16x8 *>(a.q + ((int64_t)qi_c * H + head) * BF_D);
#pragma unroll
        for (int s = 0; s < 8; ++s) Q[s] = qp[2 * s + lh];
    }

    // ---- per-lane LDS read addresses
    // MFMA row rho = lq gets key 16*a1 + 8*hb + 4*a0 + b  (rho = 16*a1 + 8*a0 + 4*hb + b)
    const int pkey = (lq & 16) | ((lq & 4) << 1) | ((lq & 8) >> 1) | (lq & 3);
    const int kz = lh ^ (pkey & 15);
    int koff[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) koff[s] = pkey * 256 + (((2 * s) ^ kz) << 4);
    const int voff = BF_KTILE_BYTES + lh * 2048 + lq * 16;

    // ---- global -> LDS copy roles: 4 K chunks and 4 V chunks of 16 bytes per thread
    const __bf16 *kc_head = a.kc + (int64_t)head * a.k_tokens * BF_D;
    const __bf16 *kb_head = a.kb + (int64_t)head * BF_D;
    const __bf16 *vt_head = a.vt + (int64_t)head * a.v_tokens * BF_D;
    u32x4 kreg[4], vreg[4];

    auto load_tile = [&](int j0) {
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const int c = tid + x * BF_THREADS;
            const int key = c >> 4, dch = c & 15;
            int j = j0 + key;
            j = j < Lk ? j : Lk - 1;
            const __bf16 *src = (j < C) ? kc_head + (int64_t)j * BF_D : kb_head + (int64_t)(j - C) * H * BF_D;
            kreg[x] = ld16(src + dch * 8);
        }
        const __bf16 *vsrc = vt_head + (int64_t)j0 * BF_D;
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const int c = tid + x * BF_THREADS;
            u32x4 v = ld16(vsrc + (int64_t)c * 8);
            if (j0 + BF_BN > Lk) {
                // keys at or past Lk hold stale data: zero them so 0 * stale stays 0
                const int kbase = j0 + ((c >> 7) << 3);
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    uint32_t lo = (kbase + 2 * w < Lk) ? 0x0000ffffu : 0u;
                    uint32_t hi = (kbase + 2 * w + 1 < Lk) ? 0xffff0000u : 0u;
                    v[w] &= (lo | hi);
                }
            }
            vreg[x] = v;
        }
    };
    auto store_tile = [&](unsigned char *stage) {
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const int c = tid + x * BF_THREADS;
            const int key = c >> 4, dch = c & 15;
            *reinterpret_cast<u32x4 *>(stage + key * 256 + ((dch ^ (key & 15)) << 4)) = kreg[x];
        }
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const int c = tid + x * BF_THREADS;
            *reinterpret_cast<u32x4 *>(stage + BF_KTILE_BYTES + c * 16) = vreg[x];
        }
    };

    f32x16 O[4];
#pragma unroll
    for (int sl = 0; sl < 4; ++sl)
#pragma unroll
        for (int r = 0; r < 16; ++r) O[sl][r] = 0.0f;
    float m_used = -INFINITY;  // maximum the exponentials are taken against (scaled log2 units)
    float l_part = 0.0f;       // this lane's share of the row sum

    const int n_tiles = (Lk + BF_BN - 1) / BF_BN;
    load_tile(0);
    store_tile(lds);
    __syncthreads();

    for (int it = 0; it < n_tiles; ++it) {
        const unsigned char *stage = lds + (it & 1) * BF_STAGE_BYTES;
        const int j0 = it * BF_BN;
        const bool more = it + 1 < n_tiles;
        if (more) load_tile(j0 + BF_BN);

        // ---- S^T = K Q^T for two 32-key subtiles
        f32x16 S[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
#pragma unroll
            for (int r = 0; r < 16; ++r) S[u][r] = 0.0f;
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                const bf16x8 A = *reinterpret_cast<const bf16x8 *>(stage + u * 32 * 256 + koff[s]);
                S[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A, Q[s], S[u], 0, 0, 0);
            }
        }
        // register r of S[u] is key j0 + 32 u + 16 (r/8) + 8 lh + r%8
        if (j0 + BF_BN > Lk) {
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int j = j0 + 32 * u + 16 * (r >> 3) + 8 * lh + (r & 7);
                    if (j >= Lk) S[u][r] = -INFINITY;
                }
        }

        // ---- online softmax, one query per lane pair (lane, lane ^ 32)
        float mx = S[0][0];
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, S[u][r]);
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_tile = mx * a.scale_log2;
        const bool raise = m_tile > m_used + BF_RESCALE_THRESHOLD;  // always true on the first tile
        if (__any(raise)) {
            const float m_next = raise ? m_tile : m_used;
            const float alpha = __builtin_amdgcn_exp2f(m_used - m_next);  // 1 where unchanged, 0 on the first tile
            l_part *= alpha;
#pragma unroll
            for (int sl = 0; sl < 4; ++sl)
#pragma unroll
                for (int r = 0; r < 16; ++r) O[sl][r] *= alpha;
            m_used = m_next;
        }
        bf16x8 P[2][2];
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                f32x8 p;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    p[e] = __builtin_amdgcn_exp2f(fmaf(S[u][8 * t + e], a.scale_log2, -m_used));
                    l_part += p[e];
                }
                P[u][t] = __builtin_convertvector(p, bf16x8);
            }

        // ---- O^T += V^T P^T
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int sl = 0; sl < 4; ++sl) {
                    const bf16x8 A =
                        *reinterpret_cast<const bf16x8 *>(stage + voff + (4 * u + 2 * t) * 2048 + sl * 512);
                    O[sl] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A, P[u][t], O[sl], 0, 0, 0);
                }

        if (more) store_tile(lds + ((it + 1) & 1) * BF_STAGE_BYTES);
        __syncthreads();
    }

    // ---- epilogue: out[q, d] = O^T[d, q] / l;  register r of O[sl] is d = 32 sl + 8 (r/4) + 4 lh + r%4
    const float l_tot = l_part + __shfl_xor(l_part, 32);
    const float inv = 1.0f / l_tot;
    if (qi < n) {
        __bf16 *op = a.out + ((int64_t)qi * H + head) * BF_D;
#pragma unroll
        for (int sl = 0; sl < 4; ++sl)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                f32x4 o4;
#pragma unroll
                for (int b = 0; b < 4; ++b) o4[b] = O[sl][4 * g + b] * inv;
                *reinterpret_cast<bf16x4 *>(op + 32 * sl + 8 * g + 4 * lh) = __builtin_convertvector(o4, bf16x4);
            }
    }
}

}  // namespace ifx
