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
//   Pipeline: the scores of tile i+1 are computed (MFMA) while the
//   exponentials of tile i are taken (VALU) in the same instruction stream;
//   K/V tiles arrive by direct global->LDS loads, double buffered, K one tile
//   ahead of V, one barrier per tile.  The K tile is XOR-swizzled at 16-byte
//   granularity (applied on the global address side of the copy) so that the
//   16 lanes of one ds_read_b128 phase hit 16 different bank groups.
#pragma once
#include "ifx_types.hpp"

namespace ifx {

constexpr int BF_D = 128;
constexpr int BF_BM = 128;
constexpr int BF_BN = 64;
constexpr int BF_THREADS = 256;
constexpr int BF_KTILE_BYTES = BF_BN * BF_D * 2;  // 16 KiB
constexpr int BF_VTILE_BYTES = BF_BN * BF_D * 2;  // 16 KiB
constexpr int BF_LDS_K0 = 0;
constexpr int BF_LDS_V0 = 2 * BF_KTILE_BYTES;
constexpr int BF_LDS_BYTES = 2 * BF_KTILE_BYTES + 2 * BF_VTILE_BYTES;  // 64 KiB
constexpr float BF_RESCALE_THRESHOLD = 8.0f;                            // log2 units

struct attn_bf16_args {
    const __bf16 *q;    // [n, H, 128]
    const __bf16 *kc;   // layer K region [H][k_tokens][128]
    const __bf16 *vt;   // layer V region, granules [H][v_tokens/8][128][8]; cache, then the staged
                        // block, then zeros up to the next multiple of 64 keys
    const __bf16 *kb;   // [n, H, 128]
    __bf16 *out;        // [n, H, 128]
    int n, C, H;
    int64_t k_tokens, v_tokens;
    float scale_log2;   // softmax scale * log2(e)
    int q_tiles;        // ceil(n / 128)
    int total;          // q_tiles * H
    int per_xcd;        // ceil(total / 8)
};

typedef const __attribute__((address_space(1))) void *gptr_t;
typedef __attribute__((address_space(3))) void *lptr_t;

__device__ __forceinline__ void wait_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

__device__ __forceinline__ float max_across_halves(float x)
{
    // lanes l and l^32 hold the two halves of one query's keys
    const unsigned u = __builtin_bit_cast(unsigned, x);
    auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__builtin_bit_cast(float, r[0]), __builtin_bit_cast(float, r[1]));
}

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
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lq = lane & 31, lh = lane >> 5;
    const int n = a.n, C = a.C, H = a.H;
    const int Lk = C + n;
    const float c2 = a.scale_log2;

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
    const int voff = lh * 2048 + lq * 16;

    // ---- global -> LDS copy roles: 4 K chunks and 4 V chunks of 16 bytes per lane per tile.
    // LDS slot c = tid + 256 x (16 bytes each).  K: slot (key = c >> 4, pos = c & 15) receives
    // the key's chunk pos ^ (key & 15).  V: slot c receives chunk c of the contiguous tile.
    const __bf16 *kc_head = a.kc + (int64_t)head * a.k_tokens * BF_D;
    const __bf16 *kb_head = a.kb + (int64_t)head * BF_D;
    const __bf16 *vt_head = a.vt + (int64_t)head * a.v_tokens * BF_D;
    const int krow = tid >> 4;                           // + 16 x
    const int kchunk = ((tid & 15) ^ (krow & 15)) << 4;  // byte offset inside the key row
    // per-lane byte offsets inside a tile that lies wholly in the cache / wholly in the block
    const unsigned vk_cache = (unsigned)(krow * (BF_D * 2) + kchunk);
    const unsigned vk_block = (unsigned)(krow * (H * BF_D * 2) + kchunk);

    auto issue_k = [&](int j0, int buf) __attribute__((always_inline)) {
        unsigned char *dst = lds + BF_LDS_K0 + buf * BF_KTILE_BYTES + wave * 1024;
        if (j0 + BF_BN <= C) {  // tile wholly in the cache: scalar base, fixed lane offsets
            const char *base = reinterpret_cast<const char *>(kc_head) + (int64_t)j0 * (BF_D * 2);
#pragma unroll
            for (int x = 0; x < 4; ++x)
                __builtin_amdgcn_global_load_lds((gptr_t)(base + x * 16 * (BF_D * 2) + vk_cache),
                                                 (lptr_t)(dst + x * 4096), 16, 0, 0);
        } else if (j0 >= C && j0 + BF_BN <= Lk) {  // wholly in the block
            const char *base = reinterpret_cast<const char *>(kb_head) + (int64_t)(j0 - C) * H * (BF_D * 2);
#pragma unroll
            for (int x = 0; x < 4; ++x)
                __builtin_amdgcn_global_load_lds((gptr_t)(base + (int64_t)x * 16 * H * (BF_D * 2) + vk_block),
                                                 (lptr_t)(dst + x * 4096), 16, 0, 0);
        } else {  // the tile straddling the cache end, or the last, partial tile: per-lane source
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                int j = j0 + krow + 16 * x;
                j = j < Lk ? j : Lk - 1;
                const char *src = (j < C) ? reinterpret_cast<const char *>(kc_head) + (int64_t)j * (BF_D * 2)
                                          : reinterpret_cast<const char *>(kb_head) + (int64_t)(j - C) * H * (BF_D * 2);
                __builtin_amdgcn_global_load_lds((gptr_t)(src + kchunk), (lptr_t)(dst + x * 4096), 16, 0, 0);
            }
        }
    };
    auto issue_v = [&](int j0, int buf) __attribute__((always_inline)) {
        const char *base = reinterpret_cast<const char *>(vt_head) + (int64_t)j0 * (BF_D * 2);
        unsigned char *dst = lds + BF_LDS_V0 + buf * BF_VTILE_BYTES + wave * 1024;
        const unsigned voff_g = (unsigned)tid * 16u;
#pragma unroll
        for (int x = 0; x < 4; ++x)
            __builtin_amdgcn_global_load_lds((gptr_t)(base + x * 4096 + voff_g), (lptr_t)(dst + x * 4096), 16, 0, 0);
    };

    f32x16 O[4];
#pragma unroll
    for (int sl = 0; sl < 4; ++sl)
#pragma unroll
        for (int r = 0; r < 16; ++r) O[sl][r] = 0.0f;
    float m_used = -INFINITY;  // maximum the exponentials are taken against (scaled log2 units)
    float l_acc[4] = {0.f, 0.f, 0.f, 0.f};  // this lane's share of the row sum, 4 partial sums

    // S^T = K Q^T for the two 32-key subtiles of the K tile in buffer `buf`.
    // Register r of S[u] is key j0 + 32 u + 16 (r/8) + 8 lh + r%8.
    auto qk = [&](int buf, f32x16 (&S)[2]) __attribute__((always_inline)) {
        const unsigned char *kb_ = lds + BF_LDS_K0 + buf * BF_KTILE_BYTES;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            f32x16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                const bf16x8 A = *reinterpret_cast<const bf16x8 *>(kb_ + u * 32 * 256 + koff[s]);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A, Q[s], acc, 0, 0, 0);
            }
            S[u] = acc;
        }
    };

    // Raise the running maximum if this tile needs it (rare after the first tiles).
    auto update_max = [&](const f32x16 (&S)[2]) __attribute__((always_inline)) {
        float mx = fmaxf(S[0][0], S[1][0]);
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, fmaxf(S[0][r], S[1][r]));
        mx = max_across_halves(mx);
        const float m_tile = mx * c2;
        const bool raise = m_tile > m_used + BF_RESCALE_THRESHOLD;  // always true on the first tile
        if (__any(raise)) {
            const float m_next = raise ? m_tile : m_used;
            const float alpha = __builtin_amdgcn_exp2f(m_used - m_next);  // 1 where unchanged, 0 at the start
#pragma unroll
            for (int k = 0; k < 4; ++k) l_acc[k] *= alpha;
#pragma unroll
            for (int sl = 0; sl < 4; ++sl)
#pragma unroll
                for (int r = 0; r < 16; ++r) O[sl][r] *= alpha;
            m_used = m_next;
        }
    };

    // P = exp2(S c2 - m) in bf16 (chunk [u][t] = 8 consecutive keys) and the row-sum share.
    auto exps = [&](const f32x16 (&S)[2], bf16x8 (&P)[2][2]) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                f32x8 p;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    p[e] = __builtin_amdgcn_exp2f(fmaf(S[u][8 * t + e], c2, -m_used));
                    l_acc[e & 3] += p[e];
                }
                P[u][t] = __builtin_convertvector(p, bf16x8);
            }
    };

    // O^T += V^T P^T from the V tile in buffer `buf`.
    auto pv = [&](int buf, const bf16x8 (&P)[2][2]) __attribute__((always_inline)) {
        const unsigned char *vb_ = lds + BF_LDS_V0 + buf * BF_VTILE_BYTES + voff;
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int sl = 0; sl < 4; ++sl) {
                    const bf16x8 A = *reinterpret_cast<const bf16x8 *>(vb_ + (4 * u + 2 * t) * 2048 + sl * 512);
                    O[sl] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A, P[u][t], O[sl], 0, 0, 0);
                }
    };

    const int T = (Lk + BF_BN - 1) / BF_BN;

    // One steady step for tile i (a later tile exists).  PAR = i & 1.
    //   K(i+1) is in K buffer PAR^1, V(i) in V buffer PAR; K(i+2) -> K buffer PAR, V(i+1) -> V buffer PAR^1.
    auto step = [&](int i, int par, f32x16 (&Scur)[2], f32x16 (&Snext)[2]) __attribute__((always_inline)) {
        if (i + 2 < T) issue_k((i + 2) * BF_BN, par);
        issue_v((i + 1) * BF_BN, par ^ 1);
        update_max(Scur);
        bf16x8 P[2][2];
        qk(par ^ 1, Snext);
        exps(Scur, P);
        pv(par, P);
        // interleave: scores of the next tile under the exponentials, then PV
        __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);
#pragma unroll
        for (int g = 0; g < 16; ++g) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, 5, 0);
            __builtin_amdgcn_sched_group_barrier(0x400, 2, 0);
        }
#pragma unroll
        for (int g = 0; g < 16; ++g) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        wait_loads();
        __syncthreads();
    };

    // The last tile: mask keys at or past Lk, no further scores to compute.
    auto last = [&](int par, f32x16 (&Scur)[2]) __attribute__((always_inline)) {
        const int j0 = (T - 1) * BF_BN;
        if (j0 + BF_BN > Lk) {
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int j = j0 + 32 * u + 16 * (r >> 3) + 8 * lh + (r & 7);
                    if (j >= Lk) Scur[u][r] = -INFINITY;
                }
        }
        update_max(Scur);
        bf16x8 P[2][2];
        exps(Scur, P);
        pv(par, P);
    };

    // ---- prologue: tile 0 (and K of tile 1) into LDS, scores of tile 0
    issue_k(0, 0);
    issue_v(0, 0);
    if (T > 1) issue_k(BF_BN, 1);
    wait_loads();
    __syncthreads();
    f32x16 Sa[2], Sb[2];
    qk(0, Sa);

    int i = 0;
    for (; i + 2 <= T - 1; i += 2) {
        step(i, 0, Sa, Sb);
        step(i + 1, 1, Sb, Sa);
    }
    if (i < T - 1) {
        step(i, 0, Sa, Sb);
        last(1, Sb);
    } else {
        last(0, Sa);
    }

    // ---- epilogue: out[q, d] = O^T[d, q] / l;  register r of O[sl] is d = 32 sl + 8 (r/4) + 4 lh + r%4
    const float l_part = (l_acc[0] + l_acc[1]) + (l_acc[2] + l_acc[3]);
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
