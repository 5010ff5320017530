// bf16 block attention for gfx950: flash-style fused forward.
//
// Operation (paper, Introduction, framework paragraph + abstract): every query
// of the current block attends to all resident cached tokens of the layer and
// to all tokens of its own block; one softmax over that key set.
//
// Shape of the computation
//   A workgroup = 8 wavefronts = 256 query rows of one head, one workgroup per
//   CU; a wavefront owns 32 query rows.  Keys arrive in LDS tiles of 64 and
//   are consumed in subtiles of 32.  The contractions run transposed so that a
//   lane owns one query:
//     S^T (keys x queries) = K (keys x d) * Q^T (d x queries)   v_mfma_f32_32x32x16_bf16
//     O^T (d x queries)   += V^T (d x keys) * P^T (keys x queries)
//   In the 32x32 accumulator layout a lane holds column (lane % 32) and rows
//   8*(r/4) + 4*(lane/32) + r%4 for r = 0..15.  With queries as columns the
//   softmax statistics of a query live in one lane (plus its partner lane^32):
//   row max and row sum are in-register reductions and one cross-lane exchange
//   per subtile.  The K rows fed to MFMA row rho are permuted (swap of two
//   index bits) so that registers 8t..8t+7 of the S^T accumulator hold 8
//   consecutive keys: converted to bf16 they are, unchanged, the lane's B
//   operand of the PV MFMA, and the matching A operand is one 16-byte read of
//   the V granule layout (8 keys of one dimension contiguous).
//   Softmax is online in fp32 in the exp2 domain; the running maximum is only
//   raised when some query's subtile maximum exceeds it by more than 2^8 (the
//   result is identical, P stays <= 256), which removes most accumulator
//   rescales.  The row sum is taken from the fp32 exponentials with plain adds.
//   Bounded maximum: |s_ij| <= |q_i| max_j |k_j| (Cauchy-Schwarz).  The cache
//   keeps the largest key norm of every resident block and of the current
//   block per head; when that bound, in log2 units, is small enough that
//   2^(s - bound) can neither overflow nor all underflow (bound <= 50), a
//   wavefront uses it as a fixed maximum for the whole key range: no running
//   maximum, no rescale, no branch in the loop, the same softmax.  Otherwise it
//   runs the running-maximum path.  Either way only a partial last tile is masked.
//   Keys: the caller stages the current block's K and V behind the resident
//   tokens in the cache's own layouts, so a head's keys are one contiguous
//   range of its K region and of its V region (or, in the table
//   instantiation, a list of whole blocks of them).
//   Pipeline, per 32-key subtile: the scores of the next subtile (8 MFMA) are
//   issued interleaved with the exponentials of the current one (VALU), then
//   the PV product of the current one (8 MFMA) interleaved with the maximum of
//   the next taken early.  One MFMA operand is read from LDS per MFMA, eight
//   MFMAs ahead of its use.  K/V tiles arrive by direct global->LDS loads three
//   tiles ahead into rings of four buffers, issued between the PV MFMAs (a
//   steady tile is branch-free), one barrier per 64-key tile.  The
//   K tile is XOR-swizzled at 16-byte granularity (applied on the global
//   address side of the copy) so that the 16 lanes of one ds_read_b128 phase
//   hit 16 different bank groups.
#pragma once
#include <type_traits>

#include "ifx_types.hpp"

namespace ifx {

constexpr int BF_D = 128;
constexpr int BF_WAVES = 8;
constexpr int BF_BM = 32 * BF_WAVES;  // 256 query rows per workgroup
constexpr int BF_BN = 64;
constexpr int BF_THREADS = 64 * BF_WAVES;
constexpr int BF_TILE_BYTES = BF_BN * BF_D * 2;  // 16 KiB, K and V alike
constexpr int BF_NBUF = 4;
constexpr int BF_NX = (BF_TILE_BYTES / 16) / BF_THREADS;  // 16-byte chunks per lane per tile
constexpr int BF_XROWS = BF_THREADS / 16;                   // key rows covered by one chunk round
constexpr int BF_XBYTES = BF_THREADS * 16;                  // LDS bytes covered by one chunk round
constexpr int BF_LDS_V0 = 0;
constexpr int BF_LDS_K0 = BF_NBUF * BF_TILE_BYTES;
constexpr int BF_LDS_BYTES = 2 * BF_NBUF * BF_TILE_BYTES;  // 128 KiB
constexpr float BF_RESCALE_THRESHOLD = 8.0f;               // log2 units
constexpr float BF_BOUND_LIMIT = 50.0f;                    // log2 units; 2^-100 is still a normal bf16 / fp32

struct attn_bf16_args {
    const __bf16 *q;    // [n, H, 128]
    const __bf16 *kc;   // layer K region [H][k_tokens][128]: cache, then the staged block
    const __bf16 *vt;   // layer V region, granules [H][v_tokens/8][128][8]; cache, then the staged
                        // block, then zeros up to the next multiple of 64 keys
    __bf16 *out;        // [n, H, 128]
    float *lse;         // [n, H] natural-log sum of exp of the scaled scores, or nullptr
    int n, Lk, H;       // queries, keys, heads
    ifx_key_blocks blocks;  // table instantiation only: where the n keys of block j / n live
    int64_t k_tokens, v_tokens;
    float scale_log2;   // softmax scale * log2(e)
    const unsigned long long *knorm;  // [cap_blocks + 1][H]: (epoch << 32) | bits of max |k|^2; last row = current block
    int resident_blocks, cap_blocks;
    int q_tiles;        // ceil(n / 256)
    // (head, q-tile) items per XCD: first all q-tiles of whole_heads heads of its own, then its
    // share of the H % 8 heads that are left: each of those split over `share` XCDs, left_chunk
    // q-tiles apiece (when H % 8 divides 8), or (share == 0) their items dealt out contiguously,
    // left_chunk apiece.  The grid is 8 * (whole_heads * q_tiles + left_chunk) workgroups.
    int whole_heads, left_heads, share, left_chunk;
};

typedef __attribute__((address_space(3))) void *lptr_t;

// scalar offsets of the BF_NX copy instructions that bring in a wavefront's share of one K or V tile
struct tile_offs {
    int s[BF_NX];
};

// Wait until at most `keep` of this wave's global->LDS loads are still in flight (they complete in
// issue order), then meet the other waves.  No fence: LDS data of completed loads is visible.
template <int keep>
__device__ __forceinline__ void wait_loads_and_sync()
{
    // s_waitcnt vmcnt(keep) only: expcnt and lgkmcnt fields at their no-wait maxima.  A builtin
    // rather than inline asm, so the compiler keeps exact track of its own LDS read counters.
    __builtin_amdgcn_s_waitcnt((keep & 0xF) | (7 << 4) | (15 << 8) | ((keep >> 4) << 14));
    __builtin_amdgcn_s_barrier();
}

__device__ __forceinline__ float max_across_halves(float x)
{
    // lanes l and l^32 hold the two halves of one query's keys
    const unsigned u = __builtin_bit_cast(unsigned, x);
    auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__builtin_bit_cast(float, r[0]), __builtin_bit_cast(float, r[1]));
}

#define IFX_INLINE __attribute__((always_inline))


// SEG == false: the keys are the physical tokens [0, Lk) of the head's regions (resident blocks in
// slot order, then the staged block).  SEG == true: the keys are a list of up to IFX_MAX_KEY_BLOCKS
// blocks of n physical tokens each (a caller-given selection of resident blocks in any order, or
// a ring that has wrapped, then the staged block); the tile copies then look their block up
// (scalar arithmetic), everything else is the same code.
template <bool SEG>
__global__ __launch_bounds__(BF_THREADS, 1) void attn_bf16_kernel(const attn_bf16_args a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    // Workgroups are dealt round-robin to the 8 XCDs, each with an L2 of its own.  A head's K/V
    // stream is shared by all its q-tiles, so a head is given to as few XCDs as possible: whole
    // heads per XCD first, the H % 8 heads that are left over split evenly.
    const int xcd = blockIdx.x & 7;
    const int idx = blockIdx.x >> 3;
    int head, qt;
    if (idx < a.whole_heads * a.q_tiles) {
        head = xcd * a.whole_heads + idx / a.q_tiles;
        qt = idx % a.q_tiles;
    } else {
        const int rest = idx - a.whole_heads * a.q_tiles;
        if (a.share > 0) {
            head = 8 * a.whole_heads + xcd / a.share;
            qt = (xcd % a.share) * a.left_chunk + rest;
            if (qt >= a.q_tiles) return;
        } else {
            const int item = xcd * a.left_chunk + rest;
            if (item >= a.left_heads * a.q_tiles) return;
            head = 8 * a.whole_heads + item / a.q_tiles;
            qt = item % a.q_tiles;
        }
    }

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lq = lane & 31, lh = lane >> 5;
    const int n = a.n, Lk = a.Lk, H = a.H;
    const float c2 = a.scale_log2;

    const int T = (Lk + BF_BN - 1) / BF_BN;

    // ---- Q: B operand of S^T = K Q^T; lane = query lq, d = 16 s + 8 lh + [0,8)
    const int qi = qt * BF_BM + wave * 32 + lq;
    const int qi_c = qi < n ? qi : n - 1;
    bf16x8 Q[8];
    {
        const bf16x8 *qp = reinterpret_cast<const bf16x8 *>(a.q + ((int64_t)qi_c * H + head) * BF_D);
#pragma unroll
        for (int s = 0; s < 8; ++s) Q[s] = qp[2 * s + lh];
    }

    // ---- Cauchy-Schwarz bound on this query's scaled scores (log2 units)
    float m_bound;
    {
        float q2 = 0.f;
#pragma unroll
        for (int s = 0; s < 8; ++s)
#pragma unroll
            for (int e = 0; e < 8; ++e) q2 = fmaf((float)Q[s][e], (float)Q[s][e], q2);
        const unsigned u = __builtin_bit_cast(unsigned, q2);
        auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
        q2 = __builtin_bit_cast(float, r[0]) + __builtin_bit_cast(float, r[1]);
        uint32_t kbits = (uint32_t)a.knorm[(int64_t)a.cap_blocks * H + head];
        for (int sl = 0; sl < a.resident_blocks; ++sl) {
            const uint32_t b = (uint32_t)a.knorm[(int64_t)sl * H + head];
            kbits = b > kbits ? b : kbits;
        }
        m_bound = sqrtf(q2 * __builtin_bit_cast(float, kbits)) * c2 * 1.001f + 1e-6f;
    }
    const bool bounded = __all(m_bound <= BF_BOUND_LIMIT);  // false for NaN / infinite norms

    // ---- per-lane LDS read addresses
    // MFMA row rho = lq gets key 16*a1 + 8*hb + 4*a0 + b  (rho = 16*a1 + 8*a0 + 4*hb + b)
    const int pkey = (lq & 16) | ((lq & 4) << 1) | ((lq & 8) >> 1) | (lq & 3);
    const int kz = lh ^ (pkey & 15);
    int koff[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) koff[s] = BF_LDS_K0 + pkey * 256 + (((2 * s) ^ kz) << 4);
    const int voff = BF_LDS_V0 + lh * 2048 + lq * 16;

    // ---- global -> LDS copy roles: 2 K chunks and 2 V chunks of 16 bytes per lane per tile.
    // LDS slot c = tid + BF_THREADS x (16 bytes each).  K: slot (key = c >> 4, pos = c & 15) receives
    // the key's chunk pos ^ (key & 15).  V: slot c receives chunk c of the contiguous tile.
    const __bf16 *kc_head = a.kc + (int64_t)head * a.k_tokens * BF_D;
    const __bf16 *vt_head = a.vt + (int64_t)head * a.v_tokens * BF_D;
    const int krow = tid >> 4;                           // + BF_XROWS x
    const int kchunk = ((tid & 15) ^ (krow & 15)) << 4;  // byte offset inside the key row
    // Buffer descriptors (raw, byte-addressed): reads past num_records return zero and touch no
    // memory, so the rows of a partial last tile need no clamping and a load of a tile past the
    // last one is harmless.  Lane offsets are 32-bit, tile offsets are scalars.
    const __amdgpu_buffer_rsrc_t rs_k = __builtin_amdgcn_make_buffer_rsrc(
        (void *)kc_head, 0, SEG ? (int)(a.k_tokens * (BF_D * 2)) : Lk * (BF_D * 2), 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_v =
        __builtin_amdgcn_make_buffer_rsrc((void *)vt_head, 0, (int)(a.v_tokens * (BF_D * 2)), 0x00020000);
    const int vk_lane = krow * (BF_D * 2) + kchunk;
    const int vv_lane = tid * 16;
    // Selected keys.  Blocks are multiples of 8 tokens and a wavefront's share of one copy
    // instruction is 4 consecutive key rows (K) or half a granule of 8 keys (V), aligned, so the
    // block a copy instruction reads from is the same for the whole wavefront: the lookup is
    // scalar (block index by a multiply-high, its offset by a lane read of the table kept in one
    // register) and goes into the scalar offset, like the tile offset.  No memory access: an
    // indexed load of the table would wait for every outstanding tile copy.
    // The table holds byte offsets, 2^30 in the lanes behind the last entry: block_tokens divides
    // the key count, so a key is past the end exactly when its block index is, and its copy then
    // starts beyond any region (at most 2^30 bytes) and reads as zero.
    int tab = 0;
    if constexpr (SEG) tab = lane < a.blocks.count ? a.blocks.delta[lane] * (BF_D * 2) : (1 << 30);
    const unsigned blk_magic = SEG ? a.blocks.magic : 0u;
    auto key_offset = [&](int j) IFX_INLINE -> int {  // scalar byte offset of key row / granule j in the head's region
        const int p = __builtin_amdgcn_readfirstlane((int)__umulhi((unsigned)j, blk_magic));  // j / n
        return j * (BF_D * 2) + __builtin_amdgcn_readlane(tab, p < 63 ? p : 63);
    };

    // (the scalar offset must not go negative: it carries the wavefront's own first row / granule,
    // the lane offset only what is left inside those)
    const int vk_lane_seg = ((tid >> 4) & 3) * (BF_D * 2) + kchunk, vv_lane_seg = (tid & 127) * 16;
    // Scalar offsets of a tile's BF_NX K (V) copy instructions, and the copies themselves.  Two
    // steps, because with the block table an offset is a chain of a dozen scalar instructions: the
    // pipelined loop works them out a phase ahead of the copies, under other MFMAs.
    auto k_offs = [&](int j0) IFX_INLINE -> tile_offs {
        tile_offs t;
#pragma unroll
        for (int x = 0; x < BF_NX; ++x) {
            if constexpr (SEG) {
                t.s[x] = key_offset(j0 + x * BF_XROWS + wave * 4);  // first of this wavefront's 4 key rows
            } else {
                t.s[x] = (j0 + x * BF_XROWS) * (BF_D * 2);
            }
        }
        return t;
    };
    auto v_offs = [&](int j0) IFX_INLINE -> tile_offs {
        tile_offs t;
#pragma unroll
        for (int x = 0; x < BF_NX; ++x) {
            if constexpr (SEG) {
                t.s[x] = key_offset(j0 + 8 * ((wave >> 1) + (BF_XBYTES / 2048) * x));  // first key of this wavefront's granule
            } else {
                t.s[x] = j0 * (BF_D * 2) + x * BF_XBYTES;
            }
        }
        return t;
    };
    auto issue_k_at = [&](const tile_offs &t, int buf) IFX_INLINE {
        unsigned char *dst = lds + BF_LDS_K0 + buf * BF_TILE_BYTES + wave * 1024;
#pragma unroll
        for (int x = 0; x < BF_NX; ++x)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_k, (lptr_t)(dst + x * BF_XBYTES), 16, SEG ? vk_lane_seg : vk_lane, t.s[x], 0, 0);
    };
    auto issue_v_at = [&](const tile_offs &t, int buf) IFX_INLINE {
        unsigned char *dst = lds + BF_LDS_V0 + buf * BF_TILE_BYTES + wave * 1024;
#pragma unroll
        for (int x = 0; x < BF_NX; ++x)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_v, (lptr_t)(dst + x * BF_XBYTES), 16, SEG ? vv_lane_seg : vv_lane, t.s[x], 0, 0);
    };
    auto issue_k = [&](int j0, int buf) IFX_INLINE { issue_k_at(k_offs(j0), buf); };
    auto issue_v = [&](int j0, int buf) IFX_INLINE { issue_v_at(v_offs(j0), buf); };

    f32x16 O[4];
#pragma unroll
    for (int sl = 0; sl < 4; ++sl)
#pragma unroll
        for (int r = 0; r < 16; ++r) O[sl][r] = 0.0f;
    float m_used = -INFINITY;     // maximum the exponentials are taken against (scaled log2 units)
    float l_acc[4] = {0.f, 0.f, 0.f, 0.f};  // this lane's share of the row sum, in partial sums

    // The eight K operands (one per 16-wide d step) of the 32-key subtile at LDS byte offset koffs.
    // Issue order 3,2,1,0,7,6,5,4: the MFMA that consumes operand 0 (4) waits for the youngest read
    // of its group of four, so one wait covers the group.
    auto k_fetch = [&](int koffs, bf16x8 (&A)[8]) IFX_INLINE {
#pragma unroll
        for (int o = 0; o < 8; ++o) {
            const int s = (o & 4) | (3 - (o & 3));
            A[s] = *reinterpret_cast<const bf16x8 *>(lds + koffs + koff[s]);
        }
    };
    // The eight V operands (key step t, d slab sl) of the subtile whose granules start at voffs.
    auto v_fetch = [&](int voffs, bf16x8 (&A)[8]) IFX_INLINE {
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int o = 0; o < 4; ++o) {
                const int sl = 3 - o;
                A[t * 4 + sl] = *reinterpret_cast<const bf16x8 *>(lds + voffs + voff + t * 4096 + sl * 512);
            }
    };
    // S^T = K Q^T; register r of S is key (subtile base) + 16 (r/8) + 8 lh + r%8.
    auto qk = [&](const bf16x8 (&A)[8], f32x16 &S) IFX_INLINE {
        f32x16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < 8; ++s) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[s], Q[s], acc, 0, 0, 0);
        S = acc;
    };

    // Does this subtile force a higher running maximum?
    auto tile_max = [&](const f32x16 &S, float &m_tile) IFX_INLINE -> bool {
        // a shallow tree: the dependent chain is what a lone wavefront cannot hide
        const float a0 = fmaxf(fmaxf(S[0], S[1]), S[2]), a1 = fmaxf(fmaxf(S[3], S[4]), S[5]);
        const float a2 = fmaxf(fmaxf(S[6], S[7]), S[8]), a3 = fmaxf(fmaxf(S[9], S[10]), S[11]);
        const float a4 = fmaxf(fmaxf(S[12], S[13]), S[14]);
        const float b0 = fmaxf(fmaxf(a0, a1), a2), b1 = fmaxf(fmaxf(a3, a4), S[15]);
        const float mx = max_across_halves(fmaxf(b0, b1));
        m_tile = mx * c2;
        return m_tile > m_used + BF_RESCALE_THRESHOLD;  // always true on the first subtile
    };
    auto rescale = [&](bool raise, float m_tile) IFX_INLINE {
        const float m_next = raise ? m_tile : m_used;
        const float alpha = __builtin_amdgcn_exp2f(m_used - m_next);  // 1 where unchanged, 0 at the start
#pragma unroll
        for (int e = 0; e < 4; ++e) l_acc[e] *= alpha;
#pragma unroll
        for (int sl = 0; sl < 4; ++sl)
#pragma unroll
            for (int r = 0; r < 16; ++r) O[sl][r] *= alpha;
        m_used = m_next;
    };

    // P = exp2(S c2 - m) in bf16 (P[t] = 8 consecutive keys), with the fp32 exponentials left in
    // S for row_sum: plain adds, placed under the PV MFMAs.  (Summing the bf16-rounded P with
    // v_dot2c_f32_bf16 halves the instruction count but that instruction stalls next to MFMAs:
    // 6 % slower.)  The sum runs over the unrounded values; the rounding of P is unbiased, so it
    // differs from the sum of what the PV product uses by a relative 2^-9 / sqrt(keys).
    auto exps_keep = [&](f32x16 &S, bf16x8 (&P)[2]) IFX_INLINE {
#pragma unroll
        for (int r = 0; r < 16; ++r) S[r] = __builtin_amdgcn_exp2f(fmaf(S[r], c2, -m_used));
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            f32x8 p;
#pragma unroll
            for (int e = 0; e < 8; ++e) p[e] = S[8 * t + e];
            P[t] = __builtin_convertvector(p, bf16x8);
        }
    };
    auto row_sum = [&](const f32x16 &S) IFX_INLINE {
#pragma unroll
        for (int r = 0; r < 16; ++r) l_acc[r & 3] += S[r];
    };

    // O^T += V^T P^T.
    auto pv = [&](const bf16x8 (&A)[8], const bf16x8 (&P)[2]) IFX_INLINE {
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int sl = 0; sl < 4; ++sl)
                O[sl] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[t * 4 + sl], P[t], O[sl], 0, 0, 0);
    };

    // Keys at or past Lk never count.
    auto mask_keys = [&](f32x16 &S, int j_sub) IFX_INLINE {
        if (j_sub + 32 > Lk) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int j = j_sub + 16 * (r >> 3) + 8 * lh + (r & 7);
                if (j >= Lk) S[r] = -INFINITY;
            }
        }
    };

    bf16x8 Kop[8];  // K operands of the subtile whose scores are computed next
    bf16x8 Vop[8];  // V operands of the current subtile

    // One pipelined step of 16 MFMAs, one LDS operand read per MFMA, each read eight MFMAs ahead
    // of its use.  Scores of the NEXT subtile (operands already in Kop) with the V operands of the
    // CURRENT subtile fetched meanwhile and its exponentials spread under them; then the PV
    // product of the current subtile with the K operands of the subtile AFTER the next fetched
    // meanwhile and the maximum of the next subtile taken early.
    //   koffs_after: LDS offset of the subtile after the next; voffs_cur: offset of the current
    //   subtile's V granules.  Only for subtiles that lie wholly below Lk (no key masking).
    //   load_tag: which half of the tile three ahead this step brings in (0: K, 1: V), two
    //   global->LDS loads placed between the PV MFMAs; j_load / buf_load: its first key and ring slot.
    auto halfstep = [&](auto bounded_tag, auto load_tag, f32x16 &Scur, f32x16 &Snext, int koffs_after, int voffs_cur,
                        int j_load, int buf_load) IFX_INLINE {
        constexpr bool BOUNDED = decltype(bounded_tag)::value;
        bf16x8 P[2];
        const tile_offs offs = decltype(load_tag)::value == 0 ? k_offs(j_load) : v_offs(j_load);  // for the copies of the PV phase
        qk(Kop, Snext);
        v_fetch(voffs_cur, Vop);
        exps_keep(Scur, P);
#pragma unroll
        for (int g = 0; g < 8; ++g) {  // score MFMAs: V operand reads, exponentials
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, BOUNDED ? 3 : 4, 0);
            __builtin_amdgcn_sched_group_barrier(0x400, 2, 0);
        }
        // Wave priority: high while a wavefront is in its score phase (per MFMA 3-4 VALU and 2
        // transcendental instructions), low in its PV phase (per MFMA 2 VALU).  The two wavefronts
        // of a SIMD then settle into opposite phases: the one with the long instruction stream is
        // never held up, the other one's MFMAs fill the gaps.  (The instruction ends a scheduling
        // region, so each phase's instructions and its group sequence sit on their own side of it.)
        __builtin_amdgcn_s_setprio(0);
        if constexpr (decltype(load_tag)::value == 0)
            issue_k_at(offs, buf_load);
        else
            issue_v_at(offs, buf_load);
        pv(Vop, P);
        k_fetch(koffs_after, Kop);
        row_sum(Scur);
        if constexpr (BOUNDED) {
#pragma unroll
            for (int g = 0; g < 8; ++g) {  // PV MFMAs: K operand reads, row sum, the two loads
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);
                if (g == 1 || g == 5) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
            }
            // Never taken (n > 0).  Without a use of the row sum at the end of every step the
            // compiler moves all row-sum instructions of four tiles behind the last barrier of the
            // unrolled loop, where nothing hides them and the exponentials stay live meanwhile.
            if (__builtin_expect(n < 0, 0)) {
#pragma unroll
                for (int e = 0; e < 4; ++e) l_acc[e] *= 2.0f;
            }
        } else {
            float m_tile;
            const bool raise = tile_max(Snext, m_tile);
#pragma unroll
            for (int g = 0; g < 8; ++g) {  // PV MFMAs: K operand reads, maximum of the next subtile, the two loads
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                if (g >= 2 && g < 5) __builtin_amdgcn_sched_group_barrier(0x002, 5, 0);
                if (g == 1 || g == 5) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
            }
            if (__builtin_expect(__any(raise), 0)) rescale(raise, m_tile);  // rare: keep it off the fall-through path
        }
        __builtin_amdgcn_s_setprio(1);
    };

    // ---- prologue: tiles 0, 1, 2 on their way into LDS, scores and maximum of subtile (0,0)
    issue_k(0, 0);
    issue_v(0, 0);
    if (T > 1) {
        issue_k(BF_BN, 1);
        issue_v(BF_BN, 1);
    }
    if (T > 2) {
        issue_k(2 * BF_BN, 2);
        issue_v(2 * BF_BN, 2);
    }
    wait_loads_and_sync<0>();
    // Everything after the first tiles have landed, for one of the two softmax variants.
    auto run = [&](auto bounded_tag) IFX_INLINE {
        constexpr bool BOUNDED = decltype(bounded_tag)::value;
        f32x16 Sa, Sb;
        k_fetch(0, Kop);
        qk(Kop, Sa);
        if constexpr (!BOUNDED) {
            mask_keys(Sa, 0);
            float m_tile;
            const bool raise = tile_max(Sa, m_tile);
            if (__builtin_expect(__any(raise), 0)) rescale(raise, m_tile);  // rare: keep it off the fall-through path
        }
        k_fetch(8192, Kop);  // subtile (0,1)

        // Tile i: K(i) (second half), K(i+1) (first half) and V(i) are read; K(i+2), V(i+2) are
        // landing (issued during tile i-1, needed from tile i+1 on); K(i+3), V(i+3) are issued
        // during this tile into ring slot (i+3) % 4, whose last readers finished before the previous
        // barrier.  At the tile's end only the loads issued in this tile may still be in flight.
        // b = i % 4 is a compile-time constant in the unrolled steady loop; the tile has no branch.
        auto tile_steady = [&](int i, int b) IFX_INLINE {
            const int b1 = (b + 1) % 4, b3 = (b + 3) % 4;
            const int j3 = (i + 3) * BF_BN;  // past the last tile: the loads read as zero and touch no memory
            halfstep(bounded_tag, std::integral_constant<int, 0>{}, Sa, Sb, b1 * BF_TILE_BYTES, b * BF_TILE_BYTES, j3, b3);
            halfstep(bounded_tag, std::integral_constant<int, 1>{}, Sb, Sa, b1 * BF_TILE_BYTES + 8192,
                     b * BF_TILE_BYTES + 8192, j3, b3);
            wait_loads_and_sync<2 * BF_NX>();
        };
        // Steady tiles take no key mask.  Running maximum: they need tile i+1 complete, i.e.
        // i + 2 <= Lk / 64 (the maximum of the next subtile is taken early).  Bounded maximum: every
        // complete tile is a steady tile; scores computed past the last tile are never used.  What is
        // left (at most the last two tiles, one for the bounded maximum) goes through the masked loop
        // below.  Keys past Lk must not be left to their zero K rows: when every real score of a row
        // is far below the bound, 2^(0 - bound) per padded key would swamp the row sum.
        const int n_steady = BOUNDED ? Lk / BF_BN : ((Lk / BF_BN >= 2) ? Lk / BF_BN - 1 : 0);
        int i = 0;
        for (; i + 4 <= n_steady; i += 4) {
            tile_steady(i, 0);
            tile_steady(i + 1, 1);
            tile_steady(i + 2, 2);
            tile_steady(i + 3, 3);
        }
        // up to three more steady tiles (i is a multiple of 4 here, so the ring slot is the count)
        if (i < n_steady) {
            tile_steady(i, 0);
            ++i;
            if (i < n_steady) {
                tile_steady(i, 1);
                ++i;
                if (i < n_steady) {
                    tile_steady(i, 2);
                    ++i;
                }
            }
        }
        // The last tiles, one 32-key subtile at a time without software pipelining: exponentials and
        // PV of the current subtile, then scores, key mask and (running maximum) maximum of the next.
        // Sa holds the scores of subtile (i, 0); with the running maximum its maximum is already
        // taken and it is complete, with the bounded maximum it may be the partial one.
        {
            const int n_sub = (Lk + 31) >> 5;  // subtiles holding at least one key
            if constexpr (BOUNDED) mask_keys(Sa, i * BF_BN);
#pragma unroll 1
            for (int sg = 2 * i; sg < n_sub; ++sg) {
                const int ti = sg >> 1, u = sg & 1;
                if (u == 0 && ti + 3 < T) {
                    issue_k((ti + 3) * BF_BN, (ti + 3) & 3);
                    issue_v((ti + 3) * BF_BN, (ti + 3) & 3);
                }
                bf16x8 P[2];
                v_fetch((ti & 3) * BF_TILE_BYTES + u * 8192, Vop);
                exps_keep(Sa, P);
                row_sum(Sa);
                pv(Vop, P);
                if (sg + 1 < n_sub) {
                    const int tn = (sg + 1) >> 1, un = (sg + 1) & 1;
                    k_fetch((tn & 3) * BF_TILE_BYTES + un * 8192, Kop);
                    qk(Kop, Sa);
                    mask_keys(Sa, (sg + 1) * 32);
                    if constexpr (!BOUNDED) {
                        float m_tile;
                        const bool raise = tile_max(Sa, m_tile);
                        if (__builtin_expect(__any(raise), 0)) rescale(raise, m_tile);  // rare
                    }
                }
                if (u == 1 || sg + 1 == n_sub) wait_loads_and_sync<0>();  // one barrier per tile on every path
            }
        }
    };
    if (bounded) {
        m_used = m_bound;
        run(std::true_type{});
    } else {
        run(std::false_type{});
    }

    // ---- epilogue: out[q, d] = O^T[d, q] / l;  register r of O[sl] is d = 32 sl + 8 (r/4) + 4 lh + r%4
    const float l_part = (l_acc[0] + l_acc[1]) + (l_acc[2] + l_acc[3]);
    const float l_tot = l_part + __shfl_xor(l_part, 32);
    const float inv = 1.0f / l_tot;
    if (a.lse != nullptr && lh == 0 && qi < n)  // ln sum_j exp(scale s_ij) = ln 2 * (m + log2 l)
        a.lse[(int64_t)qi * H + head] = (m_used + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f;
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
