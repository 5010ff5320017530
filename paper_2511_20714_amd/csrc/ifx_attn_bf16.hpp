// bf16 block attention for gfx950: flash-style fused forward.
//
// Operation (paper, Introduction, framework paragraph + abstract): every query
// of the current block attends to all resident cached tokens of the layer and
// to all tokens of its own block; one softmax over that key set.
//
// Shape of the computation
//   A workgroup = 8 wavefronts = up to 256 query rows of one head, one workgroup
//   per CU; a wavefront owns 32 query rows.  Keys arrive in LDS tiles of 64 and
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
//   Softmax is online in fp32 in the exp2 domain.  Running maximum: the
//   exponentials are taken against a per-query reference that is raised only
//   when a score comes out above it, and then to 2^7 above that score (the
//   result is identical: numerator and denominator carry the same factor), so
//   accumulator rescales are rare; in the pipelined loop the check is
//   made after the fact, on the exponentials (an OR over their bit patterns),
//   and the rare hit redoes the subtile's exponentials from its scores.  The
//   row sum is taken with plain adds: from the fp32 exponentials where the
//   scores are bounded (below), from the exponentials as rounded to bf16 - the
//   weights the PV product uses - where they are not, so that a row dominated
//   by one key is exact whatever that key's weight; there the reference is
//   raised 2^31 above a new maximum instead of 2^7.
//   Bounded maximum: |s_ij| <= |q_i| max_j |k_j| (Cauchy-Schwarz).  The cache
//   keeps the largest key norm of every resident block and of the current
//   block per head; when that bound, in log2 units, is small enough that
//   2^(s - bound) can neither overflow nor all underflow (bound <= 50), a
//   wavefront uses it as a fixed maximum for the whole key range: no running
//   maximum, no rescale, no branch in the loop, the same softmax.  Otherwise
//   (and in a call without cached keys) it runs the running-maximum path with
//   the exact row sum.  Either way only the partial last tile of a phase is
//   masked.
//   Keys, two phases over one set of accumulators.  Phase 1: the resident
//   tokens, one contiguous range of the head's K region and of its V region
//   (or, in the table instantiation, a list of whole blocks of them).  Phase 2:
//   the current block, read where the caller has it: K rows through a second
//   buffer descriptor (row stride heads * 256 bytes), V rows copied row-major
//   into LDS and turned into MFMA operands by transposing LDS reads
//   (ds_read_b64_tr_b16: 16 lanes read 4 rows x 32 bytes, lane i receives
//   column i of the 4 rows), two per operand.  The cache keeps no key norm of
//   the current block, so phase 2 always runs a running maximum, starting
//   from the reference phase 1 ended with.  Nothing is staged and nothing but
//   `out` (and `lse`) is written.
//   Pipeline, per 32-key subtile: the scores of the next subtile (8 MFMA) are
//   issued interleaved with the exponentials of the current one (VALU), then
//   the PV product of the current one (8 MFMA) interleaved with its row-sum
//   adds.  One MFMA operand is read from LDS per MFMA, eight MFMAs ahead of
//   its use (the current block's V operands, two transposing reads each: four
//   reads under each of the last four score MFMAs).  K/V tiles arrive by direct global->LDS loads three
//   tiles ahead into rings of four buffers, issued between the PV MFMAs (a
//   steady tile is branch-free), one barrier per 64-key tile.  The
//   K tile is XOR-swizzled at 16-byte granularity (applied on the global
//   address side of the copy) so that the 16 lanes of one ds_read_b128 phase
//   hit 16 different bank groups.
#pragma once
#include <type_traits>

#include "ifx_launch.hpp"
#include "ifx_types.hpp"

namespace ifx {

constexpr int BF_D = 128;
constexpr int BF_WAVES = 8;
constexpr int BF_BM = 32 * BF_WAVES;  // 256 query rows per workgroup
static_assert(BF_BM == 256 && BF_WAVES == 8, "ifx_launch.hpp deals query rows to workgroups of 8 wavefronts");
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
// log2 units: a raised reference lies this far above the largest score seen.  Larger values mean
// fewer raises, but a query dominated by one key then more often meets that key with a weight
// that is not a power of two, i.e. not exact in bf16 (2^-9 relative on the output; with 31 a
// peaked case went over the 2e-2 gate on outputs above 4, with 7 the dominant key of such a row
// nearly always is the one that raised the reference, weight 2^-7 exactly)
constexpr float BF_HEADROOM = 7.0f;
// the same where the row sum is taken from the rounded weights (see softmax_running_exact): there a
// weight need not be a power of two to cancel, and raises can be made rare
constexpr float BF_HEADROOM_EXACT = 31.0f;
constexpr float BF_BOUND_LIMIT = 50.0f;                    // log2 units; 2^-100 is still a normal bf16 / fp32

struct attn_bf16_args {
    const __bf16 *q;    // [n, H, 128]
    const unsigned char *kc;  // layer K region [H][k_tokens][128], bf16 or (FP8 instantiation) E4M3 codes
    const unsigned char *vt;  // layer V region, granules [H][v_tokens/8][128][8], likewise
    const __bf16 *kb;   // current block's K [n, H, 128], or nullptr when nb == 0
    const __bf16 *vb;   // current block's V [n, H, 128]
    __bf16 *out;        // [n, H, 128]
    float *lse;         // [n, H] natural-log sum of exp of the scaled scores, or nullptr
    int n, H;           // queries (= tokens of a block), heads
    int C, nb;          // cached keys (phase 1), keys of the current block (phase 2: n or 0); C + nb > 0
    ifx_key_blocks blocks;  // table instantiation only: where the n keys of each selected cached block live
    int64_t k_tokens, v_tokens;
    float scale_log2;   // softmax scale * log2(e)
    const uint32_t *knorm;  // [H][cap_blocks][parts]: float bits of max |k|^2 over a part of the block in that slot
    int resident_blocks, cap_blocks, parts;
    attn_shape shape;   // workgroup -> (head, query rows), see ifx_launch.hpp
};

typedef __attribute__((address_space(3))) void *lptr_t;
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 *lds_s16x4_ptr;

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

// "finite" as an integer test on the bit pattern (the library is built with -fno-honor-nans, under
// which a floating-point comparison against NaN may be folded away)
__device__ __forceinline__ bool finite_bits(float x) { return (__builtin_bit_cast(unsigned, x) & 0x7f800000u) != 0x7f800000u; }

#define IFX_INLINE __attribute__((always_inline))

// How a phase takes its softmax.  fixed: against the norm bound, no maximum kept.  running: against
// a reference raised when a score comes out above it; the row sum adds up the fp32 exponentials.
// running_exact: the same, but the row sum adds up the exponentials as rounded to bf16, i.e. exactly
// the weights the PV product uses: a row dominated by one key then comes out as that key's V row
// whatever the key's weight (with the unrounded sum numerator and denominator differ by up to
// 2^-9 there, which on outputs above 4, where bf16 is spaced 2^-5, can cost a whole unit in the
// last place).  16 more VALU instructions per subtile; used by the wavefronts whose scores are
// not bounded, which are the ones that meet such rows; their raises use the larger headroom.
struct softmax_fixed {
    static constexpr bool value = true, exact = false;
};
struct softmax_running {
    static constexpr bool value = false, exact = false;
};
struct softmax_running_exact {
    static constexpr bool value = false, exact = true;
};

// Where a phase's keys come from.
struct src_cache {
    static constexpr bool blk = false;
};
struct src_block {
    static constexpr bool blk = true;
};

// SEG == false: the cached keys are the physical tokens [0, C) of the head's regions (resident
// blocks in slot order).  SEG == true: they are a list of up to IFX_MAX_KEY_BLOCKS blocks of n
// physical tokens each (a caller-given selection of resident blocks in any order, or a ring that
// has wrapped); the tile copies then look their block up (scalar arithmetic), everything else is
// the same code.  The current block (nb keys, when given) follows in both.
// FP8: the cache holds E4M3 codes, one byte per element in the same two layouts.  A tile's codes
// are loaded into registers a tile ahead, widened (exactly) to bf16 and written into the same LDS
// tile rings the bf16 cache's tiles are copied into; everything downstream is the same code and
// the same arithmetic.  The current block is bf16 either way.
template <bool SEG, bool FP8 = false>
__global__ __launch_bounds__(BF_THREADS, 1) void attn_bf16_kernel(const attn_bf16_args a)
{
    constexpr int KEYB = FP8 ? BF_D : BF_D * 2;  // bytes of a cached key row, and of a key's share of its V granule
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    const attn_item item = attn_item_of(a.shape, blockIdx.x);
    if (item.waves == 0) return;
    const int head = item.head;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lq = lane & 31, lh = lane >> 5;
    const int n = a.n, H = a.H;
    const float c2 = a.scale_log2;

    // ---- Q: B operand of S^T = K Q^T; lane = query lq, d = 16 s + 8 lh + [0,8)
    const int waves_here = item.waves;  // wavefronts of this workgroup that hold rows
    const int qi = item.row0 + wave * 32 + lq;
    const int qi_c = qi < n ? qi : n - 1;
    bf16x8 Q[8];
    {
        const bf16x8 *qp = reinterpret_cast<const bf16x8 *>(a.q + ((int64_t)qi_c * H + head) * BF_D);
#pragma unroll
        for (int s = 0; s < 8; ++s) Q[s] = qp[2 * s + lh];
    }

    // ---- Cauchy-Schwarz bound on this query's scaled scores against the cached keys (log2 units)
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
        // the resident slots are a prefix, so the head's entries to look at are one run of words
        uint32_t kbits = 0u;  // non-negative floats (and +inf, NaN above them) order like their bit patterns
        const uint32_t *kn = a.knorm + (int64_t)head * a.cap_blocks * a.parts;
        for (int e = lane; e < a.resident_blocks * a.parts; e += 64) kbits = kn[e] > kbits ? kn[e] : kbits;
#pragma unroll
        for (int sh = 32; sh >= 1; sh >>= 1) {
            const uint32_t o = (uint32_t)__shfl_xor((int)kbits, sh);
            kbits = o > kbits ? o : kbits;
        }
        m_bound = sqrtf(q2 * __builtin_bit_cast(float, kbits)) * c2 * 1.001f + 1e-6f;
    }
    // (0 * inf, an overflowed norm or a NaN key give a bound that is not finite: running maximum;
    // so does a call without cached keys, where the bound says nothing about the scores to come)
    const bool bounded = a.C > 0 && __all(finite_bits(m_bound) && m_bound <= BF_BOUND_LIMIT);

    // ---- per-lane LDS read addresses
    // MFMA row rho = lq gets key 16*a1 + 8*hb + 4*a0 + b  (rho = 16*a1 + 8*a0 + 4*hb + b)
    const int pkey = (lq & 16) | ((lq & 4) << 1) | ((lq & 8) >> 1) | (lq & 3);
    const int kz = lh ^ (pkey & 15);
    int koff[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) koff[s] = BF_LDS_K0 + pkey * 256 + (((2 * s) ^ kz) << 4);
    const int voff = BF_LDS_V0 + lh * 2048 + lq * 16;
    // Row-major V tile of the current block ([64 keys][128 d], 16-byte chunk c of key row r stored
    // at chunk c ^ 4 (r & 3)): lane l of a transposing read supplies the address of 8 bytes of row
    // (l & 15) / 4 of a group of 4 key rows, d columns 16 (l / 16 & 1) + 4 (l & 3) .. + 3 of a
    // 32-wide d slab, and receives column l & 31 of those 4 rows.  The 4 rows of a group then lie
    // in 4 different quarters of the 64 banks.
    int vtoff[4];
    {
        const int l16 = lane & 15, g = lane >> 4;
        const int base = BF_LDS_V0 + (8 * (g >> 1) + (l16 >> 2)) * 256 + (2 * (g & 1) + ((l16 & 3) >> 1)) * 16 + 8 * (l16 & 1);
#pragma unroll
        for (int sl = 0; sl < 4; ++sl) vtoff[sl] = base + ((sl ^ (l16 >> 2)) << 6);
    }

    // ---- global -> LDS copy roles: 2 K chunks and 2 V chunks of 16 bytes per lane per tile.
    // LDS slot c = tid + BF_THREADS x (16 bytes each).  K: slot (key = c >> 4, pos = c & 15) receives
    // the key's chunk pos ^ (key & 15).  V granules: slot c receives chunk c of the contiguous tile.
    // V rows of the current block: slot (key, pos) receives the key's chunk pos ^ 4 (key & 3).
    const unsigned char *kc_head = a.kc + (int64_t)head * a.k_tokens * KEYB;
    const unsigned char *vt_head = a.vt + (int64_t)head * a.v_tokens * KEYB;
    const int krow = tid >> 4;                           // + BF_XROWS x
    const int kchunk = ((tid & 15) ^ (krow & 15)) << 4;  // byte offset inside the key row
    const int vchunk = ((tid & 15) ^ ((krow & 3) << 2)) << 4;
    // Buffer descriptors (raw, byte-addressed): reads past num_records return zero and touch no
    // memory, so the rows of a partial last tile need no clamping and a load of a tile past the
    // last one is harmless.  Lane offsets are 32-bit, tile offsets are scalars.  Cached tokens: key
    // row j and key j's share of its V granule both start at byte 256 j of the head's region.
    const __amdgpu_buffer_rsrc_t rs_k = __builtin_amdgcn_make_buffer_rsrc(
        (void *)kc_head, 0, SEG ? (int)(a.k_tokens * KEYB) : a.C * KEYB, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_v = __builtin_amdgcn_make_buffer_rsrc(
        (void *)vt_head, 0, SEG ? (int)(a.v_tokens * KEYB) : a.C * KEYB, 0x00020000);
    // Current block, [n, H, 128] where the caller has it: the head's rows are H * 256 bytes apart
    // and the last one ends at ((nb - 1) H + 1) * 256.
    const int row_pitch = H * (BF_D * 2);
    const int blk_bytes = a.nb > 0 ? (a.nb - 1) * row_pitch + BF_D * 2 : 0;
    const __amdgpu_buffer_rsrc_t rs_kb =
        __builtin_amdgcn_make_buffer_rsrc((void *)(a.kb + (int64_t)head * BF_D), 0, blk_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_vb =
        __builtin_amdgcn_make_buffer_rsrc((void *)(a.vb + (int64_t)head * BF_D), 0, blk_bytes, 0x00020000);
    const int vk_lane = krow * (BF_D * 2) + kchunk;
    const int vv_lane = tid * 16;
    const int bk_lane = krow * row_pitch + kchunk;
    const int bv_lane = krow * row_pitch + vchunk;
    // Selected keys.  Blocks are multiples of 8 tokens and a wavefront's share of a tile's copies
    // is 8 consecutive key rows (K) and the granule of the same 8 keys (V), aligned, so the block
    // they come from is the same for the whole wavefront and for all of them: the lookup is
    // scalar (block index by a multiply-high, its offset by a lane read of the table kept in one
    // register) and goes into the scalar offset, like the tile offset.  No memory access: an
    // indexed load of the table would wait for every outstanding tile copy.
    // The register holds, for up to IFX_MAX_KEY_BLOCKS entries at a time (a "segment" of the list,
    // whose keys are numbered from 0), the byte offset between key i * n of the segment and the
    // first token of entry i, and 2^30 in the lanes behind the last entry: block_tokens divides
    // the key count, so a key is past the end exactly when its block index is, and its copy then
    // starts beyond any region (at most 2^30 bytes) and reads as zero.
    int tab = 0;
    auto load_segment = [&](int base, int cnt) IFX_INLINE {
        // (two plain indexed reads, of the device list or of the kernel arguments: a pointer chosen
        // between the two would make the compiler copy the argument array to the stack)
        int first = 0;
        if (a.blocks.list != nullptr) {
            if (lane < cnt) first = a.blocks.list[base + lane];
        } else {
            first = a.blocks.first[lane];
        }
        tab = lane < cnt ? (first - lane * n) * KEYB : (1 << 30);
    };
    const unsigned blk_magic = SEG ? a.blocks.magic : 0u;
    auto key_offset = [&](int j) IFX_INLINE -> int {  // scalar byte offset of key row / granule j in the head's region
        const int p = __builtin_amdgcn_readfirstlane((int)__umulhi((unsigned)j, blk_magic));  // j / n
        return j * KEYB + __builtin_amdgcn_readlane(tab, p < 63 ? p : 63);
    };

    // Table instantiation: a wavefront copies the 8 key rows 8 wave .. 8 wave + 7 of a K tile (4 per
    // instruction) and granule `wave` of a V tile (half per instruction): 8 consecutive keys, aligned,
    // hence one block and one lookup for all four instructions, which differ by 1 KiB steps.
    // (The scalar offset must not go negative: it carries the wavefront's own first row / granule,
    // the lane offset only what is left inside those.)
    int vk_lane_seg[BF_NX];
#pragma unroll
    for (int x = 0; x < BF_NX; ++x) {
        const int r = 8 * wave + 4 * x + (lane >> 4);  // key row of the tile this lane copies a chunk of
        vk_lane_seg[x] = (lane >> 4) * (BF_D * 2) + (((lane & 15) ^ (r & 15)) << 4);
    }
    const int vv_lane_seg = lane * 16;
    // Scalar offsets of a tile's BF_NX K (V) copy instructions, and the copies themselves.  Two
    // steps, because with the block table an offset is a chain of a dozen scalar instructions: the
    // pipelined loop works them out a phase ahead of the copies, under other MFMAs.
    auto k_offs = [&](auto src, int j0) IFX_INLINE -> tile_offs {
        tile_offs t;
#pragma unroll
        for (int x = 0; x < BF_NX; ++x) {
            if constexpr (decltype(src)::blk) {
                t.s[x] = (j0 + x * BF_XROWS) * row_pitch;
            } else if constexpr (SEG) {
                if (x == 0)
                    t.s[0] = key_offset(j0 + 8 * wave);  // first of this wavefront's 8 key rows
                else
                    t.s[x] = t.s[0] + x * 1024;
            } else {
                t.s[x] = (j0 + x * BF_XROWS) * (BF_D * 2);
            }
        }
        return t;
    };
    auto v_offs = [&](auto src, int j0) IFX_INLINE -> tile_offs {
        tile_offs t;
#pragma unroll
        for (int x = 0; x < BF_NX; ++x) {
            if constexpr (decltype(src)::blk) {
                t.s[x] = (j0 + x * BF_XROWS) * row_pitch;
            } else if constexpr (SEG) {
                if (x == 0)
                    t.s[0] = key_offset(j0 + 8 * wave);  // first key of this wavefront's granule
                else
                    t.s[x] = t.s[0] + x * 1024;
            } else {
                t.s[x] = j0 * (BF_D * 2) + x * BF_XBYTES;
            }
        }
        return t;
    };
    auto issue_k_at = [&](auto src, const tile_offs &t, int buf) IFX_INLINE {
        unsigned char *dst = lds + BF_LDS_K0 + buf * BF_TILE_BYTES + wave * 1024;
        unsigned char *dst_seg = lds + BF_LDS_K0 + buf * BF_TILE_BYTES + wave * 2048;
#pragma unroll
        for (int x = 0; x < BF_NX; ++x) {
            if constexpr (decltype(src)::blk)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_kb, (lptr_t)(dst + x * BF_XBYTES), 16, bk_lane, t.s[x], 0, 0);
            else if constexpr (SEG)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_k, (lptr_t)(dst_seg + x * 1024), 16, vk_lane_seg[x], t.s[x], 0, 0);
            else
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_k, (lptr_t)(dst + x * BF_XBYTES), 16, vk_lane, t.s[x], 0, 0);
        }
    };
    auto issue_v_at = [&](auto src, const tile_offs &t, int buf) IFX_INLINE {
        unsigned char *dst = lds + BF_LDS_V0 + buf * BF_TILE_BYTES + wave * 1024;
        unsigned char *dst_seg = lds + BF_LDS_V0 + buf * BF_TILE_BYTES + wave * 2048;
#pragma unroll
        for (int x = 0; x < BF_NX; ++x) {
            if constexpr (decltype(src)::blk)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_vb, (lptr_t)(dst + x * BF_XBYTES), 16, bv_lane, t.s[x], 0, 0);
            else if constexpr (SEG)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_v, (lptr_t)(dst_seg + x * 1024), 16, vv_lane_seg, t.s[x], 0, 0);
            else
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_v, (lptr_t)(dst + x * BF_XBYTES), 16, vv_lane, t.s[x], 0, 0);
        }
    };
    auto issue_k = [&](auto src, int j0, int buf) IFX_INLINE { issue_k_at(src, k_offs(src, j0), buf); };
    auto issue_v = [&](auto src, int j0, int buf) IFX_INLINE { issue_v_at(src, v_offs(src, j0), buf); };

    // FP8 cache tiles: 64 keys x 128 codes of K and 8 granules x 1 KiB of V are 8 KiB each and
    // contiguous, 16 bytes per lane.  Loaded into one of two register sets (by tile parity), a tile
    // before they are widened into ring slot `buf`: lane t holds K codes of key row t / 8,
    // dimensions 16 (t % 8) .. + 15 (two 16-byte chunks of the row, swizzled like the copies'), and V
    // codes of granule t / 64, dimensions 2 (t % 64) and + 1 (32 contiguous bytes of the granule).
    typedef uint32_t raw_u32x4 __attribute__((__vector_size__(16)));
    raw_u32x4 R8k[2], R8v[2];
    auto fp8_load = [&](int j0, int set) IFX_INLINE {
        int so, lo;
        if constexpr (SEG) {
            so = key_offset(j0 + 8 * wave);  // this wavefront's 8 key rows / its granule lie in one block
            lo = lane * 16;
        } else {
            so = j0 * KEYB;
            lo = tid * 16;
        }
        R8k[set] = __builtin_amdgcn_raw_buffer_load_b128(rs_k, lo, so, 0);
        R8v[set] = __builtin_amdgcn_raw_buffer_load_b128(rs_v, lo, so, 0);
    };
    auto widen16 = [&](const raw_u32x4 &c, u32x4 &lo8, u32x4 &hi8) IFX_INLINE {
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
#pragma unroll
        for (int w = 0; w < 2; ++w) {
            lo8[2 * w] = __builtin_bit_cast(uint32_t, (bf16x2)__builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((int)c[w], 1.0f, false));
            lo8[2 * w + 1] = __builtin_bit_cast(uint32_t, (bf16x2)__builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((int)c[w], 1.0f, true));
            hi8[2 * w] = __builtin_bit_cast(uint32_t, (bf16x2)__builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((int)c[2 + w], 1.0f, false));
            hi8[2 * w + 1] = __builtin_bit_cast(uint32_t, (bf16x2)__builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((int)c[2 + w], 1.0f, true));
        }
    };
    const int k8_row = tid >> 3, k8_c = (tid & 7) * 2;
    const int k8_at = BF_LDS_K0 + k8_row * 256, k8_z = k8_row & 15;
    const int v8_at = BF_LDS_V0 + (tid >> 6) * 2048 + (tid & 63) * 32;
    auto fp8_store = [&](int set, int buf) IFX_INLINE {
        u32x4 a8, b8;
        widen16(R8k[set], a8, b8);
        *reinterpret_cast<u32x4 *>(lds + buf * BF_TILE_BYTES + k8_at + ((k8_c ^ k8_z) << 4)) = a8;
        *reinterpret_cast<u32x4 *>(lds + buf * BF_TILE_BYTES + k8_at + (((k8_c + 1) ^ k8_z) << 4)) = b8;
        widen16(R8v[set], a8, b8);
        *reinterpret_cast<u32x4 *>(lds + buf * BF_TILE_BYTES + v8_at) = a8;
        *reinterpret_cast<u32x4 *>(lds + buf * BF_TILE_BYTES + v8_at + 16) = b8;
    };
    // every LDS write of this wavefront done, then the barrier (the widened tiles are plain stores)
    auto wait_lds_and_sync = [&]() IFX_INLINE {
        __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0); vmcnt and expcnt at their no-wait maxima
        __builtin_amdgcn_s_barrier();
    };

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
    // The eight V operands (key step t, d slab sl) of the subtile whose V data starts at voffs:
    // one 16-byte read of a granule each, or (current block, row-major) two transposing reads of
    // 4 keys each.
    auto v_fetch = [&](auto src, int voffs, bf16x8 (&A)[8]) IFX_INLINE {
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int o = 0; o < 4; ++o) {
                const int sl = 3 - o;
                if constexpr (decltype(src)::blk) {
                    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (lds_s16x4_ptr)(lptr_t)(lds + voffs + vtoff[sl] + (16 * t) * 256));
                    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (lds_s16x4_ptr)(lptr_t)(lds + voffs + vtoff[sl] + (16 * t + 4) * 256));
                    typedef short s16x8 __attribute__((ext_vector_type(8)));
                    const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    A[t * 4 + sl] = __builtin_bit_cast(bf16x8, both);
                } else {
                    A[t * 4 + sl] = *reinterpret_cast<const bf16x8 *>(lds + voffs + voff + t * 4096 + sl * 512);
                }
            }
    };
    // S^T = K Q^T; register r of S is key (subtile base) + 16 (r/8) + 8 lh + r%8.
    auto qk = [&](const bf16x8 (&A)[8], f32x16 &S) IFX_INLINE {
        f32x16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < 8; ++s) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[s], Q[s], acc, 0, 0, 0);
        S = acc;
    };

    // Largest scaled score of the subtile, per query (both halves).
    auto tile_max = [&](const f32x16 &S) IFX_INLINE -> float {
        // a shallow tree: the dependent chain is what a lone wavefront cannot hide
        const float a0 = fmaxf(fmaxf(S[0], S[1]), S[2]), a1 = fmaxf(fmaxf(S[3], S[4]), S[5]);
        const float a2 = fmaxf(fmaxf(S[6], S[7]), S[8]), a3 = fmaxf(fmaxf(S[9], S[10]), S[11]);
        const float a4 = fmaxf(fmaxf(S[12], S[13]), S[14]);
        const float b0 = fmaxf(fmaxf(a0, a1), a2), b1 = fmaxf(fmaxf(a3, a4), S[15]);
        return max_across_halves(fmaxf(b0, b1)) * c2;
    };
    // Running maximum: the exponentials are taken against a reference m_used that a query raises
    // only when one of its scores comes out above it, and then to BF_HEADROOM above that score:
    // the result is the same softmax (numerator and denominator carry the same factor), P stays
    // at or below 2^-7 until a score exceeds everything before it by 2^7, so few subtiles
    // rescale.  Here: raise where the subtile S demands it (always on a query's first subtile).
    auto raise_for = [&](const f32x16 &S, const float headroom) IFX_INLINE {
        const float m_tile = tile_max(S);
        const bool raise = m_tile > m_used;
        if (__builtin_expect(__any(raise), 0)) {  // rare: keep it off the fall-through path
            const float m_next = raise ? m_tile + headroom : m_used;
            const float alpha = __builtin_amdgcn_exp2f(m_used - m_next);  // 1 where unchanged, 0 at the start
#pragma unroll
            for (int e = 0; e < 4; ++e) l_acc[e] *= alpha;
#pragma unroll
            for (int sl = 0; sl < 4; ++sl)
#pragma unroll
                for (int r = 0; r < 16; ++r) O[sl][r] *= alpha;
            m_used = m_next;
        }
    };

    // E = exp2(S c2 - m) in fp32 and P = E in bf16 (P[t] = 8 consecutive keys).  The row sum is
    // taken from E with plain adds, placed under the PV MFMAs.  (Summing the bf16-rounded P with
    // v_dot2c_f32_bf16 halves the instruction count but that instruction stalls next to MFMAs:
    // 6 % slower.)  The sum runs over the unrounded values; the rounding of P is unbiased, so it
    // differs from the sum of what the PV product uses by a relative 2^-9 / sqrt(keys).
    auto exps = [&](const f32x16 &S, f32x16 &E, bf16x8 (&P)[2]) IFX_INLINE {
#pragma unroll
        for (int r = 0; r < 16; ++r) E[r] = __builtin_amdgcn_exp2f(fmaf(S[r], c2, -m_used));
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            f32x8 p;
#pragma unroll
            for (int e = 0; e < 8; ++e) p[e] = E[8 * t + e];
            P[t] = __builtin_convertvector(p, bf16x8);
        }
    };
    // E := P widened back to fp32 (a shift or a mask per value): what the PV product will use.
    auto as_rounded = [&](f32x16 &E, const bf16x8 (&P)[2]) IFX_INLINE {
#pragma unroll
        for (int r = 0; r < 16; ++r) E[r] = (float)P[r >> 3][r & 7];
    };
    // Does any of the lane's 16 values of P reach 2, i.e. did a score come out a whole unit above
    // the reference?  P >= 0, so that is "the top exponent bit is set somewhere": an OR over the
    // packed pairs and one mask (infinity, from a score 2^7 units above, has the bit set too).
    auto p_reaches_two = [&](const bf16x8 (&P)[2]) IFX_INLINE -> bool {
        const u32x4 a = __builtin_bit_cast(u32x4, P[0]), b = __builtin_bit_cast(u32x4, P[1]);
        const uint32_t o = (a[0] | a[1] | a[2]) | (a[3] | b[0] | b[1]) | (b[2] | b[3]);
        return (o & 0x40004000u) != 0u;
    };
    auto row_sum = [&](const f32x16 &E) IFX_INLINE {
#pragma unroll
        for (int r = 0; r < 16; ++r) l_acc[r & 3] += E[r];
    };

    // O^T += V^T P^T.
    auto pv = [&](const bf16x8 (&A)[8], const bf16x8 (&P)[2]) IFX_INLINE {
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int sl = 0; sl < 4; ++sl)
                O[sl] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[t * 4 + sl], P[t], O[sl], 0, 0, 0);
    };

    // Keys at or past the end of the phase never count.
    auto mask_keys = [&](f32x16 &S, int j_sub, int Lp) IFX_INLINE {
        if (j_sub + 32 > Lp) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int j = j_sub + 16 * (r >> 3) + 8 * lh + (r & 7);
                if (j >= Lp) S[r] = -INFINITY;
            }
        }
    };

    bf16x8 Kop[8];  // K operands of the subtile whose scores are computed next
    bf16x8 Vop[8];  // V operands of the current subtile

    // One pipelined step of 16 MFMAs, one LDS operand per MFMA, each read about eight MFMAs
    // ahead of its use.  Scores of the NEXT subtile (operands already in Kop) with the V operands of
    // the CURRENT subtile fetched meanwhile and its exponentials spread under them; then the PV
    // product of the current subtile with the K operands of the subtile AFTER the next fetched
    // meanwhile and the current subtile's row-sum adds.
    //   koffs_after: LDS offset of the subtile after the next; voffs_cur: offset of the current
    //   subtile's V data.  Only for subtiles that lie wholly inside the phase (no key masking).
    //   load_tag: which half of the tile three ahead this step brings in (0: K, 1: V), two
    //   global->LDS loads placed between the PV MFMAs; j_load / buf_load: its first key and ring slot.
    auto halfstep = [&](auto src, auto bounded_tag, auto load_tag, auto idle_tag, f32x16 &Scur, f32x16 &Snext,
                        int koffs_after, int voffs_cur, int j_load, int buf_load) IFX_INLINE {
        constexpr bool BOUNDED = decltype(bounded_tag)::value;
        constexpr bool EXACT = decltype(bounded_tag)::exact;
        constexpr float HEADROOM = EXACT ? BF_HEADROOM_EXACT : BF_HEADROOM;
        constexpr int V_READS = decltype(src)::blk ? 2 : 1;  // LDS reads per V operand
        bf16x8 P[2];
        f32x16 E;
        constexpr bool CODES = FP8 && !decltype(src)::blk;  // this phase's tiles come as E4M3 codes through registers
        tile_offs offs;
        if constexpr (!CODES) offs = decltype(load_tag)::value == 0 ? k_offs(src, j_load) : v_offs(src, j_load);  // for the copies of the PV phase
        if constexpr (decltype(idle_tag)::value) {
            // a wavefront without a query row: its share of the tile copies and nothing else
            if constexpr (CODES) {
                if constexpr (decltype(load_tag)::value == 0)
                    fp8_load(j_load, buf_load & 1);
                else
                    fp8_store((buf_load + 1) & 1, (buf_load + 3) & 3);
            } else if constexpr (decltype(load_tag)::value == 0) {
                issue_k_at(src, offs, buf_load);
            } else {
                issue_v_at(src, offs, buf_load);
            }
            return;
        }
        qk(Kop, Snext);
        v_fetch(src, voffs_cur, Vop);
        exps(Scur, E, P);
#pragma unroll
        for (int g = 0; g < 8; ++g) {  // score MFMAs: V operand reads, exponentials
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            // The V operands are first used eight MFMAs on.  Cached keys: one operand read per MFMA
            // from the first on.  Current block (two transposing reads per operand): under the last
            // four score MFMAs only, four reads apiece; measured 3 % faster on that phase.
            if constexpr (decltype(src)::blk) {
                if (g >= 4) __builtin_amdgcn_sched_group_barrier(0x100, 2 * V_READS, 0);
            } else {
                __builtin_amdgcn_sched_group_barrier(0x100, V_READS, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);
            __builtin_amdgcn_sched_group_barrier(0x400, 2, 0);
        }
        if constexpr (!BOUNDED) {
            // Running maximum, checked after the fact: the exponentials were taken against the
            // reference as it stood; only if one of them shows that a score lies above it, the
            // reference is raised from the scores (still in Scur) and the exponentials are redone.
            // Nothing of this subtile has reached the accumulators yet.
            if (__builtin_expect(__any(p_reaches_two(P)), 0)) {
                raise_for(Scur, HEADROOM);
                exps(Scur, E, P);
            }
        }
        // Wave priority: high while a wavefront is in its score phase (per MFMA 3 VALU and 2
        // transcendental instructions), low in its PV phase (per MFMA 2 VALU).  The two wavefronts
        // of a SIMD then settle into opposite phases: the one with the long instruction stream is
        // never held up, the other one's MFMAs fill the gaps.  (The instruction ends a scheduling
        // region, so each phase's instructions and its group sequence sit on their own side of it.)
        __builtin_amdgcn_s_setprio(0);
        if constexpr (CODES) {
            // first half of tile i: the codes of tile i + 3 start on their way into register set
            // (i + 3) % 2; second half: those of tile i + 2 (set i % 2, asked for a tile ago) are
            // widened into ring slot (i + 2) % 4, which tile i - 2 left free
            if constexpr (decltype(load_tag)::value == 0)
                fp8_load(j_load, buf_load & 1);
            else
                fp8_store((buf_load + 1) & 1, (buf_load + 3) & 3);
        } else if constexpr (decltype(load_tag)::value == 0) {
            issue_k_at(src, offs, buf_load);
        } else {
            issue_v_at(src, offs, buf_load);
        }
        pv(Vop, P);
        k_fetch(koffs_after, Kop);
        if constexpr (EXACT) as_rounded(E, P);  // (here, under the PV MFMAs: the score phase has no VALU slots to spare)
        row_sum(E);
        // (a step that widens a tile of codes: its 16 conversions and 4 LDS stores go under the first
        // PV MFMAs, so that the stores have landed when the tile's barrier asks for them)
        constexpr bool WIDENS = CODES && decltype(load_tag)::value == 1;
#pragma unroll
        for (int g = 0; g < 8; ++g) {  // PV MFMAs: K operand reads, row sum, the two loads
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            if (WIDENS && g < 4)
                __builtin_amdgcn_sched_group_barrier(0x002, EXACT ? 8 : 6, 0);
            else
                __builtin_amdgcn_sched_group_barrier(0x002, EXACT ? 4 : 2, 0);
            if (WIDENS && (g == 1 || g == 3)) __builtin_amdgcn_sched_group_barrier(0x200, 2, 0);
            if (g == 1 || g == 5) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
        if constexpr (BOUNDED) {
            // Never taken (n > 0).  Without a use of the row sum at the end of every step the
            // compiler moves all row-sum instructions of four tiles behind the last barrier of the
            // unrolled loop, where nothing hides them and the exponentials stay live meanwhile.
            // (The running maximum's check at the next step's phase boundary is such a use.)
            if (__builtin_expect(n < 0, 0)) {
#pragma unroll
                for (int e = 0; e < 4; ++e) l_acc[e] *= 2.0f;
            }
        }
        __builtin_amdgcn_s_setprio(1);
    };

    // One phase: the Lp > 0 keys of one source, tiles of 64, through the accumulators O, l_acc and
    // against m_used.  Entered and left with every wavefront of the workgroup past a barrier behind
    // its last LDS read, so the tile ring is free; all wavefronts meet the same number of barriers
    // (one behind the first tiles' arrival, one per tile) whichever softmax variant they run.
    //   idle_tag: a wavefront that was given no query rows.  It copies
    //   its share of every tile and meets every barrier (same loops, same counts) and skips the
    //   arithmetic: the other wavefronts of its workgroup need the tiles, nobody needs its MFMAs.
    auto phase = [&](auto src, auto bounded_tag, auto idle_tag, const int Lp) IFX_INLINE {
        constexpr bool BOUNDED = decltype(bounded_tag)::value;
        constexpr bool EXACT = decltype(bounded_tag)::exact;
        constexpr float HEADROOM = EXACT ? BF_HEADROOM_EXACT : BF_HEADROOM;
        constexpr bool IDLE = decltype(idle_tag)::value;
        constexpr bool CODES = FP8 && !decltype(src)::blk;
        const int T = (Lp + BF_BN - 1) / BF_BN;
        if constexpr (CODES) {
            // tiles 0 and 1 widened into their ring slots, the codes of tile 2 on their way
            fp8_load(0, 0);
            fp8_load(BF_BN, 1);
            fp8_store(0, 0);
            fp8_store(1, 1);
            fp8_load(2 * BF_BN, 0);
            wait_lds_and_sync();
        } else {
            // tiles 0, 1, 2 on their way into LDS
            issue_k(src, 0, 0);
            issue_v(src, 0, 0);
            if (T > 1) {
                issue_k(src, BF_BN, 1);
                issue_v(src, BF_BN, 1);
            }
            if (T > 2) {
                issue_k(src, 2 * BF_BN, 2);
                issue_v(src, 2 * BF_BN, 2);
            }
            wait_loads_and_sync<0>();
        }
        // scores and maximum of subtile (0,0)
        f32x16 Sa, Sb;
        if constexpr (!IDLE) {
            k_fetch(0, Kop);
            qk(Kop, Sa);
            if constexpr (!BOUNDED) {
                mask_keys(Sa, 0, Lp);
                raise_for(Sa, HEADROOM);
            }
            k_fetch(8192, Kop);  // subtile (0,1)
        }

        // Tile i: K(i) (second half), K(i+1) (first half) and V(i) are read; K(i+2), V(i+2) are
        // landing (issued during tile i-1, needed from tile i+1 on); K(i+3), V(i+3) are issued
        // during this tile into ring slot (i+3) % 4, whose last readers finished before the previous
        // barrier.  At the tile's end only the loads issued in this tile may still be in flight.
        // b = i % 4 is a compile-time constant in the unrolled steady loop; the tile has no branch.
        auto tile_steady = [&](int i, int b) IFX_INLINE {
            const int b1 = (b + 1) % 4, b3 = (b + 3) % 4;
            const int j3 = (i + 3) * BF_BN;  // past the last tile: the loads read as zero and touch no memory
            halfstep(src, bounded_tag, std::integral_constant<int, 0>{}, idle_tag, Sa, Sb, b1 * BF_TILE_BYTES,
                     b * BF_TILE_BYTES, j3, b3);
            halfstep(src, bounded_tag, std::integral_constant<int, 1>{}, idle_tag, Sb, Sa, b1 * BF_TILE_BYTES + 8192,
                     b * BF_TILE_BYTES + 8192, j3, b3);
            if constexpr (CODES)
                wait_lds_and_sync();
            else
                wait_loads_and_sync<2 * BF_NX>();
        };
        // Steady tiles take no key mask: every complete tile is one; scores computed past the last
        // tile are never used.  What is left (the partial last tile) goes through the masked loop
        // below.  Keys past Lp must not be left to their zero K rows: when every real score of a row
        // is far below the reference, 2^(0 - reference) per padded key would swamp the row sum.
        const int n_steady = Lp / BF_BN;
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
        // The last tile, one 32-key subtile at a time without software pipelining: key mask and
        // (running maximum) reference check, exponentials and PV of the current subtile, then the
        // scores of the next.  Sa holds the scores of subtile (i, 0), not yet masked or checked
        // (unless i == 0 on the running maximum, where doing it again changes nothing).
        {
            const int n_sub = (Lp + 31) >> 5;  // subtiles holding at least one key
            if constexpr (!IDLE) {
                if (2 * i < n_sub) {
                    mask_keys(Sa, i * BF_BN, Lp);
                    if constexpr (!BOUNDED) raise_for(Sa, HEADROOM);
                }
            }
#pragma unroll 1
            for (int sg = 2 * i; sg < n_sub; ++sg) {
                const int ti = sg >> 1, u = sg & 1;
                if constexpr (!CODES) {
                    if (u == 0 && ti + 3 < T) {
                        issue_k(src, (ti + 3) * BF_BN, (ti + 3) & 3);
                        issue_v(src, (ti + 3) * BF_BN, (ti + 3) & 3);
                    }
                }
                if constexpr (!IDLE) {
                    bf16x8 P[2];
                    f32x16 E;
                    v_fetch(src, (ti & 3) * BF_TILE_BYTES + u * 8192, Vop);
                    exps(Sa, E, P);
                    if constexpr (EXACT) as_rounded(E, P);
                    row_sum(E);
                    pv(Vop, P);
                    if (sg + 1 < n_sub) {
                        const int tn = (sg + 1) >> 1, un = (sg + 1) & 1;
                        k_fetch((tn & 3) * BF_TILE_BYTES + un * 8192, Kop);
                        qk(Kop, Sa);
                        mask_keys(Sa, (sg + 1) * 32, Lp);
                        if constexpr (!BOUNDED) raise_for(Sa, HEADROOM);
                    }
                }
                if (u == 1 || sg + 1 == n_sub) wait_loads_and_sync<0>();  // one barrier per tile on every path
            }
        }
    };

    // ---- phase 1: the cached keys (a selection: one pass per segment of the list)
    auto cached_keys = [&](auto bounded_tag, auto idle_tag) IFX_INLINE {
        if constexpr (SEG) {
            const int total = a.blocks.count;
#pragma unroll 1
            for (int base = 0; base < total; base += IFX_MAX_KEY_BLOCKS) {
                const int cnt = total - base < IFX_MAX_KEY_BLOCKS ? total - base : IFX_MAX_KEY_BLOCKS;
                load_segment(base, cnt);
                phase(src_cache{}, bounded_tag, idle_tag, cnt * n);
            }
        } else {
            phase(src_cache{}, bounded_tag, idle_tag, a.C);
        }
    };
    // A wavefront that holds no query row only helps with the copies.
    if (wave >= waves_here) {
        if (a.C > 0) cached_keys(softmax_running{}, std::true_type{});
        if (a.nb > 0) phase(src_block{}, softmax_running{}, std::true_type{}, a.nb);
        return;
    }
    // A wavefront whose scores the norm bound covers: fixed maximum over the cached keys, then the
    // current block (no key norm is known for it) on the running maximum, starting from the bound,
    // which such rows hardly ever exceed.  Any other wavefront: the running maximum with exact row
    // sums throughout.
    if (bounded) {
        if (a.C > 0) {
            m_used = m_bound;
            cached_keys(softmax_fixed{}, std::false_type{});
        }
        if (a.nb > 0) phase(src_block{}, softmax_running{}, std::false_type{}, a.nb);
    } else {
        if (a.C > 0) cached_keys(softmax_running_exact{}, std::false_type{});
        if (a.nb > 0) phase(src_block{}, softmax_running_exact{}, std::false_type{}, a.nb);
    }

    // ---- epilogue: out[q, d] = O^T[d, q] / l;  register r of O[sl] is d = 32 sl + 8 (r/4) + 4 lh + r%4
    const float l_part = (l_acc[0] + l_acc[1]) + (l_acc[2] + l_acc[3]);
    const float l_tot = l_part + __shfl_xor(l_part, 32);
    const float inv = 1.0f / l_tot;
    if (a.lse != nullptr && lh == 0 && qi < n)  // ln sum_j exp(scale s_ij) = ln 2 * (m + log2 l)
        a.lse[(int64_t)qi * H + head] = (m_used + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f;
    // A lane holds 4 consecutive d per (sl, g), its partner lane ^ 32 the 4 that follow.  The two
    // trade halves (the lower lane gives its g-odd group for the partner's g-even one), so that
    // each stores 8 consecutive d, 16 bytes: v_permlane32_swap puts lanes 0..31 of its second
    // operand into lanes 32..63 of the first and the other way round.  (Partners share the query
    // row, so both or neither are past the end; the exchange itself runs in all lanes.)
    __bf16 *op = a.out + ((int64_t)qi_c * H + head) * BF_D;
#pragma unroll
    for (int sl = 0; sl < 4; ++sl)
#pragma unroll
        for (int gp = 0; gp < 2; ++gp) {
            f32x4 e4, o4;
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                e4[b] = O[sl][8 * gp + b] * inv;
                o4[b] = O[sl][8 * gp + 4 + b] * inv;
            }
            typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
            const u32x2 even = __builtin_bit_cast(u32x2, __builtin_convertvector(e4, bf16x4));
            const u32x2 odd = __builtin_bit_cast(u32x2, __builtin_convertvector(o4, bf16x4));
            u32x4 w;
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                auto r = __builtin_amdgcn_permlane32_swap(even[c], odd[c], false, false);
                w[c] = r[0];
                w[2 + c] = r[1];
            }
            if (qi < n) *reinterpret_cast<u32x4 *>(op + 32 * sl + 8 * (2 * gp + lh)) = w;
        }
}

}  // namespace ifx
