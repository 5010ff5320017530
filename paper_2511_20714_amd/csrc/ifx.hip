// C-ABI of the ifx library: host-side cache object, argument checks and kernel
// launches.  See include/ifx.h for the contract of every entry point.
#include "../../include/ifx.h"

#include <hip/hip_runtime.h>

#include <climits>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <numeric>
#include <utility>
#include <vector>

#include "ifx_attn_bf16.hpp"
#include "ifx_merge.hpp"
#include "ifx_attn_f32.hpp"
#include "ifx_commit.hpp"
#include "ifx_ring.hpp"

static_assert(IFX_MAX_KEY_BLOCKS == IFX_MAX_LISTED_BLOCKS, "block table size and its documented limit");

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

#define IFX_HIP(expr)                                                                          \
    do {                                                                                       \
        hipError_t e_ = (expr);                                                                \
        if (e_ != hipSuccess) return fail(IFX_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }


struct event_pair {
    hipEvent_t start, stop;
};

}  // namespace

// A piece of physical memory mapped into a reserved address range.
struct vmm_chunk {
    hipMemGenericAllocationHandle_t handle;
    unsigned char *va;
    size_t bytes;
};

struct ifx_kv_cache {
    int layers = 0, heads = 0, head_dim = 0;
    int64_t capacity_tokens = 0;
    int64_t reserve_tokens = 0;  // ifx_kv_cache_reserve: the capacity may grow to this in place (0: no reservation)
    bool configured = false;
    int64_t n = 0;  // block tokens
    int dtype = -1;
    float scale = 0.f;
    int64_t cap_blocks = 0;
    int64_t stride_blocks = 0;  // blocks the side tables are laid out for: cap_blocks, or the reservation in blocks
    int device = -1;
    size_t elem = 0;
    int64_t k_tokens = 0, v_tokens = 0;  // tokens between two heads' regions (the capacity, or the reservation)
    size_t k_layer_bytes = 0, v_layer_bytes = 0;
    // K and V of all layers: one hipMalloc, or (reserved) an address range of its own into which
    // physical memory is mapped piece by piece as the capacity grows: behind every head's
    // resident tokens lies address space without memory
    unsigned char *slab = nullptr;
    size_t va_bytes = 0, gran = 0;  // (gran: the device's mapping granularity, which must divide the piece size)
    std::vector<vmm_chunk> chunks;
    void *aux = nullptr;        // one side allocation: knorm, then blk_list
    uint32_t *knorm = nullptr;  // bf16: [layers][heads][stride_blocks][parts] float bits of max |k|^2 (see ifx_commit.hpp)
    int parts = 0;              // bf16: workgroups per head that copy K rows in a commit
    int *blk_list = nullptr;    // [layers][stride_blocks]: first tokens of a selection too long for the kernel arguments,
                                // written by the attention call that uses it, in stream order
    std::vector<ifx_ring> rings;
    bool profile = false;
    std::vector<event_pair> attn_events, commit_events;

    bool mfma() const { return dtype == IFX_BF16 || dtype == IFX_FP8_E4M3; }  // bf16 tensors at the boundary, MFMA kernel
    size_t io_elem() const { return dtype == IFX_F32 ? 4 : 2; }             // bytes of an element of the caller's tensors
    unsigned char *k_of(int layer) const { return slab + (size_t)layer * (k_layer_bytes + v_layer_bytes); }
    unsigned char *v_of(int layer) const { return k_of(layer) + k_layer_bytes; }
    int *list_of(int layer) const { return blk_list + (size_t)layer * (size_t)stride_blocks; }
    uint32_t *knorm_of(int layer) const { return knorm + (size_t)layer * (size_t)heads * (size_t)stride_blocks * (size_t)parts; }
};

namespace {

int check_call(const ifx_kv_cache *c, int layer)
{
    if (!c) return fail(IFX_ERR_INVALID_ARG, "cache is NULL");
    if (!c->configured) return fail(IFX_ERR_NOT_CONFIGURED, "ifx_kv_cache_configure has not been called");
    if (layer < 0 || layer >= c->layers) return fail(IFX_ERR_INVALID_ARG, "layer %d out of range [0,%d)", layer, c->layers);
    return IFX_OK;
}

int check_ptr(const void *p, const char *name)
{
    if (!p) return fail(IFX_ERR_INVALID_ARG, "%s is NULL", name);
    if (!aligned16(p)) return fail(IFX_ERR_INVALID_ARG, "%s is not 16-byte aligned", name);
    return IFX_OK;
}

int grid_for(int64_t items, int per_block = 256, int max_blocks = 256 * 16)
{
    int64_t b = (items + per_block - 1) / per_block;
    if (b < 1) b = 1;
    if (b > max_blocks) b = max_blocks;
    return (int)b;
}

// One timing sample (a pair of HIP events around what a call enqueues), taken only while
// profiling is on and the stream is not being captured (an event recorded into a graph has no
// time of its own to read back).  A sample that is not closed by end() - the call failed in
// between - is dropped again, so the list only ever holds pairs whose stop event was recorded.
constexpr size_t MAX_TIMING_SAMPLES = 1u << 20;

class timing_sample {
  public:
    timing_sample(ifx_kv_cache *c, std::vector<event_pair> &v, hipStream_t s) : c_(c), v_(v), s_(s) {}
    timing_sample(const timing_sample &) = delete;
    timing_sample &operator=(const timing_sample &) = delete;
    ~timing_sample()
    {
        if (armed_) drop();
    }
    int begin();
    int end()
    {
        if (!armed_) return IFX_OK;
        const hipError_t e = hipEventRecord(v_.back().stop, s_);
        if (e == hipSuccess) {
            armed_ = false;
            return IFX_OK;
        }
        drop();
        return fail(IFX_ERR_HIP, "profiling events: %s", hipGetErrorString(e));
    }

  private:
    void drop()
    {
        (void)hipEventDestroy(v_.back().start);
        (void)hipEventDestroy(v_.back().stop);
        v_.pop_back();
        armed_ = false;
    }
    ifx_kv_cache *c_;
    std::vector<event_pair> &v_;
    hipStream_t s_;
    bool armed_ = false;
};

int timing_sample::begin()
{
    if (!c_->profile) return IFX_OK;
    if (v_.size() >= MAX_TIMING_SAMPLES) return IFX_OK;  // never read back: stop collecting rather than grow for ever
    hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s_, &capturing) != hipSuccess) (void)hipGetLastError();
    if (capturing != hipStreamCaptureStatusNone) return IFX_OK;
    event_pair ev{nullptr, nullptr};
    IFX_HIP(hipEventCreate(&ev.start));
    hipError_t e = hipEventCreate(&ev.stop);
    if (e == hipSuccess) e = hipEventRecord(ev.start, s_);
    bool stored = false;
    if (e == hipSuccess) {
        try {
            v_.push_back(ev);
            stored = true;
        } catch (...) {
        }
    }
    if (!stored) {
        (void)hipEventDestroy(ev.start);
        if (ev.stop) (void)hipEventDestroy(ev.stop);
        return e != hipSuccess ? fail(IFX_ERR_HIP, "profiling events: %s", hipGetErrorString(e))
                               : fail(IFX_ERR_OOM, "profiling events: host allocation failed");
    }
    armed_ = true;
    return IFX_OK;
}

// fp32: enqueue the copy of one block's V into the layer's private layout at token offset tok0.
int launch_store_v(const ifx_kv_cache *c, int layer, const void *v_blk, int64_t tok0, hipStream_t s)
{
    const int64_t n = c->n;
    const int H = c->heads;
    const int cpr = (int)(c->head_dim * c->elem / 16);
    hipLaunchKernelGGL(ifx::rows_to_heads_kernel, dim3(grid_for(n * H * cpr)), dim3(256), 0, s, (const u32x4 *)v_blk,
                       (u32x4 *)c->v_of(layer), n, H, cpr, c->v_tokens, tok0);
    IFX_HIP(hipGetLastError());
    return IFX_OK;
}

// bf16, one launch for the blocks of layers [first_layer, first_layer + n_layers), n_layers <=
// COMMIT_MAX_LAYERS: each layer's K rows copied to its next slot with the block's largest key norms
// recorded in the slot's knorm entries, its V turned into granules there.
int launch_store_blocks_bf16(ifx_kv_cache *c, int first_layer, int n_layers, const void *const *k_blks, const void *const *v_blks,
                             hipStream_t s)
{
    const int64_t n = c->n;
    const int H = c->heads, D = c->head_dim;
    // V: a wavefront turns half a granule of one head (8 tokens x 64 dimensions) at a time, 4 in
    // flight: 16 per workgroup and round
    const int v_blocks = grid_for((n / 8) * H * (D / 64), 16, 2048);
    ifx::commit_layers args = {};
    for (int i = 0; i < n_layers; ++i) {
        const int layer = first_layer + i;
        const int64_t slot = c->rings[(size_t)layer].next_slot();
        args.l[i] = ifx::commit_layer{k_blks[i], v_blks[i], c->k_of(layer), c->v_of(layer), c->knorm_of(layer), slot * n, (int)slot};
    }
    const dim3 grid((unsigned)(H * c->parts + v_blocks), (unsigned)n_layers);
    if (c->dtype == IFX_FP8_E4M3)
        hipLaunchKernelGGL((ifx::store_block_bf16_kernel<4, true>), grid, dim3(256), 0, s, args, n, H, c->k_tokens, c->v_tokens, c->parts,
                           (int)c->stride_blocks);
    else
        hipLaunchKernelGGL((ifx::store_block_bf16_kernel<4, false>), grid, dim3(256), 0, s, args, n, H, c->k_tokens, c->v_tokens, c->parts,
                           (int)c->stride_blocks);
    IFX_HIP(hipGetLastError());
    return IFX_OK;
}

int launch_store_k(const ifx_kv_cache *c, int layer, const void *k_blk, int64_t tok0, hipStream_t s)
{
    const int64_t n = c->n;
    const int H = c->heads;
    const int cpr = (int)(c->head_dim * c->elem / 16);
    hipLaunchKernelGGL(ifx::rows_to_heads_kernel, dim3(grid_for(n * H * cpr)), dim3(256), 0, s,
                       (const u32x4 *)k_blk, (u32x4 *)c->k_of(layer), n, H, cpr, c->k_tokens, tok0);
    IFX_HIP(hipGetLastError());
    return IFX_OK;
}

}  // namespace

extern "C" {

const char *ifx_last_error(void) { return g_err; }

ifx_kv_cache *ifx_kv_cache_create(int layers, int heads, int head_dim, int64_t capacity_tokens)
{
    if (layers <= 0 || heads <= 0 || head_dim <= 0 || capacity_tokens <= 0) {
        fail(IFX_ERR_INVALID_ARG, "create: layers, heads, head_dim and capacity_tokens must be positive");
        return nullptr;
    }
    if (heads > 65535) {
        fail(IFX_ERR_INVALID_ARG, "create: at most 65535 heads");
        return nullptr;
    }
    ifx_kv_cache *c = new (std::nothrow) ifx_kv_cache;
    if (!c) {
        fail(IFX_ERR_OOM, "create: host allocation failed");
        return nullptr;
    }
    c->layers = layers;
    c->heads = heads;
    c->head_dim = head_dim;
    c->capacity_tokens = capacity_tokens;
    return c;
}

// ---- device memory of a cache -------------------------------------------------

// Reserved caches: physical memory comes in pieces of one size, each mapped at a multiple of that
// size inside the reserved range.  (Pieces of differing sizes next to each other are not all
// taken by the runtime's hipMemSetAccess; equal pieces at aligned addresses always were.)
constexpr size_t VMM_CHUNK = (size_t)1 << 20;

// Give the tokens [old_tokens, new_tokens) of every head's K and V region of every layer physical
// memory.  A head's region starts on a piece boundary; the pieces that hold its first old_tokens
// tokens are mapped already.  On failure everything this call mapped is taken back; memory is
// only ever touched behind a mapping whose every call succeeded.
static hipError_t map_tokens(ifx_kv_cache *c, int64_t old_tokens, int64_t new_tokens)
{
    const size_t row = (size_t)c->head_dim * c->elem;
    const size_t have = ((size_t)old_tokens * row + VMM_CHUNK - 1) / VMM_CHUNK, need = ((size_t)new_tokens * row + VMM_CHUNK - 1) / VMM_CHUNK;
    if (need <= have) return hipSuccess;
    const size_t first_new = c->chunks.size();
    hipMemAllocationProp prop = {};
    prop.type = hipMemAllocationTypePinned;
    prop.location.type = hipMemLocationTypeDevice;
    prop.location.id = c->device;
    hipMemAccessDesc access = {};
    access.location = prop.location;
    access.flags = hipMemAccessFlagsProtReadWrite;
    hipError_t e = hipSuccess;
    try {
        c->chunks.reserve(first_new + (size_t)c->layers * 2 * (size_t)c->heads * (need - have));
    } catch (...) {
        return hipErrorOutOfMemory;
    }
    for (int l = 0; l < c->layers && e == hipSuccess; ++l)
        for (int which = 0; which < 2 && e == hipSuccess; ++which)
            for (int h = 0; h < c->heads && e == hipSuccess; ++h) {
                unsigned char *head_base = (which ? c->v_of(l) : c->k_of(l)) + (size_t)h * (size_t)(which ? c->v_tokens : c->k_tokens) * row;
                for (size_t k = have; k < need && e == hipSuccess; ++k) {
                    vmm_chunk ch{{}, head_base + k * VMM_CHUNK, VMM_CHUNK};
                    e = hipMemCreate(&ch.handle, ch.bytes, &prop, 0);
                    if (e != hipSuccess) break;
                    e = hipMemMap(ch.va, ch.bytes, 0, ch.handle, 0);
                    if (e == hipSuccess) {
                        e = hipMemSetAccess(ch.va, ch.bytes, &access, 1);
                        if (e != hipSuccess) (void)hipMemUnmap(ch.va, ch.bytes);
                    }
                    if (e != hipSuccess) {
                        (void)hipMemRelease(ch.handle);
                        break;
                    }
                    c->chunks.push_back(ch);
                }
            }
    if (e != hipSuccess) {
        (void)hipGetLastError();
        while (c->chunks.size() > first_new) {
            (void)hipMemUnmap(c->chunks.back().va, c->chunks.back().bytes);
            (void)hipMemRelease(c->chunks.back().handle);
            c->chunks.pop_back();
        }
    }
    return e;
}

static void release_memory(ifx_kv_cache *c)
{
    if (c->va_bytes) {
        for (auto &ch : c->chunks) {
            (void)hipMemUnmap(ch.va, ch.bytes);
            (void)hipMemRelease(ch.handle);
        }
        c->chunks.clear();
        if (c->slab) (void)hipMemAddressFree(c->slab, c->va_bytes);
        c->va_bytes = 0;
    } else if (c->slab) {
        (void)hipFree(c->slab);
    }
    c->slab = nullptr;
    if (c->aux) (void)hipFree(c->aux);
    c->aux = nullptr;
    c->knorm = nullptr;
    c->blk_list = nullptr;
}

// Side tables for `blocks` slots per layer (key norms for bf16, block lists): allocated and zeroed.
static hipError_t alloc_aux(const ifx_kv_cache *c, int64_t blocks, int parts, void **aux, size_t *kn_bytes)
{
    *kn_bytes = (size_t)c->layers * (size_t)c->heads * (size_t)blocks * (size_t)parts * 4;
    const size_t list_bytes = (size_t)c->layers * (size_t)blocks * sizeof(int);
    hipError_t e = hipMalloc(aux, *kn_bytes + list_bytes);
    if (e == hipSuccess) e = hipMemset(*aux, 0, *kn_bytes + list_bytes);
    return e;
}

int ifx_kv_cache_reserve(ifx_kv_cache *c, int64_t max_capacity_tokens)
{
    if (!c) return fail(IFX_ERR_INVALID_ARG, "cache is NULL");
    if (c->configured) return fail(IFX_ERR_INVALID_ARG, "reserve: must be called before ifx_kv_cache_configure");
    if (max_capacity_tokens < c->capacity_tokens)
        return fail(IFX_ERR_INVALID_ARG, "reserve: max_capacity_tokens (%lld) is below the capacity (%lld)", (long long)max_capacity_tokens,
                    (long long)c->capacity_tokens);
    c->reserve_tokens = max_capacity_tokens;
    return IFX_OK;
}

int ifx_kv_cache_configure(ifx_kv_cache *c, int64_t block_tokens, int dtype, float softmax_scale)
{
    if (!c) return fail(IFX_ERR_INVALID_ARG, "cache is NULL");
    if (c->configured) return fail(IFX_ERR_INVALID_ARG, "configure: already configured");
    if (block_tokens <= 0 || c->capacity_tokens % block_tokens != 0)
        return fail(IFX_ERR_INVALID_ARG, "configure: capacity_tokens (%lld) must be a positive multiple of block_tokens (%lld)",
                    (long long)c->capacity_tokens, (long long)block_tokens);
    if (c->reserve_tokens % block_tokens != 0)
        return fail(IFX_ERR_INVALID_ARG, "configure: the reserved capacity (%lld) must be a multiple of block_tokens (%lld)",
                    (long long)c->reserve_tokens, (long long)block_tokens);
    if (dtype != IFX_F32 && dtype != IFX_BF16 && dtype != IFX_FP8_E4M3) return fail(IFX_ERR_INVALID_ARG, "configure: unknown dtype %d", dtype);
    if (!(softmax_scale >= 0.f) || !std::isfinite(softmax_scale))
        return fail(IFX_ERR_INVALID_ARG, "configure: softmax_scale must be finite and >= 0");
    const int64_t most_tokens = c->reserve_tokens ? c->reserve_tokens : c->capacity_tokens;
    if (most_tokens + block_tokens > (int64_t)1 << 30)
        return fail(IFX_ERR_UNSUPPORTED, "configure: capacity_tokens + block_tokens must not exceed 2^30");
    const int D = c->head_dim;
    size_t elem;
    if (dtype == IFX_BF16 || dtype == IFX_FP8_E4M3) {
        if (D != ifx::BF_D) return fail(IFX_ERR_UNSUPPORTED, "configure: the bf16 path supports head_dim 128 only (got %d)", D);
        if (block_tokens % 8 != 0) return fail(IFX_ERR_UNSUPPORTED, "configure: the bf16 path needs block_tokens %% 8 == 0");
        // 32-bit byte offsets inside one head's K / V region and inside the caller's block tensors
        if (most_tokens + block_tokens + 4096 > ((int64_t)1 << 22) || block_tokens * c->heads > ((int64_t)1 << 22))
            return fail(IFX_ERR_UNSUPPORTED, "configure: the bf16 path needs capacity_tokens + block_tokens + 4096 <= 2^22 and block_tokens * heads <= 2^22");
        elem = dtype == IFX_BF16 ? 2 : 1;
    } else {
        if (D % 8 != 0 || D > ifx::F32_MAXD)
            return fail(IFX_ERR_UNSUPPORTED, "configure: the fp32 path needs head_dim %% 8 == 0 and head_dim <= %d", ifx::F32_MAXD);
        elem = 4;
    }
    int dev = -1;
    IFX_HIP(hipGetDevice(&dev));
    c->device = dev;
    c->elem = elem;
    const size_t row = (size_t)D * elem;
    // about 512 workgroups copy a layer's K rows, a whole number per head
    const int parts = dtype == IFX_F32 ? 0 : c->heads >= 512 ? 1 : (512 + c->heads - 1) / c->heads;

    hipError_t e = hipSuccess;
    if (c->reserve_tokens) {
        int vmm = 0;
        e = hipDeviceGetAttribute(&vmm, hipDeviceAttributeVirtualMemoryManagementSupported, dev);
        if (e != hipSuccess || !vmm) {
            (void)hipGetLastError();
            return fail(IFX_ERR_UNSUPPORTED, "configure: this device cannot map memory into a reserved address range; create the cache "
                                             "without ifx_kv_cache_reserve");
        }
        hipMemAllocationProp prop = {};
        prop.type = hipMemAllocationTypePinned;
        prop.location.type = hipMemLocationTypeDevice;
        prop.location.id = dev;
        e = hipMemGetAllocationGranularity(&c->gran, &prop, hipMemAllocationGranularityMinimum);
        if (e != hipSuccess || c->gran == 0 || VMM_CHUNK % c->gran != 0) {
            (void)hipGetLastError();
            return fail(IFX_ERR_UNSUPPORTED, "configure: unusable mapping granularity");
        }
        // a head's region (reserve_tokens rows, rounded up) starts on a piece boundary
        const int64_t align_tokens = (int64_t)(VMM_CHUNK / std::gcd(VMM_CHUNK, row));
        c->k_tokens = c->v_tokens = (c->reserve_tokens + align_tokens - 1) / align_tokens * align_tokens;
    } else {
        c->k_tokens = c->v_tokens = c->capacity_tokens;
    }
    c->k_layer_bytes = (size_t)c->heads * (size_t)c->k_tokens * row;
    c->v_layer_bytes = (size_t)c->heads * (size_t)c->v_tokens * row;
    const size_t total = (size_t)c->layers * (c->k_layer_bytes + c->v_layer_bytes);
    c->stride_blocks = most_tokens / block_tokens;

    void *p = nullptr;
    if (c->reserve_tokens) {
        e = hipMemAddressReserve(&p, total, VMM_CHUNK, nullptr, 0);
        if (e == hipSuccess && reinterpret_cast<uintptr_t>(p) % VMM_CHUNK != 0) {
            (void)hipMemAddressFree(p, total);
            e = hipErrorInvalidValue;
        }
        if (e == hipSuccess) {
            c->slab = static_cast<unsigned char *>(p);
            c->va_bytes = total;
            e = map_tokens(c, 0, c->capacity_tokens);
        }
    } else {
        e = hipMalloc(&p, total);
        if (e == hipSuccess) {
            c->slab = static_cast<unsigned char *>(p);
            e = hipMemset(p, 0, total);
        }
    }
    size_t kn_bytes = 0;
    if (e == hipSuccess) e = alloc_aux(c, c->stride_blocks, parts, &c->aux, &kn_bytes);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e == hipSuccess && dtype == IFX_F32)
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(ifx::attn_f32_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)ifx::attn_f32_lds_bytes(D));
    if (e == hipSuccess && dtype == IFX_BF16)
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(ifx::attn_bf16_kernel<false, false>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, ifx::BF_LDS_BYTES);
    if (e == hipSuccess && dtype == IFX_BF16)
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(ifx::attn_bf16_kernel<true, false>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, ifx::BF_LDS_BYTES);
    if (e == hipSuccess && dtype == IFX_FP8_E4M3)
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(ifx::attn_bf16_kernel<false, true>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, ifx::BF_LDS_BYTES);
    if (e == hipSuccess && dtype == IFX_FP8_E4M3)
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(ifx::attn_bf16_kernel<true, true>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, ifx::BF_LDS_BYTES);
    bool host_ok = e == hipSuccess;
    if (host_ok) {
        try {
            c->rings.clear();
            c->rings.reserve((size_t)c->layers);
            for (int l = 0; l < c->layers; ++l) c->rings.emplace_back(c->capacity_tokens / block_tokens);
        } catch (...) {
            host_ok = false;
        }
    }
    if (!host_ok) {
        (void)hipGetLastError();
        release_memory(c);
        c->rings.clear();
        if (e == hipSuccess) return fail(IFX_ERR_OOM, "configure: host allocation failed");
        return fail(e == hipErrorOutOfMemory ? IFX_ERR_OOM : IFX_ERR_HIP, "configure: device set-up (%zu bytes of cache): %s", total,
                    hipGetErrorString(e));
    }
    c->knorm = static_cast<uint32_t *>(c->aux);
    c->blk_list = reinterpret_cast<int *>(static_cast<unsigned char *>(c->aux) + kn_bytes);
    c->parts = parts;
    c->n = block_tokens;
    c->dtype = dtype;
    c->scale = softmax_scale > 0.f ? softmax_scale : 1.0f / std::sqrt((float)D);
    c->cap_blocks = c->capacity_tokens / block_tokens;
    c->configured = true;
    return IFX_OK;
}

void ifx_kv_cache_destroy(ifx_kv_cache *c)
{
    if (!c) return;
    if (c->slab || c->aux) {
        (void)hipDeviceSynchronize();
        release_memory(c);
    }
    for (auto *v : {&c->attn_events, &c->commit_events})
        for (auto &ev : *v) {
            (void)hipEventDestroy(ev.start);
            (void)hipEventDestroy(ev.stop);
        }
    delete c;
}

int ifx_kv_cache_reset(ifx_kv_cache *c, int layer)
{
    if (!c) return fail(IFX_ERR_INVALID_ARG, "cache is NULL");
    if (!c->configured) return fail(IFX_ERR_NOT_CONFIGURED, "ifx_kv_cache_configure has not been called");
    if (layer < -1 || layer >= c->layers) return fail(IFX_ERR_INVALID_ARG, "layer %d out of range", layer);
    for (int l = 0; l < c->layers; ++l)
        if (layer == -1 || layer == l) c->rings[(size_t)l].reset();
    return IFX_OK;
}

// Reserved cache: more capacity by mapping more memory behind every head's resident tokens.
static int grow_in_place(ifx_kv_cache *c, int64_t new_capacity_tokens)
{
    if (new_capacity_tokens > c->reserve_tokens)
        return fail(IFX_ERR_UNSUPPORTED, "grow: %lld tokens asked for, %lld were reserved (ifx_kv_cache_reserve)", (long long)new_capacity_tokens,
                    (long long)c->reserve_tokens);
    const int64_t new_cap_blocks = new_capacity_tokens / c->n;
    std::vector<ifx_ring> rings;
    try {
        rings = c->rings;
        for (auto &r : rings) r.grow_in_place(new_cap_blocks);
    } catch (...) {
        return fail(IFX_ERR_OOM, "grow: host allocation failed");
    }
    const hipError_t e = map_tokens(c, c->capacity_tokens, new_capacity_tokens);
    if (e != hipSuccess) return fail(e == hipErrorOutOfMemory ? IFX_ERR_OOM : IFX_ERR_HIP, "grow: mapping memory: %s", hipGetErrorString(e));
    c->rings.swap(rings);
    c->capacity_tokens = new_capacity_tokens;
    c->cap_blocks = new_cap_blocks;
    return IFX_OK;
}

int ifx_kv_cache_grow(ifx_kv_cache *c, int64_t new_capacity_tokens)
{
    if (!c) return fail(IFX_ERR_INVALID_ARG, "cache is NULL");
    if (!c->configured) return fail(IFX_ERR_NOT_CONFIGURED, "ifx_kv_cache_configure has not been called");
    if (new_capacity_tokens <= c->capacity_tokens || new_capacity_tokens % c->n != 0)
        return fail(IFX_ERR_INVALID_ARG, "grow: the new capacity (%lld) must be larger than the old one (%lld) and a multiple of block_tokens (%lld)",
                    (long long)new_capacity_tokens, (long long)c->capacity_tokens, (long long)c->n);
    if (c->reserve_tokens) return grow_in_place(c, new_capacity_tokens);
    if (new_capacity_tokens + c->n + 4096 > (c->mfma() ? (int64_t)1 << 22 : (int64_t)1 << 30))
        return fail(IFX_ERR_UNSUPPORTED, "grow: capacity_tokens + block_tokens is beyond what configure accepts");
    const int H = c->heads, D = c->head_dim;
    const int64_t new_cap_blocks = new_capacity_tokens / c->n;
    const int64_t k_tokens = new_capacity_tokens, v_tokens = new_capacity_tokens;
    const size_t row = (size_t)D * c->elem;  // bytes of one token of one head, K and V alike (V granules: 8 tokens in 8 rows' worth)
    const size_t k_bytes = (size_t)H * k_tokens * row, v_bytes = (size_t)H * v_tokens * row;
    const size_t total = (size_t)c->layers * (k_bytes + v_bytes);
    std::vector<ifx_ring> rings;
    try {
        rings = c->rings;
        for (auto &r : rings) r.grow_moved(new_cap_blocks);
    } catch (...) {
        return fail(IFX_ERR_OOM, "grow: host allocation failed");
    }

    hipError_t e = hipDeviceSynchronize();  // everything enqueued on the old memory has run
    void *p = nullptr, *aux = nullptr;
    size_t kn_bytes = 0;
    if (e == hipSuccess) e = hipMalloc(&p, total);
    if (e == hipSuccess) e = hipMemset(p, 0, total);
    if (e == hipSuccess) e = alloc_aux(c, new_cap_blocks, c->parts, &aux, &kn_bytes);
    // the resident blocks go to slots 0, 1, ... of the new memory, oldest first
    unsigned char *np = static_cast<unsigned char *>(p);
    uint32_t *nkn = static_cast<uint32_t *>(aux);
    const size_t blk = (size_t)c->n * row;  // bytes of one block of one head
    for (int l = 0; l < c->layers && e == hipSuccess; ++l) {
        const ifx_ring &ring = c->rings[(size_t)l];
        unsigned char *nk = np + (size_t)l * (k_bytes + v_bytes), *nv = nk + k_bytes;
        for (int64_t i = 0; i < ring.resident() && e == hipSuccess; ++i) {
            const int64_t s = ring.slot_of_logical(i);
            e = hipMemcpy2D(nk + (size_t)i * blk, (size_t)k_tokens * row, c->k_of(l) + (size_t)s * blk, (size_t)c->k_tokens * row, blk,
                            (size_t)H, hipMemcpyDeviceToDevice);
            if (e == hipSuccess)
                e = hipMemcpy2D(nv + (size_t)i * blk, (size_t)v_tokens * row, c->v_of(l) + (size_t)s * blk, (size_t)c->v_tokens * row,
                                blk, (size_t)H, hipMemcpyDeviceToDevice);
            if (e == hipSuccess && c->parts > 0)  // the block's key-norm entries: one run of `parts` words per head
                e = hipMemcpy2D(nkn + ((size_t)l * (size_t)H * (size_t)new_cap_blocks + (size_t)i) * (size_t)c->parts,
                                (size_t)new_cap_blocks * (size_t)c->parts * 4, c->knorm_of(l) + (size_t)s * (size_t)c->parts,
                                (size_t)c->stride_blocks * (size_t)c->parts * 4, (size_t)c->parts * 4, (size_t)H, hipMemcpyDeviceToDevice);
        }
    }
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        (void)hipGetLastError();
        if (p) (void)hipFree(p);
        if (aux) (void)hipFree(aux);
        return fail(e == hipErrorOutOfMemory ? IFX_ERR_OOM : IFX_ERR_HIP, "grow: %s", hipGetErrorString(e));
    }
    release_memory(c);
    c->slab = np;
    c->aux = aux;
    c->knorm = nkn;
    c->blk_list = reinterpret_cast<int *>(static_cast<unsigned char *>(aux) + kn_bytes);
    c->capacity_tokens = new_capacity_tokens;
    c->cap_blocks = new_cap_blocks;
    c->stride_blocks = new_cap_blocks;
    c->k_tokens = k_tokens;
    c->v_tokens = v_tokens;
    c->k_layer_bytes = k_bytes;
    c->v_layer_bytes = v_bytes;
    c->rings.swap(rings);
    return IFX_OK;
}

int64_t ifx_kv_cache_len(const ifx_kv_cache *c, int layer)
{
    int rc = check_call(c, layer);
    if (rc) return rc;
    return c->rings[(size_t)layer].resident() * c->n;
}

int64_t ifx_kv_cache_committed(const ifx_kv_cache *c, int layer)
{
    int rc = check_call(c, layer);
    if (rc) return rc;
    return c->rings[(size_t)layer].count;
}

int ifx_kv_cache_block_ids(const ifx_kv_cache *c, int layer, int64_t *ids, int max)
{
    int rc = check_call(c, layer);
    if (rc) return rc;
    if (!ids || max < 0) return fail(IFX_ERR_INVALID_ARG, "block_ids: ids is NULL or max < 0");
    return ifx_ring_block_ids(&c->rings[(size_t)layer], ids, max);
}

// Block list of ifx_block_attention_blocks_noalloc: device memory that exists from the moment the
// library is loaded, so that call allocates nothing.  One copy per GPU; its address on a GPU is
// asked for once, with that GPU current, and kept.  In host code the array's name is only a
// handle for that query, never a pointer to pass on.
static __device__ __align__(256) int scratch[IFX_NOALLOC_MAX_LISTED_BLOCKS];

constexpr int MAX_DEVICES = 64;
static std::mutex g_scratch_mutex;
static int *g_scratch_ptr[MAX_DEVICES] = {};

// The current device's copy of `scratch`; the current device must be `device`.
static int scratch_on_device(int device, int **ptr)
{
    int cur = -1;
    IFX_HIP(hipGetDevice(&cur));
    if (cur != device) return fail(IFX_ERR_INVALID_ARG, "the cache lives on device %d, the current device is %d", device, cur);
    if (device < 0 || device >= MAX_DEVICES) return fail(IFX_ERR_UNSUPPORTED, "device %d: at most %d devices", device, MAX_DEVICES);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void *p = nullptr;
        IFX_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        g_scratch_ptr[device] = static_cast<int *>(p);
    }
    *ptr = g_scratch_ptr[device];
    return IFX_OK;
}

// A run of ints handed to a kernel by value: how a host list reaches device memory in stream
// order without pinned memory or a synchronising copy (and a captured graph keeps the values).
constexpr int LIST_CHUNK = 896;
struct int_chunk {
    int v[LIST_CHUNK];
};
__global__ void write_list_kernel(int *dst, const int_chunk vals, int count)
{
    for (int i = threadIdx.x; i < count; i += blockDim.x) dst[i] = vals.v[i];
}

// first_token[0 .. count) -> dst (device), enqueued on s
static int enqueue_list(int *dst, const std::vector<int> &first_token, hipStream_t s)
{
    for (size_t done = 0; done < first_token.size(); done += LIST_CHUNK) {
        int_chunk ch;
        const int cnt = (int)(first_token.size() - done < (size_t)LIST_CHUNK ? first_token.size() - done : (size_t)LIST_CHUNK);
        std::memcpy(ch.v, first_token.data() + done, (size_t)cnt * sizeof(int));
        hipLaunchKernelGGL(write_list_kernel, dim3(1), dim3(256), 0, s, dst + done, ch, cnt);
        IFX_HIP(hipGetLastError());
    }
    return IFX_OK;
}

// Attention of q against the resident blocks `blocks[0 .. n_blocks)` (logical numbers, 0 = oldest,
// already validated; nullptr: all resident blocks in slot order) and, when k_blk / v_blk are given,
// the current block, read where the caller has it.  One attention launch; a selection of more than
// IFX_MAX_KEY_BLOCKS blocks is first written to `list_mem` (device, room for max_list entries:
// the layer's own list, or the caller's), a tiny launch per LIST_CHUNK entries.
static int attention_impl(ifx_kv_cache *c, int layer, const void *q, const void *k_blk, const void *v_blk,
                          const int64_t *blocks, int n_blocks, void *out, float *lse, hipStream_t s, int *list_mem,
                          int64_t max_list, bool always_list)
{
    const ifx_ring &ring = c->rings[(size_t)layer];
    const int n = (int)c->n, H = c->heads, D = c->head_dim;
    const bool with_block = k_blk != nullptr;

    // first physical token of entry i of the cached key set: the selected blocks in the caller's order
    const int64_t n_sel = blocks ? n_blocks : ring.resident();
    auto tok_of = [&](int64_t i) -> int64_t { return (blocks ? ring.slot_of_logical(blocks[i]) : i) * c->n; };
    const int64_t cached = n_sel * c->n;
    if (cached == 0 && !with_block) return fail(IFX_ERR_INVALID_ARG, "attention: no keys selected");
    bool in_place = true;  // block i of the key set is block i of the region: no table needed
    for (int64_t i = 0; i < n_sel && in_place; ++i) in_place = tok_of(i) == i * c->n;
    const bool use_table = !in_place;
    ifx_key_blocks table;
    std::memset(&table, 0, sizeof table);
    if (use_table) {
        table.count = (int)n_sel;
        if (n_sel > IFX_MAX_KEY_BLOCKS || always_list) {
            if (n_sel > max_list)
                return fail(IFX_ERR_UNSUPPORTED, "attention: %lld blocks listed, this call has room for %lld", (long long)n_sel,
                            (long long)max_list);
            try {
                std::vector<int> first((size_t)n_sel);
                for (int64_t i = 0; i < n_sel; ++i) first[(size_t)i] = (int)tok_of(i);
                int rc = enqueue_list(list_mem, first, s);
                if (rc) return rc;
            } catch (const std::bad_alloc &) {
                return fail(IFX_ERR_OOM, "attention: out of host memory");
            }
            table.list = list_mem;
        } else {
            for (int64_t i = 0; i < n_sel; ++i) table.first[i] = (int)tok_of(i);
        }
        // (a copy "past the end" starts 2^30 bytes into a head's region: that must be outside)
        if (c->mfma() && (c->k_tokens > (1 << 22) || c->v_tokens > (1 << 22)))
            return fail(IFX_ERR_UNSUPPORTED, "attention: the block table needs at most 2^22 tokens per head in the cache");
        table.magic = 1;  // fp32 kernel: "the table is in use" (it divides)
        if (c->mfma()) {
            // j / n as the high word of j * magic: exact for all j the kernel forms iff exact at both
            // sides of every block boundary up to there (the quotient estimate is monotone in j);
            // the kernel numbers the keys of each segment of IFX_MAX_KEY_BLOCKS blocks from 0
            table.magic = (unsigned)(0x100000000ull / (uint64_t)c->n) + 1u;
            const uint64_t seg_blocks = n_sel < IFX_MAX_KEY_BLOCKS ? (uint64_t)n_sel : (uint64_t)IFX_MAX_KEY_BLOCKS;
            const uint64_t j_max = seg_blocks * (uint64_t)c->n + 1024;
            for (uint64_t pb = 1; (pb - 1) * (uint64_t)c->n <= j_max; ++pb) {
                const uint64_t j = pb * (uint64_t)c->n;
                if (j > 0xffffffffull || ((j * table.magic) >> 32) != pb || (((j - 1) * table.magic) >> 32) != pb - 1)
                    return fail(IFX_ERR_UNSUPPORTED, "attention: block size %lld is beyond the block table's index arithmetic",
                                (long long)c->n);
            }
        }
    }

    timing_sample sample(c, c->attn_events, s);  // the whole call: everything it enqueues lies between the two events
    int rc = sample.begin();
    if (rc) return rc;
    if (c->mfma()) {
        ifx::attn_bf16_args a;
        a.q = static_cast<const __bf16 *>(q);
        a.kc = c->k_of(layer);
        a.vt = c->v_of(layer);
        a.kb = static_cast<const __bf16 *>(k_blk);
        a.vb = static_cast<const __bf16 *>(v_blk);
        a.out = static_cast<__bf16 *>(out);
        a.lse = lse;
        a.n = n;
        a.H = H;
        a.C = (int)cached;
        a.nb = with_block ? n : 0;
        a.k_tokens = c->k_tokens;
        a.v_tokens = c->v_tokens;
        a.scale_log2 = c->scale * 1.4426950408889634f;
        a.knorm = c->knorm_of(layer);
        a.cap_blocks = (int)c->stride_blocks;
        a.parts = c->parts;
        a.resident_blocks = (int)ring.resident();
        a.shape = ifx::attn_shape_for(n, H);
        const unsigned grid = a.shape.grid;
        a.blocks = table;
        const bool fp8 = c->dtype == IFX_FP8_E4M3;
        if (!use_table && !fp8)
            hipLaunchKernelGGL((ifx::attn_bf16_kernel<false, false>), dim3(grid), dim3(ifx::BF_THREADS), ifx::BF_LDS_BYTES, s, a);
        else if (!fp8)
            hipLaunchKernelGGL((ifx::attn_bf16_kernel<true, false>), dim3(grid), dim3(ifx::BF_THREADS), ifx::BF_LDS_BYTES, s, a);
        else if (!use_table)
            hipLaunchKernelGGL((ifx::attn_bf16_kernel<false, true>), dim3(grid), dim3(ifx::BF_THREADS), ifx::BF_LDS_BYTES, s, a);
        else
            hipLaunchKernelGGL((ifx::attn_bf16_kernel<true, true>), dim3(grid), dim3(ifx::BF_THREADS), ifx::BF_LDS_BYTES, s, a);
    } else {
        dim3 grid((n + ifx::F32_BM - 1) / ifx::F32_BM, H);
        hipLaunchKernelGGL(ifx::attn_f32_kernel, grid, dim3(256), ifx::attn_f32_lds_bytes(D), s,
                           static_cast<const float *>(q), reinterpret_cast<const float *>(c->k_of(layer)),
                           reinterpret_cast<const float *>(c->v_of(layer)), static_cast<const float *>(k_blk),
                           static_cast<const float *>(v_blk), static_cast<float *>(out), lse, n, (int)cached,
                           with_block ? n : 0, H, D, c->k_tokens, c->scale, table);
    }
    IFX_HIP(hipGetLastError());
    return sample.end();
}

int ifx_block_attention(ifx_kv_cache *c, int layer, const void *q, const void *k_blk, const void *v_blk, void *out,
                        ifx_stream_t stream)
{
    int rc = check_call(c, layer);
    if (rc) return rc;
    if ((rc = check_ptr(q, "q")) || (rc = check_ptr(k_blk, "k_blk")) || (rc = check_ptr(v_blk, "v_blk")) ||
        (rc = check_ptr(out, "out")))
        return rc;
    return attention_impl(c, layer, q, k_blk, v_blk, nullptr, 0, out, nullptr, static_cast<hipStream_t>(stream), c->list_of(layer),
                          c->cap_blocks, false);
}

int ifx_block_attention_ranges(ifx_kv_cache *c, int layer, const void *q, const void *k_blk, const void *v_blk,
                               const ifx_block_range *ranges, int n_ranges, void *out, float *lse, ifx_stream_t stream)
{
    int rc = check_call(c, layer);
    if (rc) return rc;
    if ((rc = check_ptr(q, "q")) || (rc = check_ptr(out, "out"))) return rc;
    if ((k_blk == nullptr) != (v_blk == nullptr)) return fail(IFX_ERR_INVALID_ARG, "attention: k_blk and v_blk must both be given or both be NULL");
    if (k_blk && ((rc = check_ptr(k_blk, "k_blk")) || (rc = check_ptr(v_blk, "v_blk")))) return rc;
    if (n_ranges < 0 || (n_ranges > 0 && !ranges)) return fail(IFX_ERR_INVALID_ARG, "attention: n_ranges < 0, or ranges is NULL");
    if (lse && (reinterpret_cast<uintptr_t>(lse) & 3u)) return fail(IFX_ERR_INVALID_ARG, "lse is not 4-byte aligned");
    const ifx_ring &ring = c->rings[(size_t)layer];
    int64_t next_free = 0;
    for (int r = 0; r < n_ranges; ++r) {
        const int64_t first = ranges[r].first_block, count = ranges[r].block_count;
        if (first < next_free) return fail(IFX_ERR_INVALID_ARG, "attention: block ranges must be ascending and must not overlap");
        if (count < 0 || count > ring.resident() || first > ring.resident() - count)
            return fail(IFX_ERR_INVALID_ARG, "attention: block range [%lld, %lld) is not resident (%lld blocks are)",
                        (long long)first, (long long)(first + count), (long long)ring.resident());
        next_free = first + count;
    }
    try {
        std::vector<int64_t> blocks;
        for (int r = 0; r < n_ranges; ++r)
            for (int64_t t = 0; t < ranges[r].block_count; ++t) blocks.push_back(ranges[r].first_block + t);
        static const int64_t none = 0;
        return attention_impl(c, layer, q, k_blk, v_blk, blocks.empty() ? &none : blocks.data(), (int)blocks.size(), out, lse,
                              static_cast<hipStream_t>(stream), c->list_of(layer), c->cap_blocks, false);
    } catch (const std::bad_alloc &) {
        return fail(IFX_ERR_OOM, "attention: out of host memory");
    }
}

// ifx_block_attention_blocks and its variant that keeps the list in the library's static memory.
static int attention_blocks_impl(ifx_kv_cache *c, int layer, const void *q, const void *k_blk, const void *v_blk,
                                 const int64_t *blocks, int n_blocks, void *out, float *lse, ifx_stream_t stream, bool noalloc)
{
    int rc = check_call(c, layer);
    if (rc) return rc;
    if ((rc = check_ptr(q, "q")) || (rc = check_ptr(out, "out"))) return rc;
    if ((k_blk == nullptr) != (v_blk == nullptr)) return fail(IFX_ERR_INVALID_ARG, "attention: k_blk and v_blk must both be given or both be NULL");
    if (k_blk && ((rc = check_ptr(k_blk, "k_blk")) || (rc = check_ptr(v_blk, "v_blk")))) return rc;
    if (n_blocks < -1 || (n_blocks > 0 && !blocks)) return fail(IFX_ERR_INVALID_ARG, "attention: n_blocks < -1, or blocks is NULL");
    if (lse && (reinterpret_cast<uintptr_t>(lse) & 3u)) return fail(IFX_ERR_INVALID_ARG, "lse is not 4-byte aligned");
    int *list_mem = c->list_of(layer);
    int64_t max_list = c->cap_blocks;
    if (noalloc) {
        if (n_blocks > IFX_NOALLOC_MAX_LISTED_BLOCKS)
            return fail(IFX_ERR_UNSUPPORTED, "attention: %d blocks listed, ifx_block_attention_blocks_noalloc takes at most %d", n_blocks,
                        IFX_NOALLOC_MAX_LISTED_BLOCKS);
        if ((rc = scratch_on_device(c->device, &list_mem))) return rc;
        max_list = IFX_NOALLOC_MAX_LISTED_BLOCKS;
    }
    if (n_blocks == -1)  // every resident block, where it lies: the key set of ifx_block_attention
        return attention_impl(c, layer, q, k_blk, v_blk, nullptr, 0, out, lse, static_cast<hipStream_t>(stream), list_mem, max_list,
                              noalloc);
    const ifx_ring &ring = c->rings[(size_t)layer];
    if (n_blocks > ring.resident()) return fail(IFX_ERR_INVALID_ARG, "attention: %d blocks listed, %lld are resident", n_blocks, (long long)ring.resident());
    try {
        std::vector<char> seen((size_t)ring.resident(), 0);
        for (int t = 0; t < n_blocks; ++t) {
            if (blocks[t] < 0 || blocks[t] >= ring.resident())
                return fail(IFX_ERR_INVALID_ARG, "attention: block %lld is not resident (%lld blocks are)", (long long)blocks[t],
                            (long long)ring.resident());
            if (seen[(size_t)blocks[t]]) return fail(IFX_ERR_INVALID_ARG, "attention: block %lld is listed twice", (long long)blocks[t]);
            seen[(size_t)blocks[t]] = 1;
        }
    } catch (const std::bad_alloc &) {
        return fail(IFX_ERR_OOM, "attention: out of host memory");
    }
    static const int64_t none = 0;
    return attention_impl(c, layer, q, k_blk, v_blk, n_blocks ? blocks : &none, n_blocks, out, lse, static_cast<hipStream_t>(stream),
                          list_mem, max_list, noalloc);
}

int ifx_block_attention_blocks(ifx_kv_cache *c, int layer, const void *q, const void *k_blk, const void *v_blk,
                               const int64_t *blocks, int n_blocks, void *out, float *lse, ifx_stream_t stream)
{
    return attention_blocks_impl(c, layer, q, k_blk, v_blk, blocks, n_blocks, out, lse, stream, false);
}

int ifx_block_attention_blocks_noalloc(ifx_kv_cache *c, int layer, const void *q, const void *k_blk, const void *v_blk,
                                       const int64_t *blocks, int n_blocks, void *out, float *lse, ifx_stream_t stream)
{
    return attention_blocks_impl(c, layer, q, k_blk, v_blk, blocks, n_blocks, out, lse, stream, true);
}

int ifx_attention_merge(const void *out_a, const float *lse_a, const void *out_b, const float *lse_b, void *out, float *lse,
                        int64_t rows, int head_dim, int dtype, ifx_stream_t stream)
{
    int rc;
    if ((rc = check_ptr(out_a, "out_a")) || (rc = check_ptr(out_b, "out_b")) || (rc = check_ptr(out, "out"))) return rc;
    if (!lse_a || !lse_b) return fail(IFX_ERR_INVALID_ARG, "merge: lse_a or lse_b is NULL");
    if (rows <= 0 || head_dim <= 0 || head_dim % 8 != 0) return fail(IFX_ERR_INVALID_ARG, "merge: rows must be positive, head_dim a positive multiple of 8");
    if (dtype != IFX_F32 && dtype != IFX_BF16) return fail(IFX_ERR_INVALID_ARG, "merge: unknown dtype %d", dtype);
    const int chunks = head_dim / 8;
    if ((lse == lse_a || lse == lse_b) && lse && 64 % chunks != 0)
        return fail(IFX_ERR_UNSUPPORTED, "merge: lse may alias an input only when 64 %% (head_dim / 8) == 0");
    const int64_t total = rows * chunks;
    if ((total + 255) / 256 > 0x7fffffffLL) return fail(IFX_ERR_UNSUPPORTED, "merge: too many rows");
    hipStream_t s = static_cast<hipStream_t>(stream);
    const dim3 grid((unsigned)((total + 255) / 256));
    if (dtype == IFX_BF16)
        hipLaunchKernelGGL(ifx::merge_kernel<__bf16>, grid, dim3(256), 0, s, static_cast<const __bf16 *>(out_a), lse_a,
                           static_cast<const __bf16 *>(out_b), lse_b, static_cast<__bf16 *>(out), lse, rows, head_dim);
    else
        hipLaunchKernelGGL(ifx::merge_kernel<float>, grid, dim3(256), 0, s, static_cast<const float *>(out_a), lse_a,
                           static_cast<const float *>(out_b), lse_b, static_cast<float *>(out), lse, rows, head_dim);
    IFX_HIP(hipGetLastError());
    return IFX_OK;
}

int ifx_kv_cache_commit(ifx_kv_cache *c, int layer, const void *k_blk, const void *v_blk, ifx_stream_t stream)
{
    int rc = check_call(c, layer);
    if (rc) return rc;
    if ((rc = check_ptr(k_blk, "k_blk")) || (rc = check_ptr(v_blk, "v_blk"))) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    ifx_ring &ring = c->rings[(size_t)layer];
    const int64_t tok0 = ring.next_slot() * c->n;
    timing_sample sample(c, c->commit_events, s);
    if ((rc = sample.begin())) return rc;
    if (c->mfma()) {
        if ((rc = launch_store_blocks_bf16(c, layer, 1, &k_blk, &v_blk, s))) return rc;
    } else {
        if ((rc = launch_store_k(c, layer, k_blk, tok0, s))) return rc;
        if ((rc = launch_store_v(c, layer, v_blk, tok0, s))) return rc;
    }
    ring.commit();  // the copy is enqueued: the slot now holds this block
    return sample.end();
}

int ifx_kv_cache_commit_layers(ifx_kv_cache *c, int first_layer, int n_layers, const void *const *k_blks,
                               const void *const *v_blks, ifx_stream_t stream)
{
    int rc = check_call(c, first_layer);
    if (rc) return rc;
    if (n_layers <= 0 || n_layers > c->layers - first_layer)
        return fail(IFX_ERR_INVALID_ARG, "commit_layers: layers [%d, %d + %d) are not all in [0, %d)", first_layer, first_layer,
                    n_layers, c->layers);
    if (!k_blks || !v_blks) return fail(IFX_ERR_INVALID_ARG, "commit_layers: k_blks or v_blks is NULL");
    for (int i = 0; i < n_layers; ++i)
        if ((rc = check_ptr(k_blks[i], "k_blks[i]")) || (rc = check_ptr(v_blks[i], "v_blks[i]"))) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    timing_sample sample(c, c->commit_events, s);
    if ((rc = sample.begin())) return rc;
    // Rings advance as their launch is enqueued; a launch that fails leaves the layers before it
    // committed (the call reports the error; ifx_kv_cache_committed tells how far it got).
    for (int done = 0; done < n_layers;) {
        const int chunk = n_layers - done < ifx::COMMIT_MAX_LAYERS ? n_layers - done : ifx::COMMIT_MAX_LAYERS;
        if (c->mfma()) {
            if ((rc = launch_store_blocks_bf16(c, first_layer + done, chunk, k_blks + done, v_blks + done, s))) return rc;
            for (int i = 0; i < chunk; ++i) c->rings[(size_t)(first_layer + done + i)].commit();
        } else {
            for (int i = 0; i < chunk; ++i) {
                const int layer = first_layer + done + i;
                const int64_t tok0 = c->rings[(size_t)layer].next_slot() * c->n;
                if ((rc = launch_store_k(c, layer, k_blks[done + i], tok0, s))) return rc;
                if ((rc = launch_store_v(c, layer, v_blks[done + i], tok0, s))) return rc;
                c->rings[(size_t)layer].commit();
            }
        }
        done += chunk;
    }
    return sample.end();
}

int ifx_kv_cache_read(const ifx_kv_cache *c, int layer, void *k_out, void *v_out, int logical_order, ifx_stream_t stream)
{
    int rc = check_call(c, layer);
    if (rc) return rc;
    const ifx_ring &ring = c->rings[(size_t)layer];
    if (ring.resident() == 0) return IFX_OK;
    if ((rc = check_ptr(k_out, "k_out")) || (rc = check_ptr(v_out, "v_out"))) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int H = c->heads, D = c->head_dim;
    const int cpr = (int)(D * c->elem / 16);
    const size_t blk_bytes = (size_t)c->n * H * D * c->io_elem();
    // one block per launch: block b of the order asked for comes from slot slot_of_logical(b) or b
    for (int64_t b = 0; b < ring.resident(); ++b) {
        const int64_t slot = logical_order ? ring.slot_of_logical(b) : b;
        unsigned char *kd = static_cast<unsigned char *>(k_out) + (size_t)b * blk_bytes, *vd = static_cast<unsigned char *>(v_out) + (size_t)b * blk_bytes;
        if (c->dtype == IFX_FP8_E4M3) {  // the codes widened to bf16
            hipLaunchKernelGGL(ifx::e4m3_block_to_rows_kernel, dim3(grid_for(c->n * H * 16)), dim3(256), 0, s, c->k_of(layer), c->v_of(layer),
                               (u32x4 *)kd, (u32x4 *)vd, c->n, H, c->k_tokens, c->v_tokens, slot);
            IFX_HIP(hipGetLastError());
            continue;
        }
        hipLaunchKernelGGL(ifx::heads_to_rows_kernel, dim3(grid_for(c->n * H * cpr)), dim3(256), 0, s, (const u32x4 *)c->k_of(layer),
                           (u32x4 *)kd, c->n, H, cpr, c->k_tokens, slot);
        if (c->dtype == IFX_BF16)
            hipLaunchKernelGGL(ifx::granules_to_rows_kernel, dim3(grid_for(c->n * H * (D / 8))), dim3(256), 0, s,
                               (const uint16_t *)c->v_of(layer), (u16x8 *)vd, c->n, H, D, c->v_tokens, slot);
        else
            hipLaunchKernelGGL(ifx::heads_to_rows_kernel, dim3(grid_for(c->n * H * cpr)), dim3(256), 0, s, (const u32x4 *)c->v_of(layer),
                               (u32x4 *)vd, c->n, H, cpr, c->v_tokens, slot);
        IFX_HIP(hipGetLastError());
    }
    return IFX_OK;
}

int ifx_kv_cache_profile(ifx_kv_cache *c, int enable)
{
    if (!c) return fail(IFX_ERR_INVALID_ARG, "cache is NULL");
    c->profile = enable != 0;
    return IFX_OK;
}

int ifx_kv_cache_profile_read(ifx_kv_cache *c, double *attention_ms, int64_t *attention_launches, double *commit_ms,
                              int64_t *commit_launches)
{
    if (!c) return fail(IFX_ERR_INVALID_ARG, "cache is NULL");
    double sums[2] = {0.0, 0.0};
    int64_t counts[2] = {0, 0};
    std::vector<event_pair> *vs[2] = {&c->attn_events, &c->commit_events};
    int rc = IFX_OK;
    for (int k = 0; k < 2; ++k) {
        for (auto &ev : *vs[k]) {
            float ms = 0.f;
            hipError_t e = hipEventSynchronize(ev.stop);
            if (e == hipSuccess) e = hipEventElapsedTime(&ms, ev.start, ev.stop);
            if (e == hipSuccess) {
                sums[k] += ms;
                counts[k] += 1;
            } else if (rc == IFX_OK) {
                rc = fail(IFX_ERR_HIP, "profile_read: %s", hipGetErrorString(e));
            }
            (void)hipEventDestroy(ev.start);
            (void)hipEventDestroy(ev.stop);
        }
        vs[k]->clear();
    }
    if (attention_ms) *attention_ms = sums[0];
    if (attention_launches) *attention_launches = counts[0];
    if (commit_ms) *commit_ms = sums[1];
    if (commit_launches) *commit_launches = counts[1];
    return rc;
}

// ---- ring bookkeeping on its own -------------------------------------------

ifx_ring *ifx_ring_create(int64_t capacity_blocks)
{
    if (capacity_blocks <= 0) {
        fail(IFX_ERR_INVALID_ARG, "ring_create: capacity_blocks must be positive");
        return nullptr;
    }
    try {
        return new ifx_ring(capacity_blocks);
    } catch (...) {
        fail(IFX_ERR_OOM, "ring_create: host allocation failed");
        return nullptr;
    }
}
void ifx_ring_destroy(ifx_ring *r) { delete r; }
int64_t ifx_ring_commit(ifx_ring *r) { return r ? r->commit() : IFX_ERR_INVALID_ARG; }
int64_t ifx_ring_next_slot(const ifx_ring *r) { return r ? r->next_slot() : IFX_ERR_INVALID_ARG; }
int64_t ifx_ring_resident(const ifx_ring *r) { return r ? r->resident() : IFX_ERR_INVALID_ARG; }
int64_t ifx_ring_committed(const ifx_ring *r) { return r ? r->count : IFX_ERR_INVALID_ARG; }
int64_t ifx_ring_slot_of_logical(const ifx_ring *r, int64_t logical) { return r ? r->slot_of_logical(logical) : IFX_ERR_INVALID_ARG; }
int ifx_ring_block_ids(const ifx_ring *r, int64_t *ids, int max)
{
    if (!r || !ids || max < 0) return fail(IFX_ERR_INVALID_ARG, "ring_block_ids: NULL argument or max < 0");
    int64_t k = r->cap_blocks < max ? r->cap_blocks : max;
    for (int64_t s = 0; s < k; ++s) ids[s] = r->ordinal_in_slot(s);
    return (int)k;
}

void ifx_ring_reset(ifx_ring *r)
{
    if (r) r->reset();
}

int ifx_ring_grow(ifx_ring *r, int64_t new_capacity_blocks, int in_place)
{
    if (!r) return fail(IFX_ERR_INVALID_ARG, "ring is NULL");
    try {
        if (!(in_place ? r->grow_in_place(new_capacity_blocks) : r->grow_moved(new_capacity_blocks)))
            return fail(IFX_ERR_INVALID_ARG, "ring: the new capacity must be larger");
    } catch (...) {
        return fail(IFX_ERR_OOM, "ring_grow: host allocation failed");
    }
    return IFX_OK;
}

int ifx_attention_launch_grid(int block_tokens, int heads)
{
    if (block_tokens < 1 || heads < 1) return fail(IFX_ERR_INVALID_ARG, "launch_grid: block_tokens and heads must be positive");
    return (int)ifx::attn_shape_for(block_tokens, heads).grid;
}

int ifx_attention_launch_item(int block_tokens, int heads, int workgroup, int *item)
{
    if (block_tokens < 1 || heads < 1) return fail(IFX_ERR_INVALID_ARG, "launch_item: block_tokens and heads must be positive");
    if (!item) return fail(IFX_ERR_INVALID_ARG, "launch_item: item is NULL");
    const ifx::attn_shape shape = ifx::attn_shape_for(block_tokens, heads);
    if (workgroup < 0 || (unsigned)workgroup >= shape.grid)
        return fail(IFX_ERR_INVALID_ARG, "launch_item: workgroup %d outside the grid of %u", workgroup, shape.grid);
    const ifx::attn_item it = ifx::attn_item_of(shape, (unsigned)workgroup);
    item[0] = it.head;
    item[1] = it.q_tile;
    item[2] = it.row0;
    item[3] = it.waves;
    item[4] = workgroup & 7;
    return IFX_OK;
}

}  // extern "C"
