// C ABI of libkvc (see include/kvc.h): argument checks and kernel launches only.
#include <algorithm>
#include <new>

#include "kvc_common.h"

// Workspace of kvc_prefetch_layers_window_static: device memory that exists from the moment the library
// is loaded, one copy per GPU, so that the call allocates nothing.  In host code the array's name is
// only a handle for hipGetSymbolAddress; kvc_create asks once per context for the address on its device
// and every later use goes through that pointer.
static constexpr int64_t kStaticWindowBlocks = 65536;  // slots one static-workspace call may cover
static constexpr int32_t kStaticWindowLayers = 1024;   // layers one static-workspace call may cover
static constexpr uint64_t kStaticWindowBytes = 256 + (uint64_t)kStaticWindowLayers * 4 + (uint64_t)kStaticWindowBlocks * 4;
static __device__ __align__(256) unsigned char scratch[kStaticWindowBytes];

struct kvc_ctx {
    int prefetch_policy = 0;
    int window_capacity = 0;      // window engines this device holds at once (0: unknown); an upper bound on useful omega
    void* static_work = nullptr;  // device address of `scratch` on this context's device
    kvc_config cfg;
    kvc::Geometry g;
    int device;
    kvc::DevState* st;  // device
    uint8_t* pool;
    uint64_t pool_bytes;
    kvc_desc* desc;
    uint64_t n_desc;
};

static_assert(sizeof(kvc_desc) == 16, "descriptor is 16 bytes");

// One data call handles at most this many pages: a launch may hold at most 2^32 - 1 threads in all, and
// the decoder spends a 64-thread wave on a page in workgroups of four waves, so its grid of
// ceil(pages / 4) workgroups of 256 threads must stay below 2^24 workgroups (256 GiB of 4 KB pages per
// call; task indices then also divide in 32 bits).
static constexpr int64_t kMaxPagesPerCall = (1ll << 26) - 4;

// Text of the last HIP failure seen by this thread (for kvc_strerror(KVC_ERR_HIP)).
static thread_local hipError_t t_last_hip = hipSuccess;

static bool hip_ok(hipError_t e) {
    if (e != hipSuccess) t_last_hip = e;
    return e == hipSuccess;
}

// Every call must be made with the context's device current: buffers and streams belong to it.
static bool on_ctx_device(const kvc_ctx* ctx);

static bool config_ok(const kvc_config* c) {
    if (!c) return false;
    if (c->tokens_per_block < 1 || c->pages_per_block < 1) return false;
    if (c->scheme < 0 || c->scheme > KVC_MODE_CHAN) return false;
    if (c->scheme == KVC_MODE_CHAN && !(c->tokens_per_block == 16 && (c->head_dim == 64 || c->head_dim == 128 || c->head_dim == 256))) return false;
    const int d = c->head_dim;
    if (d < 32 || d > 256 || d % 32 != 0) return false;
    const int64_t E = (int64_t)c->tokens_per_block * d;
    return E <= 4096;
}

static bool on_ctx_device(const kvc_ctx* ctx) {
    int dev = -1;
    return hip_ok(hipGetDevice(&dev)) && dev == ctx->device;
}

extern "C" {

int kvc_create(kvc_ctx** out, const kvc_config* cfg) {
    if (!out) return KVC_ERR_ARG;
    *out = nullptr;
    if (!cfg) return KVC_ERR_ARG;
    if (cfg->tokens_per_block < 1 || cfg->pages_per_block < 1 || cfg->scheme < 0 || cfg->scheme > KVC_MODE_CHAN ||
        cfg->head_dim < 32 || cfg->head_dim % 32 != 0)
        return KVC_ERR_ARG;
    if (!config_ok(cfg)) return KVC_ERR_UNSUPPORTED;
    kvc_ctx* c = new (std::nothrow) kvc_ctx();
    if (!c) return KVC_ERR_HIP;
    c->cfg = *cfg;
    c->g.N = cfg->tokens_per_block;
    c->g.d = cfg->head_dim;
    c->g.ppb = cfg->pages_per_block;
    c->g.E = cfg->tokens_per_block * cfg->head_dim;
    c->g.lpr = cfg->head_dim / 8;
    c->g.d_magic = ((1u << 22) + (uint32_t)cfg->head_dim - 1) / (uint32_t)cfg->head_dim;
    // the kernels divide by d with this multiplier: it must be exact over the whole range
    for (uint32_t e = 0; e < 8192; ++e)
        if (((e * c->g.d_magic) >> 22) != e / (uint32_t)cfg->head_dim) {
            delete c;
            return KVC_ERR_UNSUPPORTED;
        }
    c->g.row_stride = cfg->head_dim;
    c->g.page_stride = c->g.E;
    c->g.block_stride = (int64_t)c->g.E * cfg->pages_per_block;
    c->pool = nullptr;
    c->pool_bytes = 0;
    c->desc = nullptr;
    c->n_desc = 0;
    if (!hip_ok(hipGetDevice(&c->device)) || !hip_ok(hipMalloc(&c->st, sizeof(kvc::DevState)))) {
        delete c;
        return KVC_ERR_HIP;
    }
    if (!hip_ok(hipMemset(c->st, 0, sizeof(kvc::DevState))) ||
        !hip_ok(hipGetSymbolAddress(&c->static_work, HIP_SYMBOL(scratch))) || !c->static_work) {
        (void)hipFree(c->st);
        delete c;
        return KVC_ERR_HIP;
    }
    c->window_capacity = kvc::window_engine_capacity(c->g);
    *out = c;
    return KVC_OK;
}

void kvc_destroy(kvc_ctx* ctx) {
    if (!ctx) return;
    (void)hipFree(ctx->st);
    delete ctx;
}

int kvc_set_scheme(kvc_ctx* ctx, int32_t scheme) {
    if (!ctx || scheme < 0 || scheme > KVC_MODE_CHAN) return KVC_ERR_ARG;
    if (scheme == KVC_MODE_CHAN && !(ctx->g.N == 16 && (ctx->g.d == 64 || ctx->g.d == 128 || ctx->g.d == 256))) return KVC_ERR_UNSUPPORTED;
    ctx->cfg.scheme = scheme;
    return KVC_OK;
}

int kvc_set_cache_layout(kvc_ctx* ctx, int64_t block_stride, int64_t page_stride, int64_t row_stride) {
    if (!ctx) return KVC_ERR_ARG;
    if (block_stride == 0 && page_stride == 0 && row_stride == 0) {  // back to the contiguous default
        row_stride = ctx->g.d;
        page_stride = ctx->g.E;
        block_stride = (int64_t)ctx->g.E * ctx->g.ppb;
    }
    // 128-bit accesses need 8-element granularity; rows may not overlap their own channels
    if (row_stride < ctx->g.d || page_stride <= 0 || block_stride <= 0) return KVC_ERR_ARG;
    if ((row_stride & 7) || (page_stride & 7) || (block_stride & 7)) return KVC_ERR_ARG;
    if (row_stride * ctx->g.N >= (1ll << 30)) return KVC_ERR_ARG;  // a page's rows span less than 2 GiB
    ctx->g.row_stride = row_stride;
    ctx->g.page_stride = page_stride;
    ctx->g.block_stride = block_stride;
    return KVC_OK;
}

int kvc_bind_pool(kvc_ctx* ctx, void* d_pool, uint64_t pool_bytes, kvc_desc* d_desc, uint64_t n_desc_pages) {
    if (!ctx || !d_pool || !d_desc || pool_bytes == 0 || n_desc_pages == 0) return KVC_ERR_ARG;
    if ((reinterpret_cast<uintptr_t>(d_pool) & 15u) || (reinterpret_cast<uintptr_t>(d_desc) & 15u) || (pool_bytes & 15u))
        return KVC_ERR_ARG;
    // The pool may also live in pinned, device-mapped host memory (a slow-link tier): take the address
    // the device sees.  Pageable host memory is rejected here rather than faulting in a kernel.
    hipPointerAttribute_t attr;
    if (!hip_ok(hipPointerGetAttributes(&attr, d_pool))) {
        (void)hipGetLastError();  // the failed query is ours: leave no error behind for the caller's next check
        return KVC_ERR_ARG;
    }
    if (attr.type == hipMemoryTypeHost) {
        if (!attr.devicePointer) return KVC_ERR_ARG;
        d_pool = attr.devicePointer;
    } else if (attr.type != hipMemoryTypeDevice && attr.type != hipMemoryTypeManaged) {
        return KVC_ERR_ARG;
    }
    hipPointerAttribute_t dattr;
    if (!hip_ok(hipPointerGetAttributes(&dattr, d_desc))) {
        (void)hipGetLastError();
        return KVC_ERR_ARG;
    }
    if (dattr.type == hipMemoryTypeUnregistered) return KVC_ERR_ARG;
    if (dattr.type == hipMemoryTypeHost) {
        if (!dattr.devicePointer) return KVC_ERR_ARG;
        d_desc = static_cast<kvc_desc*>(dattr.devicePointer);
    }
    ctx->pool = static_cast<uint8_t*>(d_pool);
    ctx->pool_bytes = pool_bytes;
    ctx->desc = d_desc;
    ctx->n_desc = n_desc_pages;
    return KVC_OK;
}

int kvc_reset_pool(kvc_ctx* ctx, void* stream) {
    if (!ctx) return KVC_ERR_ARG;
    if (!ctx->pool) return KVC_ERR_NOT_BOUND;
    if (!on_ctx_device(ctx)) return KVC_ERR_ARG;
    return hip_ok(kvc::launch_reset(ctx->st, ctx->desc, ctx->n_desc, static_cast<hipStream_t>(stream)))
               ? KVC_OK
               : KVC_ERR_HIP;
}

int kvc_restore_pool(kvc_ctx* ctx, uint64_t used_bytes, void* stream) {
    if (!ctx) return KVC_ERR_ARG;
    if (!ctx->pool) return KVC_ERR_NOT_BOUND;
    if ((used_bytes & 15u) || used_bytes > ctx->pool_bytes) return KVC_ERR_ARG;
    if (!on_ctx_device(ctx)) return KVC_ERR_ARG;
    return hip_ok(kvc::launch_set_cursor(ctx->st, used_bytes / 16, static_cast<hipStream_t>(stream))) ? KVC_OK : KVC_ERR_HIP;
}

static int compress_impl(kvc_ctx* ctx, const void* d_cache, int64_t n_cache_blocks, const int32_t* d_src_block_ids,
                         const int32_t* d_pool_block_ids, const uint8_t* d_block_scheme, int32_t n, void* stream) {
    if (!ctx || n < 0 || n_cache_blocks < 0) return KVC_ERR_ARG;
    if (!ctx->pool) return KVC_ERR_NOT_BOUND;
    if (n == 0) return KVC_OK;
    if (!on_ctx_device(ctx)) return KVC_ERR_ARG;
    if (!d_cache || (reinterpret_cast<uintptr_t>(d_cache) & 15u)) return KVC_ERR_ARG;
    // identity ids are checked here; explicit id arrays live on the device and are checked there
    if (!d_src_block_ids && (int64_t)n > n_cache_blocks) return KVC_ERR_ARG;
    if (!d_pool_block_ids && (uint64_t)n * (uint64_t)ctx->g.ppb > ctx->n_desc) return KVC_ERR_ARG;
    if ((int64_t)n * ctx->g.ppb > kMaxPagesPerCall) return KVC_ERR_ARG;
    kvc::EncodeArgs a;
    a.cache = static_cast<const uint16_t*>(d_cache);
    a.n_cache_blocks = n_cache_blocks;
    a.src_ids = d_src_block_ids;
    a.pool_ids = d_pool_block_ids;
    a.n_pages = (int64_t)n * ctx->g.ppb;
    a.g = ctx->g;
    a.scheme = ctx->cfg.scheme;
    a.block_scheme = d_block_scheme;
    a.pool = ctx->pool;
    a.pool_units = ctx->pool_bytes / 16;
    a.desc = ctx->desc;
    a.n_desc = ctx->n_desc;
    a.st = ctx->st;
    return hip_ok(kvc::launch_compress(a, static_cast<hipStream_t>(stream))) ? KVC_OK : KVC_ERR_HIP;
}

int kvc_compress_blocks(kvc_ctx* ctx, const void* d_cache, int64_t n_cache_blocks, const int32_t* d_src_block_ids,
                        const int32_t* d_pool_block_ids, int32_t n, void* stream) {
    return compress_impl(ctx, d_cache, n_cache_blocks, d_src_block_ids, d_pool_block_ids, nullptr, n, stream);
}

int kvc_compress_blocks_mixed(kvc_ctx* ctx, const void* d_cache, int64_t n_cache_blocks, const int32_t* d_src_block_ids,
                              const int32_t* d_pool_block_ids, const uint8_t* d_block_scheme, int32_t n, void* stream) {
    if (!d_block_scheme) return KVC_ERR_ARG;
    return compress_impl(ctx, d_cache, n_cache_blocks, d_src_block_ids, d_pool_block_ids, d_block_scheme, n, stream);
}

static void fill_decode_common(kvc_ctx* ctx, kvc::DecodeArgs& a) {
    a.g = ctx->g;
    a.pool = ctx->pool;
    a.pool_units = ctx->pool_bytes / 16;
    a.desc = ctx->desc;
    a.n_desc = ctx->n_desc;
    a.st = ctx->st;
    a.pool_ids = nullptr;
    a.dst_ids = nullptr;
    a.block_table = nullptr;
    a.pred = nullptr;
    a.max_blocks = a.n_seq = a.k = a.n_layers = 0;
    a.pool_blocks_per_layer = 0;
}

int kvc_decompress_blocks(kvc_ctx* ctx, void* d_cache_out, int64_t n_out_blocks, const int32_t* d_pool_block_ids,
                          const int32_t* d_dst_block_ids, int32_t n, void* stream) {
    if (!ctx || n < 0 || n_out_blocks < 0) return KVC_ERR_ARG;
    if (!ctx->pool) return KVC_ERR_NOT_BOUND;
    if (n == 0) return KVC_OK;
    if (!on_ctx_device(ctx)) return KVC_ERR_ARG;
    if (!d_cache_out || (reinterpret_cast<uintptr_t>(d_cache_out) & 15u)) return KVC_ERR_ARG;
    if (!d_dst_block_ids && (int64_t)n > n_out_blocks) return KVC_ERR_ARG;
    if (!d_pool_block_ids && (uint64_t)n * (uint64_t)ctx->g.ppb > ctx->n_desc) return KVC_ERR_ARG;
    if ((int64_t)n * ctx->g.ppb > kMaxPagesPerCall) return KVC_ERR_ARG;
    kvc::DecodeArgs a;
    fill_decode_common(ctx, a);
    a.out = static_cast<uint16_t*>(d_cache_out);
    a.n_out_blocks = n_out_blocks;
    a.pool_ids = d_pool_block_ids;
    a.dst_ids = d_dst_block_ids;
    a.n_pages = (int64_t)n * ctx->g.ppb;
    return hip_ok(kvc::launch_decompress(a, static_cast<hipStream_t>(stream))) ? KVC_OK : KVC_ERR_HIP;
}

int kvc_gather_decompress(kvc_ctx* ctx, void* d_out, const int32_t* d_block_table, int32_t max_blocks,
                          const int32_t* d_pred, int32_t n_seq, int32_t k, int32_t n_layers,
                          int64_t pool_blocks_per_layer, void* stream) {
    if (!ctx || n_seq < 0 || k < 0 || n_layers < 0 || max_blocks < 0 || pool_blocks_per_layer < 0) return KVC_ERR_ARG;
    if (!ctx->pool) return KVC_ERR_NOT_BOUND;
    const int64_t n_blocks = (int64_t)n_layers * n_seq * k;
    if (n_blocks == 0) return KVC_OK;
    if (!on_ctx_device(ctx)) return KVC_ERR_ARG;
    if (!d_out || !d_block_table || !d_pred || max_blocks == 0 || (reinterpret_cast<uintptr_t>(d_out) & 15u))
        return KVC_ERR_ARG;
    if ((uint64_t)n_layers * (uint64_t)pool_blocks_per_layer * (uint64_t)ctx->g.ppb > ctx->n_desc) return KVC_ERR_ARG;
    if (n_blocks > kMaxPagesPerCall / ctx->g.ppb) return KVC_ERR_ARG;
    kvc::DecodeArgs a;
    fill_decode_common(ctx, a);
    a.out = static_cast<uint16_t*>(d_out);
    a.n_out_blocks = n_blocks;
    a.n_pages = n_blocks * ctx->g.ppb;
    a.block_table = d_block_table;
    a.pred = d_pred;
    a.max_blocks = max_blocks;
    a.n_seq = n_seq;
    a.k = k;
    a.n_layers = n_layers;
    a.pool_blocks_per_layer = pool_blocks_per_layer;
    return hip_ok(kvc::launch_decompress(a, static_cast<hipStream_t>(stream))) ? KVC_OK : KVC_ERR_HIP;
}

int kvc_set_prefetch_policy(kvc_ctx* ctx, int32_t policy) {
    if (!ctx || (policy != 0 && policy != 1)) return KVC_ERR_ARG;
    ctx->prefetch_policy = policy;
    return KVC_OK;
}

int kvc_prefetch_reset(kvc_ctx* ctx, int32_t* d_tags, int32_t n_seq, int32_t k, int32_t n_layers, void* stream) {
    if (!ctx || !d_tags || n_seq < 0 || k < 0 || n_layers < 0) return KVC_ERR_ARG;
    if (!on_ctx_device(ctx)) return KVC_ERR_ARG;
    return hip_ok(kvc::launch_fill_i32(d_tags, -1, 2ull * (uint64_t)n_layers * (uint64_t)n_seq * (uint64_t)k,
                                       static_cast<hipStream_t>(stream)))
               ? KVC_OK
               : KVC_ERR_HIP;
}

// Shared body of the prefetch calls.  omega = 0: one decode launch over the call's slots (no bound on
// the transfers in flight); omega > 0: the outstanding-request window, with its queue in `work`.
static int prefetch_impl(kvc_ctx* ctx, void* d_l2, int32_t* d_tags, int32_t* d_fetch, int32_t* d_loc,
                         const int32_t* d_block_table, int32_t max_blocks, const int32_t* d_pred,
                         const int32_t* d_l1_first_block, int32_t n_seq, int32_t k, int32_t n_layers, int32_t layer_begin,
                         int32_t layer_end, int64_t pool_blocks_per_layer, int32_t fill_half, int32_t omega,
                         long long* d_notify, void* work, uint64_t work_bytes, void* stream) {
    if (!ctx || n_seq < 0 || k < 0 || n_layers < 0 || max_blocks < 0 || pool_blocks_per_layer < 0 || omega < 0) return KVC_ERR_ARG;
    if (k > kvc::kMaxPrefetchK) return KVC_ERR_ARG;
    if (layer_begin < 0 || layer_end < layer_begin || layer_end > n_layers || (fill_half != 0 && fill_half != 1))
        return KVC_ERR_ARG;
    if (!ctx->pool) return KVC_ERR_NOT_BOUND;
    const int64_t n_slots = (int64_t)n_layers * n_seq * k;
    const int64_t n_now = (int64_t)(layer_end - layer_begin) * n_seq * k;
    if (n_now == 0) return KVC_OK;
    if (!on_ctx_device(ctx)) return KVC_ERR_ARG;
    if (!d_l2 || !d_tags || !d_fetch || !d_loc || !d_block_table || !d_pred || max_blocks == 0 ||
        (reinterpret_cast<uintptr_t>(d_l2) & 15u))
        return KVC_ERR_ARG;
    if (2 * n_slots > INT32_MAX || n_now > kMaxPagesPerCall / ctx->g.ppb) return KVC_ERR_ARG;
    if ((uint64_t)n_layers * (uint64_t)pool_blocks_per_layer * (uint64_t)ctx->g.ppb > ctx->n_desc ||
        (uint64_t)n_layers * (uint64_t)pool_blocks_per_layer > (uint64_t)INT32_MAX)
        return KVC_ERR_ARG;
    if (omega > 0) {
        if (!d_notify || !work || (reinterpret_cast<uintptr_t>(work) & 255u) || (reinterpret_cast<uintptr_t>(d_notify) & 7u) ||
            work_bytes < kvc::window_workspace_bytes(n_now, layer_end - layer_begin))
            return KVC_ERR_ARG;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    kvc::PlanArgs p;
    p.block_table = d_block_table;
    p.pred = d_pred;
    p.l1_first = d_l1_first_block;
    p.max_blocks = max_blocks;
    p.n_seq = n_seq;
    p.k = k;
    p.layer_begin = layer_begin;
    p.layer_end = layer_end;
    p.n_layers = n_layers;
    p.fill_half = fill_half;
    p.policy = ctx->prefetch_policy;
    p.pool_blocks_per_layer = pool_blocks_per_layer;
    p.tags = d_tags;
    p.fetch = d_fetch;
    p.loc = d_loc;
    p.st = ctx->st;
    if (!hip_ok(kvc::launch_prefetch_plan(p, s))) return KVC_ERR_HIP;
    // decode the listed pool blocks into their slots of the half being filled; slots are blocks of the
    // cache layout in force (block_stride elements apart)
    const int64_t first = (int64_t)layer_begin * n_seq * k;
    kvc::DecodeArgs a;
    fill_decode_common(ctx, a);
    a.out = static_cast<uint16_t*>(d_l2) + ((int64_t)fill_half * n_slots + first) * ctx->g.block_stride;
    a.n_out_blocks = n_now;
    a.pool_ids = d_fetch + first;
    a.n_pages = n_now * ctx->g.ppb;
    if (omega == 0) return hip_ok(kvc::launch_decompress(a, s)) ? KVC_OK : KVC_ERR_HIP;
    // engines beyond what the device holds at once would never get a turn: the bound stays "at most omega"
    if (ctx->window_capacity > 0) omega = std::min(omega, ctx->window_capacity);
    kvc::WindowArgs w;
    char* wb = static_cast<char*>(work);
    w.hdr = reinterpret_cast<kvc::WindowHdr*>(wb);
    w.pending = reinterpret_cast<int32_t*>(wb + sizeof(kvc::WindowHdr));
    w.queue = reinterpret_cast<int32_t*>(wb + kvc::window_workspace_bytes(0, layer_end - layer_begin));
    w.fetch = d_fetch + first;
    w.n_now = (int32_t)n_now;
    w.per_layer = n_seq * k;
    w.layer_begin = layer_begin;
    w.n_layers_call = layer_end - layer_begin;
    w.n_layers = n_layers;
    w.omega = omega;
    w.notify = d_notify;
    if (!hip_ok(kvc::launch_window_build(w, s))) return KVC_ERR_HIP;
    return hip_ok(kvc::launch_decompress_window(a, w, omega, s)) ? KVC_OK : KVC_ERR_HIP;
}

int kvc_prefetch_layers(kvc_ctx* ctx, void* d_l2, int32_t* d_tags, int32_t* d_fetch, int32_t* d_loc,
                        const int32_t* d_block_table, int32_t max_blocks, const int32_t* d_pred,
                        const int32_t* d_l1_first_block, int32_t n_seq, int32_t k, int32_t n_layers, int32_t layer_begin,
                        int32_t layer_end, int64_t pool_blocks_per_layer, int32_t fill_half, void* stream) {
    return prefetch_impl(ctx, d_l2, d_tags, d_fetch, d_loc, d_block_table, max_blocks, d_pred, d_l1_first_block, n_seq, k,
                         n_layers, layer_begin, layer_end, pool_blocks_per_layer, fill_half, 0, nullptr, nullptr, 0, stream);
}

uint64_t kvc_prefetch_window_workspace(int64_t n_blocks, int32_t n_layers_call) {
    if (n_blocks < 0 || n_layers_call < 0) return 0;
    return kvc::window_workspace_bytes(n_blocks, n_layers_call);
}

int kvc_wall_clock_khz(int32_t* khz) {
    if (!khz) return KVC_ERR_ARG;
    int dev = -1, v = 0;
    if (!hip_ok(hipGetDevice(&dev)) || !hip_ok(hipDeviceGetAttribute(&v, hipDeviceAttributeWallClockRate, dev))) return KVC_ERR_HIP;
    *khz = v;
    return KVC_OK;
}

int kvc_device_clocks(int32_t* shader_khz, int32_t* memory_khz, int32_t* memory_bus_bits) {
    int dev = -1;
    if (!hip_ok(hipGetDevice(&dev))) return KVC_ERR_HIP;
    const struct {
        int32_t* out;
        hipDeviceAttribute_t attr;
    } q[3] = {{shader_khz, hipDeviceAttributeClockRate}, {memory_khz, hipDeviceAttributeMemoryClockRate}, {memory_bus_bits, hipDeviceAttributeMemoryBusWidth}};
    for (const auto& e : q) {
        int v = 0;
        if (!e.out) continue;
        if (!hip_ok(hipDeviceGetAttribute(&v, e.attr, dev))) return KVC_ERR_HIP;
        *e.out = v;
    }
    return KVC_OK;
}

int kvc_prefetch_layers_window(kvc_ctx* ctx, void* d_l2, int32_t* d_tags, int32_t* d_fetch, int32_t* d_loc,
                               const int32_t* d_block_table, int32_t max_blocks, const int32_t* d_pred,
                               const int32_t* d_l1_first_block, int32_t n_seq, int32_t k, int32_t n_layers,
                               int32_t layer_begin, int32_t layer_end, int64_t pool_blocks_per_layer, int32_t fill_half,
                               int32_t omega, int64_t* d_notify, void* d_work, uint64_t work_bytes, void* stream) {
    if (omega < 1) return KVC_ERR_ARG;
    return prefetch_impl(ctx, d_l2, d_tags, d_fetch, d_loc, d_block_table, max_blocks, d_pred, d_l1_first_block, n_seq, k,
                         n_layers, layer_begin, layer_end, pool_blocks_per_layer, fill_half, omega,
                         reinterpret_cast<long long*>(d_notify), d_work, work_bytes, stream);
}

int kvc_prefetch_layers_window_static(kvc_ctx* ctx, void* d_l2, int32_t* d_tags, int32_t* d_fetch, int32_t* d_loc,
                                      const int32_t* d_block_table, int32_t max_blocks, const int32_t* d_pred,
                                      const int32_t* d_l1_first_block, int32_t n_seq, int32_t k, int32_t n_layers,
                                      int32_t layer_begin, int32_t layer_end, int64_t pool_blocks_per_layer,
                                      int32_t fill_half, int32_t omega, int64_t* d_notify, void* stream) {
    if (!ctx || omega < 1 || layer_begin < 0 || layer_end < layer_begin || n_seq < 0 || k < 0 || k > kvc::kMaxPrefetchK)
        return KVC_ERR_ARG;
    if (layer_end - layer_begin > kStaticWindowLayers || (int64_t)(layer_end - layer_begin) * n_seq * k > kStaticWindowBlocks)
        return KVC_ERR_TOO_LARGE;
    static_assert(kStaticWindowBytes >= 256 + ((uint64_t)kStaticWindowLayers * 4 + 255) / 256 * 256 + (uint64_t)kStaticWindowBlocks * 4,
                  "the static array holds the largest admitted call");
    return prefetch_impl(ctx, d_l2, d_tags, d_fetch, d_loc, d_block_table, max_blocks, d_pred, d_l1_first_block, n_seq, k,
                         n_layers, layer_begin, layer_end, pool_blocks_per_layer, fill_half, omega,
                         reinterpret_cast<long long*>(d_notify), ctx->static_work, kStaticWindowBytes, stream);
}

int kvc_stats(kvc_ctx* ctx, kvc_stats_t* out, void* stream) {
    if (!ctx || !out) return KVC_ERR_ARG;
    if (!ctx->pool) return KVC_ERR_NOT_BOUND;
    if (!on_ctx_device(ctx)) return KVC_ERR_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (!hip_ok(kvc::launch_stats(ctx->st, ctx->desc, ctx->n_desc, s))) return KVC_ERR_HIP;
    kvc::DevState h;
    if (!hip_ok(hipMemcpyAsync(&h, ctx->st, sizeof(h), hipMemcpyDeviceToHost, s))) return KVC_ERR_HIP;
    if (!hip_ok(hipStreamSynchronize(s))) return KVC_ERR_HIP;
    out->pool_bytes_used = std::min<uint64_t>(h.cursor16 * 16ull, ctx->pool_bytes);
    for (int i = 0; i < 6; ++i) out->pages[i] = h.stats[i];
    out->pages_invalid = h.stats[6];
    out->payload_bytes = h.stats[7] * 16ull;
    out->status = h.status;
    out->rsvd = 0;
    if (h.status & KVC_ST_POOL_FULL) return KVC_ERR_POOL_FULL;
    if (h.status & (KVC_ST_CORRUPT | KVC_ST_BAD_INDEX)) return KVC_ERR_CORRUPT;
    return KVC_OK;
}

int kvc_page_scales(const uint16_t* d_amax, float* d_scale, float* d_scale_inv, uint64_t n, void* stream) {
    if (n == 0) return KVC_OK;
    if (!d_amax || !d_scale || !d_scale_inv || n > (1ull << 31)) return KVC_ERR_ARG;
    return hip_ok(kvc::launch_page_scales(d_amax, d_scale, d_scale_inv, n, static_cast<hipStream_t>(stream))) ? KVC_OK
                                                                                                            : KVC_ERR_HIP;
}

int kvc_copy_bytes(void* d_dst, const void* d_src, uint64_t nbytes, void* stream) {
    if (!d_dst || !d_src || (nbytes & 15u) || (reinterpret_cast<uintptr_t>(d_dst) & 15u) ||
        (reinterpret_cast<uintptr_t>(d_src) & 15u) || nbytes > (1ull << 38) - 4096)
        return KVC_ERR_ARG;
    return hip_ok(kvc::launch_copy(d_dst, d_src, nbytes / 16, static_cast<hipStream_t>(stream))) ? KVC_OK : KVC_ERR_HIP;
}

const char* kvc_strerror(int code) {
    switch (code) {
        case KVC_OK: return "ok";
        case KVC_ERR_ARG: return "bad argument";
        case KVC_ERR_NOT_BOUND: return "no pool bound to the context";
        case KVC_ERR_HIP: return t_last_hip != hipSuccess ? hipGetErrorString(t_last_hip) : "HIP runtime error";
        case KVC_ERR_POOL_FULL: return "compressed pool exhausted; some pages were not stored";
        case KVC_ERR_CORRUPT: return "invalid descriptor, payload or block index met on the device";
        case KVC_ERR_TOO_LARGE: return "call exceeds the library's static workspace (at most 65536 slots and 1024 layers per call)";
        case KVC_ERR_UNSUPPORTED: return "page geometry not supported (head_dim a multiple of 32 up to 256, N*d <= 4096; mode 5: N = 16, d = 64, 128 or 256)";
        default: return "unknown error";
    }
}

}  // extern "C"
