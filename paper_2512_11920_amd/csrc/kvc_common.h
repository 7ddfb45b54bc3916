// Shared declarations between the C-ABI host code (kvc_api.hip) and the kernels (kvc_kernels.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kvc.h"

namespace kvc {

// Device state block owned by a context.
struct DevState {
    unsigned long long cursor16;  // next free 16-byte unit of the pool
    unsigned int status;          // sticky KVC_ST_* bits
    unsigned int pad;
    unsigned long long stats[8];  // scratch of kvc_stats: pages[0..5], invalid, payload16
};

// Page geometry and cache layout.  Element (token j, channel i) of page pg of block b sits at
// b*block_stride + pg*page_stride + j*row_stride + i of the cache buffer (all in FP16 elements).
struct Geometry {
    int32_t N, d, ppb, E;  // E = N*d elements per page
    int32_t lpr;           // lanes per token row: d / 8 (a lane owns 8 channels)
    uint32_t d_magic;      // ceil(2^22 / d):   e / d   == (e * d_magic) >> 22   for e < 8192
    int64_t row_stride, page_stride, block_stride;
};

struct EncodeArgs {
    const uint16_t* cache;
    int64_t n_cache_blocks;
    const int32_t* src_ids;
    const int32_t* pool_ids;
    int64_t n_pages;  // n blocks * ppb
    Geometry g;
    int32_t scheme;
    const uint8_t* block_scheme;  // optional: requested mode per block (overrides scheme)
    uint8_t* pool;
    uint64_t pool_units;  // pool size in 16-byte units
    kvc_desc* desc;
    uint64_t n_desc;
    DevState* st;
};

struct DecodeArgs {
    uint16_t* out;
    int64_t n_out_blocks;
    const int32_t* pool_ids;
    const int32_t* dst_ids;
    int64_t n_pages;
    Geometry g;
    const uint8_t* pool;
    uint64_t pool_units;
    const kvc_desc* desc;
    uint64_t n_desc;
    DevState* st;
    // gather form (block_table != nullptr): page task t = ((l*n_seq + s)*k + j)*ppb + pg
    const int32_t* block_table;
    const int32_t* pred;
    int32_t max_blocks, n_seq, k, n_layers;
    int64_t pool_blocks_per_layer;
};

constexpr int kMaxPrefetchK = 32;  // predictions per sequence the slot-reuse policy can plan

// Arguments of the prefetch planner (Algorithm 1: translate, residency filter, slot assignment).
struct PlanArgs {
    const int32_t* block_table;  // [n_seq][max_blocks]
    const int32_t* pred;         // [n_seq][k]
    const int32_t* l1_first;     // [n_seq] or null: logical blocks >= l1_first[s] are GPU-local (L1)
    int32_t max_blocks, n_seq, k, layer_begin, layer_end, n_layers, fill_half;
    int32_t policy;              // 0: slot j for prediction j; 1: keep wanted blocks, fill unwanted slots
    int64_t pool_blocks_per_layer;
    int32_t* tags;   // [2][n_layers*n_seq*k]
    int32_t* fetch;  // [n_layers*n_seq*k]
    int32_t* loc;    // [n_layers*n_seq*k]
    DevState* st;
};

// Outstanding-request window of the prefetch path (Algorithm 1: WaitCompletion over at most Omega_max
// concurrent transfers).  The workspace of one call: this header, then one pending counter per layer of
// the call, then the queue of issued transfers (slot indices relative to the call's first slot).
struct WindowHdr {
    unsigned int n_issued;  // entries in the queue (constant while the engines run)
    unsigned int engines;   // transfer engines of the call = min(omega, n_issued): the bound on blocks in flight
    unsigned int chunk;     // queue entries an engine takes per turn (1..8)
    unsigned int pad0[13];
    unsigned int ticket;    // next queue entry to hand out; the two hot counters sit in cache lines of their own
    unsigned int pad1[15];
    unsigned int done;      // blocks completed
    unsigned int pad2[31];
};
static_assert(sizeof(WindowHdr) == 256, "window header is 256 bytes");

struct WindowArgs {
    WindowHdr* hdr;
    int32_t* pending;      // [layers of the call]: issued transfers of the layer not yet completed
    int32_t* queue;        // [n_now]
    const int32_t* fetch;  // the call's part of the fetch list: [n_now], pool block or -1
    int32_t n_now;         // slots of the call = layers of the call * per_layer
    int32_t per_layer;     // n_seq * k
    int32_t layer_begin, n_layers_call, n_layers;
    int32_t omega;         // engines the decode launch starts at most
    long long* notify;     // [n_layers + 4], see kvc.h
};

inline uint64_t window_workspace_bytes(int64_t n_blocks, int64_t n_layers_call) {
    return sizeof(WindowHdr) + (uint64_t)((n_layers_call * 4 + 255) / 256 * 256) + (uint64_t)n_blocks * 4;
}

// Launch `kernel` and return the status of this launch itself.  (A launch through the <<<>>> form
// reports failure only through the thread's last-error slot, which may still hold an error left by
// an earlier, unrelated call of the application.)
template <typename T>
struct SameType {
    using type = T;
};
template <typename... P>
inline hipError_t launch_kernel(void (*kernel)(P...), dim3 grid, dim3 block, hipStream_t s, typename SameType<P>::type... args) {
    void* ptrs[] = {static_cast<void*>(&args)...};
    return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, 0, s);
}

hipError_t launch_prefetch_plan(const PlanArgs& a, hipStream_t s);
hipError_t launch_window_build(const WindowArgs& w, hipStream_t s);
hipError_t launch_decompress_window(const DecodeArgs& a, const WindowArgs& w, int32_t omega, hipStream_t s);
int window_engine_capacity(const Geometry& g);
hipError_t launch_fill_i32(int32_t* p, int32_t v, uint64_t n, hipStream_t s);
hipError_t launch_compress(const EncodeArgs& a, hipStream_t s);
hipError_t launch_decompress(const DecodeArgs& a, hipStream_t s);
hipError_t launch_reset(DevState* st, kvc_desc* desc, uint64_t n_desc, hipStream_t s);
hipError_t launch_set_cursor(DevState* st, uint64_t cursor16, hipStream_t s);
hipError_t launch_stats(DevState* st, const kvc_desc* desc, uint64_t n_desc, hipStream_t s);
hipError_t launch_page_scales(const uint16_t* amax, float* s, float* s_inv, uint64_t n, hipStream_t st);
hipError_t launch_copy(void* dst, const void* src, uint64_t n16, hipStream_t s);

}  // namespace kvc
