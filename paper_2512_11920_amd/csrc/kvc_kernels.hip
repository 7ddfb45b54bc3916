// The small kernels around the codec (pool reset, statistics, yardstick copy, prefetch planner and the
// window's queue builder) and the launchers of every kernel.  The codec kernels themselves -- Algorithm 2
// of the paper and its inverse, Section 3.5.3 -- are the templates of kvc_codec.h, instantiated per page
// shape by kvc_codec.hip and found here through shape_kernels().
#include <algorithm>

#include "kvc_device.h"

namespace kvc {

// ---------------------------------------------------------------------------------- small kernels

__global__ void k_reset(DevState* st, kvc_desc* desc, uint64_t n_desc) {
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i == 0) {
        st->cursor16 = 0;
        st->status = 0;
    }
    for (uint64_t k = i; k < n_desc; k += (uint64_t)gridDim.x * blockDim.x)
        reinterpret_cast<uint4*>(desc)[k] = make_uint4(0, 0, 0, (uint32_t)KVC_MODE_INVALID << 16);
}

__global__ void k_set_cursor(DevState* st, unsigned long long cursor16) {
    if (threadIdx.x == 0) {
        st->cursor16 = cursor16;
        st->status = 0;
    }
}

__global__ void k_stats_zero(DevState* st) {
    if (threadIdx.x < 8) st->stats[threadIdx.x] = 0;
}

__global__ __launch_bounds__(256) void k_stats(DevState* st, const kvc_desc* desc, uint64_t n_desc) {
    __shared__ unsigned long long s_part[4][8];
    unsigned long long cnt[8] = {0, 0, 0, 0, 0, 0, 0, 0};  // pages per mode 0..5, invalid, payload units
    for (uint64_t k = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; k < n_desc; k += (uint64_t)gridDim.x * blockDim.x) {
        const uint32_t w = reinterpret_cast<const uint4*>(desc)[k].w;
        const uint32_t mode = (w >> 16) & 0xFFu;
        if (mode <= KVC_MODE_CHAN) {
            cnt[mode] += 1;
            cnt[7] += w & 0xFFFFu;
        } else {
            cnt[6] += 1;
        }
    }
    // wave reduction, then one atomic per counter per workgroup
    for (int j = 0; j < 8; ++j) {
        unsigned long long v = cnt[j];
        for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
        if (lane_id() == 0) s_part[threadIdx.x >> 6][j] = v;
    }
    __syncthreads();
    if (threadIdx.x < 8) {
        const unsigned long long v = s_part[0][threadIdx.x] + s_part[1][threadIdx.x] + s_part[2][threadIdx.x] + s_part[3][threadIdx.x];
        if (v) atomicAdd(&st->stats[threadIdx.x], v);
    }
}

// Yardstick copy, shaped like the codec's traffic: a wave moves one contiguous 4 KB piece, its four
// 128-bit loads in flight together, then its four stores.
__global__ __launch_bounds__(kThreads) void k_copy(uint4* __restrict__ dst, const uint4* __restrict__ src, uint64_t n16) {
    const uint64_t k0 = ((uint64_t)blockIdx.x * kWavesPerWG + (threadIdx.x >> 6)) * 256u + (threadIdx.x & 63u);
    uint4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
        if (k0 + 64u * u < n16) v[u] = src[k0 + 64u * u];
#pragma unroll
    for (int u = 0; u < 4; ++u)
        if (k0 + 64u * u < n16) dst[k0 + 64u * u] = v[u];
}

// Prefetch planner, Algorithm 1 of the paper without the token predictor: one thread per
// (layer, sequence) walks the k predicted logical blocks in order -- translate through the block
// table (TranslateAddress), skip what is already in L1 or in the L2 prefetch buffer (the residency
// test), otherwise claim a slot of the half being filled and list the pool block for the decode
// launch (IssueDMA).
// Translate prediction j of sequence sq in layer l.  Returns the pool block (>= 0), -1 for "no block",
// -2 for "in L1"; sets bad for indices out of range.
__device__ __forceinline__ int32_t plan_translate(const PlanArgs& a, int32_t l, int32_t sq, int j, bool& bad) {
    const int32_t lb = a.pred[(int64_t)sq * a.k + j];
    if (lb >= a.max_blocks) {
        bad = true;
        return -1;
    }
    if (lb < 0) return -1;
    if (a.l1_first && lb >= a.l1_first[sq]) return -2;  // held in the GPU-local cache
    const int32_t e = a.block_table[(int64_t)sq * a.max_blocks + lb];
    if (e >= a.pool_blocks_per_layer) {
        bad = true;
        return -1;
    }
    if (e < 0) return -1;
    return (int32_t)((int64_t)l * a.pool_blocks_per_layer + e);
}

// KMAX: compile-time bound on k, so that the per-sequence state (wanted blocks, tags of both halves)
// lives in registers and every loop unrolls; all global reads happen once, up front.
template <int KMAX>
__global__ void k_prefetch_plan(PlanArgs a) {
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t n_ls = (int64_t)(a.layer_end - a.layer_begin) * a.n_seq;
    if (idx >= n_ls) return;
    const int32_t l = a.layer_begin + (int32_t)(idx / a.n_seq);
    const int32_t sq = (int32_t)(idx % a.n_seq);
    const int k = a.k;
    const int64_t n_slots = (int64_t)a.n_layers * a.n_seq * k;
    const int64_t base = ((int64_t)l * a.n_seq + sq) * k;
    const int64_t fill0 = (int64_t)a.fill_half * n_slots + base, other0 = (int64_t)(1 - a.fill_half) * n_slots + base;
    bool bad = false;
    int32_t want[KMAX], t_fill[KMAX], t_other[KMAX], fetch[KMAX];
#pragma unroll
    for (int j = 0; j < KMAX; ++j) {
        const bool live = j < k;
        want[j] = live ? plan_translate(a, l, sq, j, bad) : -1;
        t_fill[j] = live ? a.tags[fill0 + j] : -1;
        t_other[j] = live ? a.tags[other0 + j] : -1;
        fetch[j] = -1;
    }
    if (a.policy == 0) {
        // Algorithm 1 as printed: prediction j owns slot j of the half being filled
#pragma unroll
        for (int j = 0; j < KMAX; ++j) {
            const int32_t pb = want[j];
            int64_t where = pb == -2 ? -2 : -1;
            if (pb >= 0) {
#pragma unroll
                for (int j2 = KMAX - 1; j2 >= 0; --j2)  // lowest matching slot wins
                    if (j2 < j && t_fill[j2] == pb) where = fill0 + j2;  // slots already settled in this step
#pragma unroll
                for (int j2 = KMAX - 1; j2 >= 0; --j2)
                    if (t_other[j2] == pb) where = other0 + j2;
                if (where < 0) {
                    where = fill0 + j;
                    if (t_fill[j] != pb) {
                        t_fill[j] = pb;
                        fetch[j] = pb;
                    }
                }
            }
            if (j < k) a.loc[base + j] = (int32_t)where;
        }
    } else {
        // Slot reuse: blocks wanted by this step stay where they are; a block that is in neither half
        // takes the lowest slot whose content this step does not want.
        bool keep[KMAX];
#pragma unroll
        for (int j2 = 0; j2 < KMAX; ++j2) {  // a slot is kept if it is the first one holding a wanted block
            const int32_t t = t_fill[j2];
            bool wanted = false, dup = false;
#pragma unroll
            for (int j = 0; j < KMAX; ++j) wanted = wanted || (t >= 0 && want[j] == t);
#pragma unroll
            for (int j3 = 0; j3 < KMAX; ++j3) dup = dup || (j3 < j2 && t >= 0 && t_fill[j3] == t);
            keep[j2] = (wanted && !dup) || j2 >= k;  // slots beyond k do not exist: never claimable
        }
#pragma unroll
        for (int j = 0; j < KMAX; ++j) {
            const int32_t pb = want[j];
            int64_t where = pb == -2 ? -2 : -1;
            if (pb >= 0) {
#pragma unroll
                for (int j2 = KMAX - 1; j2 >= 0; --j2)
                    if (keep[j2] && j2 < k && t_fill[j2] == pb) where = fill0 + j2;
#pragma unroll
                for (int j2 = KMAX - 1; j2 >= 0; --j2)
                    if (t_other[j2] == pb) where = other0 + j2;
                if (where < 0) {
                    int free_slot = -1;
#pragma unroll
                    for (int j2 = KMAX - 1; j2 >= 0; --j2)
                        if (!keep[j2]) free_slot = j2;
#pragma unroll
                    for (int j2 = 0; j2 < KMAX; ++j2)
                        if (j2 == free_slot) {  // claim it: it now holds a wanted block
                            keep[j2] = true;
                            t_fill[j2] = pb;
                            fetch[j2] = pb;
                        }
                    where = fill0 + free_slot;
                }
            }
            if (j < k) a.loc[base + j] = (int32_t)where;
        }
    }
#pragma unroll
    for (int j = 0; j < KMAX; ++j)
        if (j < k) {
            a.fetch[base + j] = fetch[j];
            if (fetch[j] >= 0) a.tags[fill0 + j] = t_fill[j];
        }
    if (bad) atomicOr(&a.st->status, KVC_ST_BAD_INDEX);
}

// Opens the outstanding-request window of a prefetch call: the transfers the planner issued (entries
// >= 0 of the call's part of the fetch list) are queued in issue order -- layer, sequence, slot -- each
// layer's count becomes its pending counter, and the notification words are reset: a layer with nothing
// to transfer is ready at once, the others when their last transfer completes.  Two launches, one
// workgroup per layer each: count, then place (a layer's entries begin where the layers before it end).
__global__ __launch_bounds__(256) void k_window_count(WindowArgs w) {
    __shared__ uint32_t s_cnt[4];
    const int l = blockIdx.x;
    uint32_t n = 0;
    for (int i = threadIdx.x; i < w.per_layer; i += 256) n += w.fetch[(int64_t)l * w.per_layer + i] >= 0 ? 1u : 0u;
    n = wave_incl_scan_dpp(n);
    if (lane_id() == 63) s_cnt[threadIdx.x >> 6] = n;
    __syncthreads();
    if (threadIdx.x == 0) w.pending[l] = (int32_t)(s_cnt[0] + s_cnt[1] + s_cnt[2] + s_cnt[3]);
}

__global__ __launch_bounds__(256) void k_window_place(WindowArgs w) {
    __shared__ uint32_t s_cnt[4];
    __shared__ uint32_t s_sum[2][4];
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int l = blockIdx.x;
    const long long now = max(wall_clock64(), 1ll);
    // entries of the layers before this one, and of all layers
    uint32_t before_l = 0, all_l = 0;
    for (int j = threadIdx.x; j < w.n_layers_call; j += 256) {
        const uint32_t c = (uint32_t)w.pending[j];
        before_l += j < l ? c : 0u;
        all_l += c;
    }
    before_l = wave_incl_scan_dpp(before_l);
    all_l = wave_incl_scan_dpp(all_l);
    if (lane == 63) {
        s_sum[0][wave] = before_l;
        s_sum[1][wave] = all_l;
    }
    __syncthreads();
    const uint32_t base = s_sum[0][0] + s_sum[0][1] + s_sum[0][2] + s_sum[0][3];
    const uint32_t total = s_sum[1][0] + s_sum[1][1] + s_sum[1][2] + s_sum[1][3];
    uint32_t in_layer = 0;  // entries of this layer placed so far (workgroup-uniform)
    for (int c0 = 0; c0 < w.per_layer; c0 += 256) {
        const int i = c0 + (int)threadIdx.x;
        const bool live = i < w.per_layer && w.fetch[(int64_t)l * w.per_layer + i] >= 0;
        const uint64_t m = __builtin_amdgcn_ballot_w64(live);
        __syncthreads();  // the counts of the chunk before have been read
        if (lane == 0) s_cnt[wave] = (uint32_t)__builtin_popcountll(m);
        __syncthreads();
        uint32_t before = 0, all = 0;
        for (int k = 0; k < 4; ++k) {
            before += k < wave ? s_cnt[k] : 0u;
            all += s_cnt[k];
        }
        if (live) w.queue[base + in_layer + before + __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u))] = l * w.per_layer + i;
        in_layer += all;
    }
    if (threadIdx.x == 0) {
        w.notify[w.layer_begin + l] = in_layer ? 0ll : now;
        if (l == 0) {
            // Engines at work: at most omega, at most one per transfer -- and beyond 256 of them only as far
            // as each still has eight transfers to carry out: every turn of every engine is three atomics on
            // shared counters, and a short queue spread over a thousand engines spends its time there
            // (5,120 transfers: 0.51 ms with 1,024 engines, 0.33 ms with 256).
            unsigned int engines = min(total, (uint32_t)w.omega);
            if (engines > 256u) engines = min(engines, max(256u, total / 8u));
            w.hdr->n_issued = total;
            w.hdr->engines = engines;
            // entries per turn: long queues space out the bookkeeping, short ones keep every engine busy
            w.hdr->chunk = engines ? min(max(total / (4u * engines), 1u), 8u) : 1u;
            w.hdr->ticket = 0;
            w.hdr->done = 0;
            w.notify[w.n_layers] = now;                        // window opened
            w.notify[w.n_layers + 1] = (long long)total;       // transfers issued
            w.notify[w.n_layers + 2] = (long long)engines;     // engines at work: the bound on blocks in flight
            w.notify[w.n_layers + 3] = total ? 0ll : now;      // all complete
        }
    }
}

__global__ void k_fill_i32(int32_t* p, int32_t v, uint64_t n) {
    for (uint64_t k = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; k < n; k += (uint64_t)gridDim.x * blockDim.x) p[k] = v;
}

// The encoder's scale arithmetic for a list of page maxima (FP16 bit patterns); 0, Inf and NaN
// patterns give s = s_inv = 0, as the encoder never scales such pages.
__global__ void k_page_scales(const uint16_t* amax, float* s, float* s_inv, uint64_t n) {
    const uint64_t k = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= n) return;
    const uint32_t m = amax[k] & 0x7FFFu;
    PageScale ps;
    ps.s = ps.s_inv = 0.0f;
    if (m != 0 && m < 0x7C00u) ps = page_scale(m);
    s[k] = ps.s;
    s_inv[k] = ps.s_inv;
}

// ---------------------------------------------------------------------------------- launchers

// the kernels of a page shape: the exact instantiation when there is one, else the one that reads the
// token count at run time
const ShapeKernels* shape_kernels(int N, int d) {
    static const ShapeLookup groups[kShapeGroups] = {
        shape_kernels_group0, shape_kernels_group1, shape_kernels_group2,  shape_kernels_group3,  shape_kernels_group4,  shape_kernels_group5,
        shape_kernels_group6, shape_kernels_group7, shape_kernels_group8,  shape_kernels_group9,  shape_kernels_group10, shape_kernels_group11,
        shape_kernels_group12, shape_kernels_group13, shape_kernels_group14, shape_kernels_group15};
    if (N < 1 || d < 32 || d > 256 || d % 32 != 0 || (int64_t)N * d > 4096) return nullptr;
    const int E = N * d, np = (E + 511) / 512;
    for (int partial = E == np * 512 ? 0 : 1; partial < 2; ++partial)
        for (ShapeLookup f : groups)
            if (const ShapeKernels* k = f(d, np, partial != 0)) return k;
    return nullptr;
}

hipError_t launch_compress(const EncodeArgs& a, hipStream_t s) {
    if (a.n_pages == 0) return hipSuccess;
    const ShapeKernels* f = shape_kernels(a.g.N, a.g.d);
    return f ? f->compress(a, s) : hipErrorInvalidValue;
}

hipError_t launch_decompress(const DecodeArgs& a, hipStream_t s) {
    if (a.n_pages == 0) return hipSuccess;
    const ShapeKernels* f = shape_kernels(a.g.N, a.g.d);
    return f ? f->decompress(a, s) : hipErrorInvalidValue;
}

hipError_t launch_prefetch_plan(const PlanArgs& a, hipStream_t s) {
    const int64_t n = (int64_t)(a.layer_end - a.layer_begin) * a.n_seq;
    if (n <= 0) return hipSuccess;
    const dim3 grid((unsigned)((n + 63) / 64)), block(64);
    if (a.k <= 8) return launch_kernel(k_prefetch_plan<8>, grid, block, s, a);
    if (a.k <= 16) return launch_kernel(k_prefetch_plan<16>, grid, block, s, a);
    return launch_kernel(k_prefetch_plan<kMaxPrefetchK>, grid, block, s, a);
}

hipError_t launch_window_build(const WindowArgs& w, hipStream_t s) {
    if (w.n_layers_call <= 0) return hipSuccess;
    const hipError_t e = launch_kernel(k_window_count, dim3((unsigned)w.n_layers_call), dim3(256), s, w);
    if (e != hipSuccess) return e;
    return launch_kernel(k_window_place, dim3((unsigned)w.n_layers_call), dim3(256), s, w);
}

// At most omega workgroups, one block in flight each; the queue may turn out shorter than the grid, in
// which case the surplus workgroups leave at their first look.
hipError_t launch_decompress_window(const DecodeArgs& a, const WindowArgs& w, int32_t omega, hipStream_t s) {
    if (w.n_now <= 0) return hipSuccess;
    const unsigned grid = (unsigned)std::min<int64_t>(omega, w.n_now);
    const ShapeKernels* f = shape_kernels(a.g.N, a.g.d);
    return f ? f->decompress_window(a, w, grid, s) : hipErrorInvalidValue;
}

int window_engine_capacity(const Geometry& g) {
    const ShapeKernels* f = shape_kernels(g.N, g.d);
    return f ? f->window_capacity() : 0;
}

hipError_t launch_fill_i32(int32_t* p, int32_t v, uint64_t n, hipStream_t s) {
    if (n == 0) return hipSuccess;
    const unsigned blocks = (unsigned)std::min<uint64_t>((n + 255) / 256, 4096);
    return launch_kernel(k_fill_i32, dim3(blocks), dim3(256), s, p, v, n);
}

hipError_t launch_reset(DevState* st, kvc_desc* desc, uint64_t n_desc, hipStream_t s) {
    const unsigned blocks = (unsigned)std::min<uint64_t>(std::max<uint64_t>((n_desc + 255) / 256, 1), 65536);
    return launch_kernel(k_reset, dim3(blocks), dim3(256), s, st, desc, n_desc);
}

hipError_t launch_set_cursor(DevState* st, uint64_t cursor16, hipStream_t s) {
    return launch_kernel(k_set_cursor, dim3(1), dim3(64), s, st, (unsigned long long)cursor16);
}

hipError_t launch_stats(DevState* st, const kvc_desc* desc, uint64_t n_desc, hipStream_t s) {
    const hipError_t e = launch_kernel(k_stats_zero, dim3(1), dim3(64), s, st);
    if (e != hipSuccess || n_desc == 0) return e;
    const unsigned blocks = (unsigned)std::min<uint64_t>((n_desc + 255) / 256, 2048);
    return launch_kernel(k_stats, dim3(blocks), dim3(256), s, st, desc, n_desc);
}

hipError_t launch_page_scales(const uint16_t* amax, float* s, float* s_inv, uint64_t n, hipStream_t st) {
    if (n == 0) return hipSuccess;
    return launch_kernel(k_page_scales, dim3((unsigned)((n + 255) / 256)), dim3(256), st, amax, s, s_inv, n);
}

hipError_t launch_copy(void* dst, const void* src, uint64_t n16, hipStream_t s) {
    if (n16 == 0) return hipSuccess;
    const uint64_t per_wg = 256u * kWavesPerWG;  // 16-byte units per workgroup
    const uint64_t blocks = (n16 + per_wg - 1) / per_wg;
    if (blocks >= (1ull << 24)) return hipErrorInvalidValue;  // fewer than 2^24 workgroups of 256 threads: the launch stays below 2^32 threads
    return launch_kernel(k_copy, dim3((unsigned)blocks), dim3(kThreads), s, reinterpret_cast<uint4*>(dst), reinterpret_cast<const uint4*>(src), n16);
}

}  // namespace kvc
