// Device-side helpers shared by the kernel files: wave64 primitives (DPP), page-task resolution,
// pool reservation and copy-out.
#pragma once
#include "kvc_common.h"

namespace kvc {

// payloads are written to the pool once and not read back by the encoder: non-temporal stores
#ifndef KVC_NT_POOL_STORE
#define KVC_NT_POOL_STORE 1
#endif

// Debug build (-DKVC_DEBUG_BOUNDS=1): every LDS slot index and pool span the kernels compute is checked
// against its bounds; a violation sets status bit 8 instead of being executed silently.  Off by default.
#ifndef KVC_DEBUG_BOUNDS
#define KVC_DEBUG_BOUNDS 0
#endif
#if KVC_DEBUG_BOUNDS
#define KVC_CHECK(st, cond)                        \
    do {                                           \
        if (!(cond)) atomicOr(&(st)->status, 8u);  \
    } while (0)
#else
#define KVC_CHECK(st, cond) \
    do {                    \
    } while (0)
#endif

constexpr int kWavesPerWG = 4;
constexpr int kThreads = kWavesPerWG * 64;

// LDS bytes reserved for one page's payload under construction: header + bodies can reach
// E + E/64 bytes before the INT8 fallback is chosen, plus slack for the 3-dword body writes.
template <int MAXP>
struct Slot {
    static constexpr int kBytes = ((MAXP * 520 + 16 + 15) / 16) * 16;
    static constexpr int kWords = kBytes / 4;
};

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }

// Lanes of one wave exchange data through LDS: keep the compiler from moving accesses across.
__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// DPP data movement.  CTRL: 0x00-0xFF quad_perm, 0x110+n row_shr:n, 0x100+n row_shl:n,
// 0x140 row_mirror, 0x141 row_half_mirror, 0x142 row_bcast:15, 0x143 row_bcast:31.
// Lanes whose source is outside the row, or whose row is not in ROW_MASK, receive `old`.
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ uint32_t dpp(uint32_t old, uint32_t src) {
    return (uint32_t)__builtin_amdgcn_update_dpp((int)old, (int)src, CTRL, ROW_MASK, 0xF, false);
}

// max over the wave, result uniform (read from lane 63)
__device__ __forceinline__ uint32_t wave_max_dpp(uint32_t v) {
    v = max(v, dpp<0xB1>(0, v));        // quad_perm [1,0,3,2]
    v = max(v, dpp<0x4E>(0, v));        // quad_perm [2,3,0,1]
    v = max(v, dpp<0x141>(0, v));       // row_half_mirror
    v = max(v, dpp<0x140>(0, v));       // row_mirror: every lane holds its row's max
    v = max(v, dpp<0x142, 0xA>(0, v));  // rows 1,3 take lane 15 of the row before
    v = max(v, dpp<0x143, 0xC>(0, v));  // rows 2,3 take lane 31
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

// inclusive prefix sum over the 64 lanes
__device__ __forceinline__ uint32_t wave_incl_scan_dpp(uint32_t v) {
    v += dpp<0x111>(0, v);
    v += dpp<0x112>(0, v);
    v += dpp<0x114>(0, v);
    v += dpp<0x118>(0, v);
    v += dpp<0x142, 0xA>(0, v);
    v += dpp<0x143, 0xC>(0, v);
    return v;
}

// inclusive prefix sum over quads of a value that is uniform within each quad of lanes
__device__ __forceinline__ uint32_t quad_incl_scan_dpp(uint32_t v) {
    v += dpp<0x114>(0, v);
    v += dpp<0x118>(0, v);
    v += dpp<0x142, 0xA>(0, v);
    v += dpp<0x143, 0xC>(0, v);
    return v;
}

// inclusive prefix sum within each row of 16 lanes
__device__ __forceinline__ uint32_t row16_incl_scan_dpp(uint32_t v) {
    v += dpp<0x111>(0, v);
    v += dpp<0x112>(0, v);
    v += dpp<0x114>(0, v);
    v += dpp<0x118>(0, v);
    return v;
}

// ---- bit strings wider than 32 bits, handled as 32-bit halves --------------------------------
// No 64-bit shift by a register amount may appear in these kernels.  What was observed: one build of one
// encoder instantiation (256 channels, run-time scheme, exactly 128 VGPRs) wrote wrong body bytes for a
// few pages in a thousand, differently on every launch, only when two or more workgroups shared a compute
// unit, and every recompile that moved registers made the fault vanish.  That build held the count of a
// v_lshlrev_b64 in the last VGPR of its allocation; the working hypothesis is that v_lshlrev_b64 /
// v_lshrrev_b64 misread a count held there when another wave shares the SIMD.  The cause was not
// established beyond that (a compiler or occupancy-dependent fault in that one build fits the same
// symptoms).  The rule is harmless either way: packing and unpacking below use 32-bit shifts, funnel
// shifts and byte permutes only; a test scans the generated code for 64-bit shifts by a vector register, and
// the guard that matters is the test that runs every kernel instantiation at full occupancy against
// the CPU reference.

// u[0..7], each below 2^c with 0 <= c <= 8, as one little-endian bit string of 8c bits: x = low 32
// bits, y = the rest.  (c = 9, a run packet, gives a value the caller discards.)
__device__ __forceinline__ uint2 pack8_bits(const uint32_t (&u)[8], uint32_t c) {
    const uint32_t a01 = u[0] | (u[1] << c), a23 = u[2] | (u[3] << c);
    const uint32_t a45 = u[4] | (u[5] << c), a67 = u[6] | (u[7] << c);
    const uint32_t c2 = c << 1;
    const uint32_t b0 = a01 | (a23 << c2), b1 = a45 | (a67 << c2);  // 4c bits each
    // b1 << 4c over 64 bits is (b1 : 0) funnel-shifted right by 32 - 4c; 4c = 32 gives (b1 : 0) itself,
    // and 4c = 0 only occurs with b1 = 0.  The funnel shift reads its amount mod 32, so -4c will do.
    const uint32_t r = (uint32_t)__mul24((int)c, -4);
    return make_uint2(b0 | __builtin_amdgcn_alignbit(b1, 0u, r), __builtin_amdgcn_alignbit(0u, b1, r));
}

// The three dwords of (W.y : W.x) << 8k, k = B mod 4: one byte permute each with a common selector
// {7-k, 6-k, 5-k, 4-k}, which is the byte string 08 07 .. 01 shifted right by 3 - k bytes (the byte
// funnel shift reads its amount mod 4, so ~B will do).
__device__ __forceinline__ void shl_bytes(uint2 W, uint32_t B, uint32_t& d0, uint32_t& d1, uint32_t& d2) {
    const uint32_t sel = __builtin_amdgcn_alignbyte(0x08070605u, 0x04030201u, ~B);
    d0 = __builtin_amdgcn_perm(W.x, 0u, sel);
    d1 = __builtin_amdgcn_perm(W.y, W.x, sel);
    d2 = __builtin_amdgcn_perm(0u, W.y, sel);
}

// Low 32 bits of (hi : lo) >> 4c for 1 <= c <= 8.
__device__ __forceinline__ uint32_t shr_nibbles(uint32_t lo, uint32_t hi, uint32_t c) {
    const uint32_t v = __builtin_amdgcn_alignbit(hi, lo, c << 2);  // the shift is taken mod 32
    return c == 8u ? hi : v;
}

// element offset of a page inside a cache buffer
__device__ __forceinline__ int64_t page_base(const Geometry& g, int64_t blk, int pg) {
    return blk * g.block_stride + (int64_t)pg * g.page_stride;
}

// element offset, relative to the page base, of dense element index e (token e/d, channel e%d); d is
// any multiple of 32, the quotient comes from a multiplication (checked for every e when a context is made)
__device__ __forceinline__ int64_t elem_off(const Geometry& g, int e) {
    const uint32_t row = ((uint32_t)e * g.d_magic) >> 22;
    return (int64_t)row * g.row_stride + ((uint32_t)e - row * (uint32_t)g.d);
}

// Workgroup index used for task assignment.  Workgroups are dealt round-robin to the 8 XCDs, so with
// the identity deal (MODE 0) XCD k works on the tasks whose index is k modulo 8 for the whole launch: all
// XCDs sweep the buffers side by side, 16 KB apart.  MODE 1 gives each XCD one contiguous eighth of the
// tasks instead, so that it streams through a region of its own.  Measured on the 21 GB cache: the
// decoder's time falls into one of two clusters from process to process whatever the deal (the buffers'
// placement by the driver decides: this GPU's HBM behaves as three regions of about 96 GB, and any kernel,
// a plain copy too, runs 4-7 % slower when it reads and writes inside one of them than when it reads from
// one and writes to another); with MODE 1 the clusters are 5.0 and 5.45 ms,
// with MODE 0 5.15 and 5.45 ms, and the decode-gather step gains 7 %.  The encoder is 1-2 % faster with
// MODE 0.  (Also tried, without gain for either kernel: rotating the tasks inside every run of eight
// workgroups, shifting all tasks by a workgroup, runs of 3 to 4099 tasks per XCD in turn, and eighths
// entered at staggered points.)
template <int MODE>
__device__ __forceinline__ unsigned task_block_index() {
    const unsigned b = blockIdx.x;
    if (MODE == 1) {
        const unsigned q = gridDim.x >> 3;
        return b < (q << 3) ? (b & 7u) * q + (b >> 3) : b;
    }
    return b;
}

// A value every lane of the wave holds the same copy of, moved to scalar registers: index arithmetic
// on it (64-bit multiplies, bounds checks) then runs on the scalar unit, loads indexed by it become
// scalar loads, and an access at kernel-argument pointer + such an offset needs no per-lane base.
__device__ __forceinline__ int32_t wave_uniform(int32_t v) { return __builtin_amdgcn_readfirstlane(v); }

__device__ __forceinline__ int64_t wave_uniform(int64_t v) {
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((uint64_t)v >> 32));
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

// Scaling step of Algorithm 2 for a page whose largest magnitude is the finite, non-zero FP16 value
// with bit pattern m: s = amax / 127 and s_inv = 1 / s, each the correctly rounded binary32 quotient,
// without the general division sequence.  amax / 127 is the product with the correctly rounded
// reciprocal of 127, its exact FMA residual and one corrected FMA (Markstein's construction); 1 / s is
// the hardware reciprocal (within 1 ulp) and one Newton step on the FMA residual.  Neither binary32
// range can under- or overflow here (2^-24 <= amax <= 65504).  The domain is the 31,743 FP16
// magnitudes: kvc_page_scales exposes this function so that a test compares every one of them with
// plain IEEE division.
struct PageScale {
    float s, s_inv;
};

__device__ __forceinline__ PageScale page_scale(uint32_t m) {
    const float a = (float)__builtin_bit_cast(_Float16, (unsigned short)m);
    constexpr float kInv127 = 1.0f / 127.0f;
    const float q0 = a * kInv127;
    const float r = __builtin_fmaf(-q0, 127.0f, a);
    PageScale ps;
    ps.s = __builtin_fmaf(r, kInv127, q0);
    const float y0 = __builtin_amdgcn_rcpf(ps.s);
    const float e = __builtin_fmaf(-ps.s, y0, 1.0f);
    ps.s_inv = __builtin_fmaf(e, y0, y0);
    return ps;
}

struct PageResult {
    uint32_t n16;  // payload size in 16-byte units (0 = page skipped)
    uint32_t mode;
    float scale;
};

// Page task of the encoder: which source page, which descriptor.
struct EncTask {
    long long desc_idx;  // -1: nothing to do
    long long src_off;   // element offset of the source page in the cache buffer
    int scheme;          // mode requested for this page
};

// Position of a wave's first page task as (block, page in block); later tasks advance it by one page.
// A wave works on one page at a time, so positions and everything derived from them are wave-uniform.
struct TaskPos {
    int64_t blk;
    int pg;
};

// The host bounds the pages of one call well below 2^31, so task indices divide in 32 bits.
__device__ __forceinline__ TaskPos task_pos(int64_t t, int ppb) {
    TaskPos r;
    const uint32_t blk = (uint32_t)t / (uint32_t)ppb;
    r.pg = wave_uniform((int32_t)((uint32_t)t - blk * (uint32_t)ppb));
    r.blk = (int64_t)(uint32_t)wave_uniform((int32_t)blk);
    return r;
}

__device__ __forceinline__ void task_advance(TaskPos& p, int ppb) {
    if (++p.pg == ppb) {
        p.pg = 0;
        ++p.blk;
    }
}

// max_mode: the highest mode a per-block request may name for this page shape (higher values are read as it)
__device__ __forceinline__ EncTask resolve_enc_task(const EncodeArgs& a, int64_t t, const TaskPos& pos, int max_mode = KVC_MODE_PACK) {
    EncTask r;
    r.desc_idx = -1;
    r.src_off = -1;
    r.scheme = a.scheme;
    if (t >= a.n_pages) return r;
    const int ppb = a.g.ppb;
    const int64_t blk = pos.blk;
    const int pg = pos.pg;
    const int64_t sb = a.src_ids ? (int64_t)wave_uniform(a.src_ids[blk]) : blk;
    const int64_t pb = a.pool_ids ? (int64_t)wave_uniform(a.pool_ids[blk]) : blk;
    if (sb < 0 || pb < 0) return r;
    const uint64_t d_idx = (uint64_t)pb * (uint64_t)ppb + (uint64_t)pg;
    if (sb >= a.n_cache_blocks || d_idx >= a.n_desc) {
        if (lane_id() == 0) atomicOr(&a.st->status, KVC_ST_BAD_INDEX);
        return r;
    }
    r.src_off = page_base(a.g, sb, pg);
    r.desc_idx = (long long)d_idx;
    if (a.block_scheme) r.scheme = min(wave_uniform((int32_t)a.block_scheme[blk]), (int32_t)max_mode);
    return r;
}

// Page task of the decoder.  kind: 0 skip, 1 decode desc_idx into dst, 2 zero-fill dst (bad index).
struct DecTask {
    int kind;
    uint64_t desc_idx;
    uint16_t* dst;
};

// Second half of the resolution: pool block pb (< 0: nothing stored there) into output block db.
__device__ __forceinline__ DecTask place_dec_task(const DecodeArgs& a, int64_t pb, int64_t db, int pg, bool bad_index) {
    DecTask r;
    r.kind = 0;
    r.desc_idx = 0;
    r.dst = nullptr;
    const Geometry& g = a.g;
    if (db < 0 || db >= a.n_out_blocks) {
        if (db >= 0 && lane_id() == 0) atomicOr(&a.st->status, KVC_ST_BAD_INDEX);
        return r;
    }
    r.dst = a.out + page_base(g, db, pg);
    if (!bad_index && pb < 0) return r;  // skip
    r.desc_idx = (uint64_t)pb * (uint64_t)g.ppb + (uint64_t)pg;
    if (bad_index || r.desc_idx >= a.n_desc) {
        if (lane_id() == 0) atomicOr(&a.st->status, KVC_ST_BAD_INDEX);
        r.kind = 2;
        return r;
    }
    r.kind = 1;
    return r;
}

__device__ __forceinline__ DecTask resolve_dec_task(const DecodeArgs& a, int64_t t, const TaskPos& pos) {
    if (t >= a.n_pages) {
        DecTask r;
        r.kind = 0;
        r.desc_idx = 0;
        r.dst = nullptr;
        return r;
    }
    const int64_t blk = pos.blk;
    int64_t pb, db;
    bool bad_index = false;
    if (a.block_table) {  // translate (layer, sequence, predicted logical block) -> pool block
        const uint32_t per_layer = (uint32_t)a.n_seq * (uint32_t)a.k;  // blocks of one call fit 31 bits
        const uint32_t layer_u = (uint32_t)blk / per_layer;
        const uint32_t sj = (uint32_t)blk - layer_u * per_layer;
        const int64_t sq = sj / (uint32_t)a.k;
        const int64_t layer = layer_u;
        const int32_t lb = wave_uniform(a.pred[sj]);
        db = blk;
        pb = -1;
        if (lb >= a.max_blocks) {
            bad_index = true;
        } else if (lb >= 0) {
            const int32_t e = wave_uniform(a.block_table[sq * a.max_blocks + lb]);
            if (e >= a.pool_blocks_per_layer)
                bad_index = true;
            else if (e >= 0)
                pb = layer * a.pool_blocks_per_layer + e;
        }
    } else {
        pb = a.pool_ids ? (int64_t)wave_uniform(a.pool_ids[blk]) : blk;
        db = a.dst_ids ? (int64_t)wave_uniform(a.dst_ids[blk]) : blk;
    }
    return place_dec_task(a, pb, db, pos.pg, bad_index);
}

__device__ __forceinline__ void zero_page(uint16_t* dst, const Geometry& g) {
    for (int o = lane_id(); o < (g.E >> 3); o += 64)
        *reinterpret_cast<uint4*>(dst + elem_off(g, o * 8)) = make_uint4(0, 0, 0, 0);
}

// Per-workgroup bookkeeping of the encoder: results of the pages staged in LDS.
template <int SLOTS>
struct EncBook {
    uint32_t n16[SLOTS];
    uint32_t mode[SLOTS];
    float scale[SLOTS];
    unsigned long long off16[SLOTS];
    long long desc[SLOTS];
    long long srcoff[SLOTS];
};

// One thread reserves a contiguous pool span for all staged pages of the workgroup with a single
// atomic on the pool cursor and hands each page its offset; pages that do not fit become INVALID.
template <int SLOTS>
__device__ __forceinline__ void reserve_pool_span(const EncodeArgs& a, EncBook<SLOTS>& b) {
    uint32_t tot = 0;  // at most SLOTS * 512 units
    for (int k = 0; k < SLOTS; ++k) tot += b.n16[k];
    const unsigned long long base = tot ? atomicAdd(&a.st->cursor16, (unsigned long long)tot) : 0ull;
    const bool all_fit = base + tot <= a.pool_units;
    uint32_t rel = 0;
    for (int k = 0; k < SLOTS; ++k) {
        const uint32_t n = b.n16[k];
        if (!all_fit && n && base + rel + n > a.pool_units) b.mode[k] = KVC_MODE_INVALID;
        b.off16[k] = base + rel;
        rel += n;
    }
    if (!all_fit) atomicOr(&a.st->status, KVC_ST_POOL_FULL);
}

// A wave moves one staged payload (or, for RAW, the source page) to its pool span and writes the
// 16-byte descriptor.
template <int SLOTS>
__device__ __forceinline__ void emit_page(const EncodeArgs& a, const EncBook<SLOTS>& b, int slot, const uint32_t* stage) {
    const long long di = b.desc[slot];
    if (di < 0) return;
    const int lane = lane_id();
    const uint32_t mode = b.mode[slot];
    const uint32_t n16 = b.n16[slot];
    const unsigned long long off16 = b.off16[slot];
    if (mode != KVC_MODE_INVALID) {
        KVC_CHECK(a.st, off16 + n16 <= a.pool_units && (size_t)n16 * 16 <= sizeof(uint32_t) * Slot<8>::kWords * 2);
        uint4* dst = reinterpret_cast<uint4*>(a.pool) + off16;
        if (mode == KVC_MODE_RAW) {  // the payload is the dense page
            const uint16_t* srcp = a.cache + b.srcoff[slot];
            for (uint32_t o = lane; o < n16; o += 64) dst[o] = *reinterpret_cast<const uint4*>(srcp + elem_off(a.g, (int)o * 8));
        } else {
            const uint4* srcp = reinterpret_cast<const uint4*>(stage);
#if KVC_NT_POOL_STORE
            typedef uint32_t u4v __attribute__((ext_vector_type(4)));
            for (uint32_t o = lane; o < n16; o += 64) {
                const uint4 v = srcp[o];
                u4v w;
                w.x = v.x; w.y = v.y; w.z = v.z; w.w = v.w;
                __builtin_nontemporal_store(w, reinterpret_cast<u4v*>(dst + o));
            }
#else
            for (uint32_t o = lane; o < n16; o += 64) dst[o] = srcp[o];
#endif
        }
    }
    if (lane == 0) {
        uint4 dw;
        if (mode == KVC_MODE_INVALID) {
            dw = make_uint4(0, 0, 0, (uint32_t)KVC_MODE_INVALID << 16);
        } else {
            const unsigned long long off = off16 * 16ull;
            dw = make_uint4((uint32_t)off, (uint32_t)(off >> 32), __float_as_uint(b.scale[slot]), n16 | (mode << 16));
        }
        reinterpret_cast<uint4*>(a.desc)[di] = dw;
    }
}

// ---- outstanding-request window (Algorithm 1, WaitCompletion over at most Omega_max transfers) ----
// A workgroup is one transfer engine: it takes the next entry of the issue queue, decodes that block,
// reports completion and takes the next.  The grid has at most Omega workgroups, so never more than
// Omega blocks are in flight; every workgroup leaves as soon as the queue is exhausted.

// What an engine holds between two turns: a run of consecutive queue entries.
struct WindowTurn {
    uint32_t first;  // index of the first queue entry
    uint32_t count;  // entries in the run; 0 = the queue is exhausted, the engine leaves
};

// One turn of an engine: report the blocks of the run `done` as complete -- make them visible, count
// them, stamp the layers and the call whose last transfer was among them -- and take the next run of up
// to hdr->chunk queue entries.  Called by all threads of the workgroup; `s_turn` is two words of LDS.
// An engine decodes the blocks of its run one after the other, so it still holds one block in flight; the
// run only spaces out the bookkeeping, whose device-wide release (a write-back of the XCD's L2) and
// same-address atomics cost more than decoding a block when paid per block.
// Thread 0 does the bookkeeping between two barriers, so the single-lane region lies inside the loop
// body and not across its back edge, and the result comes back in scalar registers: the engines' loop
// and its exit branch on the scalar unit and every wave meets every barrier with all of its lanes.  (With
// the single-lane work at both ends of the loop body the compiler merges it across the back edge into
// an outer loop and lets the other lanes run ahead to the next barrier: the workgroup then never
// meets.)
__device__ __forceinline__ WindowTurn window_next(const WindowArgs& w, uint32_t* s_turn, WindowTurn done) {
    // every wave's stores have reached the XCD's L2 before the workgroup meets ...
    if (done.count) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __syncthreads();
    if (threadIdx.x == 0) {
        const long long finished = max(wall_clock64(), 1ll);  // read before the blocks are counted
        const unsigned int n_issued = w.hdr->n_issued;
        unsigned int dn = 0;
        if (done.count) {
            // ... and one device-wide release publishes them before the counters move
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
            uint32_t i = 0;
            while (i < done.count) {  // the run's entries are in layer order: one decrement per layer met
                const int32_t l_rel = w.queue[done.first + i] / w.per_layer;
                uint32_t n = 1;
                while (i + n < done.count && w.queue[done.first + i + n] / w.per_layer == l_rel) ++n;
                if (atomicSub(&w.pending[l_rel], (int)n) == (int)n)
                    __hip_atomic_store(&w.notify[w.layer_begin + l_rel], finished, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
                i += n;
            }
            dn = atomicAdd(&w.hdr->done, done.count) + done.count;
        }
        const unsigned int chunk = w.hdr->chunk;
        const unsigned int t = atomicAdd(&w.hdr->ticket, chunk);
        // WaitCompletion returns: NotifyGPU(ready).  This clock is read after the last block was counted
        // and every layer stamp before its block was: the stamp is the latest of the call.
        if (done.count && dn == n_issued)
            __hip_atomic_store(&w.notify[w.n_layers + 3], max(wall_clock64(), 1ll), __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        s_turn[0] = t;
        s_turn[1] = t < n_issued ? min(chunk, n_issued - t) : 0u;
    }
    __syncthreads();
    WindowTurn r;
    r.first = (uint32_t)__builtin_amdgcn_readfirstlane((int)s_turn[0]);
    r.count = (uint32_t)__builtin_amdgcn_readfirstlane((int)s_turn[1]);
    return r;
}

// The codec kernels are specialised at compile time for the page shape (kvc_codec.h): d channels, np
// passes of 512 elements, and whether the page fills its last pass (exact: d * N = 512 * np) or not
// (partial: the token count N is read at run time).  These are the host-side entry points of one shape.
// The shapes are compiled in groups (kvc_codec.hip), one lookup function per group; shape_kernels() finds
// the set for N tokens x d channels (nullptr: N * d exceeds eight passes).
struct ShapeKernels {
    int d, np;
    bool partial;
    hipError_t (*compress)(const EncodeArgs& a, hipStream_t s);
    hipError_t (*decompress)(const DecodeArgs& a, hipStream_t s);
    hipError_t (*decompress_window)(const DecodeArgs& a, const WindowArgs& w, unsigned grid, hipStream_t s);
    int (*window_capacity)();  // window engines resident on the current device at once (0: unknown)
};
constexpr int kShapeGroups = 16;
using ShapeLookup = const ShapeKernels* (*)(int d, int np, bool partial);
#define KVC_DECLARE_GROUP(G) const ShapeKernels* shape_kernels_group##G(int d, int np, bool partial);
KVC_DECLARE_GROUP(0) KVC_DECLARE_GROUP(1) KVC_DECLARE_GROUP(2) KVC_DECLARE_GROUP(3) KVC_DECLARE_GROUP(4) KVC_DECLARE_GROUP(5)
KVC_DECLARE_GROUP(6) KVC_DECLARE_GROUP(7) KVC_DECLARE_GROUP(8) KVC_DECLARE_GROUP(9) KVC_DECLARE_GROUP(10) KVC_DECLARE_GROUP(11)
KVC_DECLARE_GROUP(12) KVC_DECLARE_GROUP(13) KVC_DECLARE_GROUP(14) KVC_DECLARE_GROUP(15)
#undef KVC_DECLARE_GROUP
const ShapeKernels* shape_kernels(int N, int d);

}  // namespace kvc
