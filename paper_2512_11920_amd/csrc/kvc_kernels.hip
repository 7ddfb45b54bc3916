// HIP kernels of the KV page codec for gfx950 (wave64).
//
// Work decomposition: one wavefront owns one page at a time.  A lane owns 8 consecutive channels
// (16 bytes of FP16), so a 64-lane pass covers 512 elements with one fully coalesced 128-bit
// access per lane, a 32-element packet group is a quad of lanes, and a token row of d channels is
// d/8 neighbouring lanes.  Compressed payloads are assembled in (encode) or staged through (decode)
// LDS and move to/from the pool as 128-bit accesses.
//
// Encode follows Algorithm 2 of the paper (scaling, quantize, delta along the channel index,
// run-length encode); decode follows Section 3.5.3 (undo run-length coding, prefix sum,
// dequantize), with the stored-uncompressed bypass.
#include <hip/hip_fp16.h>

#include <algorithm>

#include "kvc_device.h"

namespace kvc {

// Inclusive prefix over the lanes of one token row.  Rows are runs of lpr <= 32 lanes that may begin
// anywhere, also in the pass before this one: r = the lane's position in its row.  Prefix over the whole
// wave, minus its value just before the row's first lane; a lane with r > lane belongs to a row that
// began in the previous pass and adds `carry`, that pass's value at lane 63.
__device__ __forceinline__ uint32_t row_incl_scan_u32(uint32_t v, uint32_t r, uint32_t carry) {
    const int lane = lane_id();
    const uint32_t S = wave_incl_scan_dpp(v);
    const int start = lane - (int)r;  // first lane of this lane's row (< 0: in the pass before)
    const uint32_t before = (uint32_t)__builtin_amdgcn_ds_bpermute((start > 0 ? start - 1 : 0) << 2, (int)S);
    return start > 0 ? S - before : (start < 0 ? S + carry : S);
}

__device__ __forceinline__ float half_bits_to_float(uint32_t h) {
    return __half2float(__ushort_as_half((unsigned short)h));
}

__device__ __forceinline__ uint32_t float_to_half_bits(float f) {
    return (uint32_t)__half_as_ushort(__float2half_rn(f));
}

// Quantize step of Algorithm 2 on a lane's 8 elements: q = round_half_even(x * s_inv).  The fused
// multiply-add against 1.5*2^23 rounds the exact product once, to an integer, ties to even.
__device__ __forceinline__ void quantize8(const uint4& raw, float s_inv, int q[8]) {
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        float lo = half_bits_to_float(w[k] & 0xFFFFu);
        float hi = half_bits_to_float(w[k] >> 16);
        q[2 * k] = (int)__float_as_uint(__builtin_fmaf(lo, s_inv, 12582912.0f)) - 0x4B400000;
        q[2 * k + 1] = (int)__float_as_uint(__builtin_fmaf(hi, s_inv, 12582912.0f)) - 0x4B400000;
    }
}

__device__ __forceinline__ uint32_t pack_bytes4(int a, int b, int c, int d) {
    return (uint32_t)(a & 0xFF) | ((uint32_t)(b & 0xFF) << 8) | ((uint32_t)(c & 0xFF) << 16) | ((uint32_t)d << 24);
}

// 8-bit wrap then zig-zag: 0,-1,1,-2,... -> 0,1,2,3,...
__device__ __forceinline__ uint32_t zigzag8(int delta) {
    uint32_t b = (uint32_t)delta & 0xFFu;
    return ((b << 1) ^ (0u - (b >> 7))) & 0xFFu;
}

// ---------------------------------------------------------------------------------- encode

template <int MAXP>
__device__ __forceinline__ void store_codes(const uint4 (&raw)[MAXP], float s_inv, int E, uint32_t* stage) {
    const int lane = lane_id();
#pragma unroll
    for (int p = 0; p < MAXP; ++p) {
        const int e0 = p * 512 + lane * 8;
        if (e0 < E) {
            int q[8];
            quantize8(raw[p], s_inv, q);
            uint2 v;
            v.x = pack_bytes4(q[0], q[1], q[2], q[3]);
            v.y = pack_bytes4(q[4], q[5], q[6], q[7]);
            *reinterpret_cast<uint2*>(reinterpret_cast<uint8_t*>(stage) + e0) = v;
        }
    }
}

// Encodes one page held at src into the LDS slot `stage` (modes 1..3).  A RAW page is only
// classified here; its bytes go from the source to the pool in the copy-out phase.
template <int MAXP>
__device__ PageResult encode_page(const uint16_t* __restrict__ src, const Geometry& g, int scheme, uint32_t* stage) {
    const int lane = lane_id();
    const int E = g.E;
    const int G = E >> 5;
    const int hdr = (G + 1) >> 1;
    uint8_t* stage8 = reinterpret_cast<uint8_t*>(stage);

    uint4 raw[MAXP];
#pragma unroll
    for (int p = 0; p < MAXP; ++p) {
        const int e0 = p * 512 + lane * 8;
        raw[p] = (e0 < E) ? *reinterpret_cast<const uint4*>(src + elem_off(g, e0)) : make_uint4(0, 0, 0, 0);
    }
    // scaling step: max |x| over the page on the FP16 bit patterns (monotone in magnitude)
    uint32_t m = 0;
#pragma unroll
    for (int p = 0; p < MAXP; ++p) {
        const uint32_t w[4] = {raw[p].x, raw[p].y, raw[p].z, raw[p].w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            uint32_t a = w[k] & 0x7FFF7FFFu;
            m = max(m, max(a & 0xFFFFu, a >> 16));
        }
    }
    m = wave_max_dpp(m);
    PageResult r;
    if (scheme == KVC_MODE_RAW || m >= 0x7C00u) {  // requested, or a NaN/Inf is present: bypass
        r.n16 = (uint32_t)(E >> 3);
        r.mode = KVC_MODE_RAW;
        r.scale = 0.0f;
        return r;
    }
    float s = 0.0f, s_inv = 0.0f;
    if (m != 0) {
        const PageScale ps = page_scale(m);
        s = ps.s;
        s_inv = ps.s_inv;
    }
    r.scale = s;
    if (scheme == KVC_MODE_INT8) {
        store_codes<MAXP>(raw, s_inv, E, stage);
        r.n16 = (uint32_t)(E >> 4);
        r.mode = KVC_MODE_INT8;
        return r;
    }
    // the slot must start as zeros: bodies are OR-ed in, and the padding is part of the payload
    for (int o = lane * 16; o < E; o += 1024) *reinterpret_cast<uint4*>(stage8 + o) = make_uint4(0, 0, 0, 0);
    wave_sync();

    uint32_t run = 0;  // body bytes emitted so far (wave-uniform)
    int q_last = 0;    // last code of the pass before (a token row may continue across passes)
#pragma unroll
    for (int p = 0; p < MAXP; ++p) {
        if (p * 512 < E) {
            const bool act = p * 512 + lane * 8 < E;
            int q[8];
            quantize8(raw[p], s_inv, q);
            // delta along the channel index; the first column of a token row is kept verbatim
            int prev = (int)dpp<0x138>((uint32_t)q_last, (uint32_t)q[7]);  // wave_shr:1; lane 0 keeps the pass before's last code
            if (lane_in_row(g, (uint32_t)(p * 64 + lane)) == 0) prev = 0;
            q_last = __builtin_amdgcn_readlane(q[7], 63);
            uint32_t u[8];
            if (scheme == KVC_MODE_PACK) {  // no delta step: the codes themselves are packed
#pragma unroll
                for (int k = 0; k < 8; ++k) u[k] = zigzag8(q[k]);
            } else {
                u[0] = zigzag8(q[0] - prev);
#pragma unroll
                for (int k = 1; k < 8; ++k) u[k] = zigzag8(q[k] - q[k - 1]);
            }
            uint32_t umax = u[0], umin = u[0];
#pragma unroll
            for (int k = 1; k < 8; ++k) {
                umax = max(umax, u[k]);
                umin = min(umin, u[k]);
            }
            // a group of 32 is a quad of lanes
            umax = max(umax, dpp<0xB1>(0, umax));  // quad_perm [1,0,3,2]
            umin = min(umin, dpp<0xB1>(0xFFu, umin));
            umax = max(umax, dpp<0x4E>(0, umax));  // quad_perm [2,3,0,1]
            umin = min(umin, dpp<0x4E>(0xFFu, umin));
            uint32_t c;
            const bool runs = scheme != KVC_MODE_DELTA;  // zero-run and run packets
            if (runs && umax == 0)
                c = 0;
            else if (runs && umin == umax)
                c = 9;
            else
                c = max(1u, 32u - (uint32_t)__clz((int)umax));
            if (!act) c = 0;
            const uint32_t size = (c == 0) ? 0u : (c == 9 ? 1u : 4u * c);
            const uint32_t incl = quad_incl_scan_dpp(size);  // size is the same in the four lanes of a group
            const uint32_t off = run + incl - size;
            run += (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
            // header: two 4-bit codes per byte, even group in the low nibble.  Lane 4j+i votes bit i of
            // group j's code, so the ballot is the pass's eight header bytes; a lane per byte writes its own
            // (bytes, not dwords: a short page's header ends where its first body begins)
            const uint64_t hb = __builtin_amdgcn_ballot_w64(((c >> (lane & 3)) & 1u) != 0);
            if (act && (lane & 7) == 0)
                stage8[(p * 16 + (lane >> 2)) >> 1] = (uint8_t)(lane < 32 ? (uint32_t)hb >> lane : (uint32_t)(hb >> 32) >> (lane - 32));
            // body: this lane's 8 values are bytes [qi*w, qi*w + w) of the group's bit string
            uint2 W = make_uint2(0u, 0u);
            uint32_t B = hdr + off;
            if (c >= 1 && c <= 8) {
                W = pack8_bits(u, c);
                B += (lane & 3) * c;
            } else if (c == 9) {
                W.x = (lane & 3) == 0 ? u[0] : 0;
            }
            {
                uint32_t* p0 = stage + (B >> 2);  // inside the slot for every lane (the slot has slack beyond the payload)
                uint32_t d0, d1, d2;
                shl_bytes(W, B, d0, d1, d2);
                atomicOr(p0, d0);
                atomicOr(p0 + 1, d1);
                if (d2) atomicOr(p0 + 2, d2);
            }
        }
    }
    const uint32_t n = (hdr + run + 15u) & ~15u;
    wave_sync();
    if (n >= (uint32_t)E) {  // packing did not beat plain INT8
        store_codes<MAXP>(raw, s_inv, E, stage);
        r.n16 = (uint32_t)(E >> 4);
        r.mode = KVC_MODE_INT8;
    } else {
        r.n16 = n >> 4;
        r.mode = (uint32_t)scheme;
    }
    return r;
}

// One workgroup = 4 waves x PPW pages.  Payloads wait in LDS until the workgroup has reserved
// one contiguous pool span for all of them with a single atomic on the pool cursor.
template <int MAXP, int PPW>
__global__ __launch_bounds__(kThreads) void k_compress(EncodeArgs a) {
    constexpr int kSlots = kWavesPerWG * PPW;
    __shared__ __align__(16) uint32_t s_stage[kSlots][Slot<MAXP>::kWords];
    __shared__ EncBook<kSlots> s_book;
    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t t0 = ((int64_t)blockIdx.x * kWavesPerWG + wave) * PPW;
    TaskPos pos = task_pos(t0, a.g.ppb);
    for (int i = 0; i < PPW; ++i) {
        const int slot = wave * PPW + i;
        const EncTask task = resolve_enc_task(a, t0 + i, pos);
        task_advance(pos, a.g.ppb);
        PageResult r;
        r.n16 = 0;
        r.mode = KVC_MODE_INVALID;
        r.scale = 0.0f;
        if (task.desc_idx >= 0) r = encode_page<MAXP>(a.cache + task.src_off, a.g, task.scheme, s_stage[slot]);
        if (lane == 0) {
            s_book.n16[slot] = r.n16;
            s_book.mode[slot] = r.mode;
            s_book.scale[slot] = r.scale;
            s_book.desc[slot] = task.desc_idx;
            s_book.srcoff[slot] = task.src_off;
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) reserve_pool_span<kSlots>(a, s_book);
    __syncthreads();
    for (int i = 0; i < PPW; ++i) emit_page<kSlots>(a, s_book, wave * PPW + i, s_stage[wave * PPW + i]);
}

// ---------------------------------------------------------------------------------- decode

// dequantize step: x = fp16(fp32(q) * s) for a lane's 8 codes (low 8 bits of each q[k], signed)
__device__ __forceinline__ uint4 dequant8(const int q[8], float s) {
    uint32_t h[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) h[k] = float_to_half_bits((float)(int)(int8_t)(q[k] & 0xFF) * s);
    return make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
}

// Decodes the page described by descriptor d_idx into dst.  Returns false (dst zero-filled) if the
// descriptor or the payload fails validation.
template <int MAXP>
__device__ bool decode_page(const DecodeArgs& a, uint64_t d_idx, uint16_t* __restrict__ dst, uint32_t* stage,
                            uint32_t* ginfo) {
    const int lane = lane_id();
    const int E = a.g.E;
    const int G = E >> 5;
    const int hdr = (G + 1) >> 1;
    const uint4 dw = reinterpret_cast<const uint4*>(a.desc)[d_idx];
    const uint64_t off = (uint64_t)dw.x | ((uint64_t)dw.y << 32);
    const float s = __uint_as_float(dw.z);
    const uint32_t n16 = dw.w & 0xFFFFu;
    const uint32_t mode = (dw.w >> 16) & 0xFFu;

    bool ok = (off & 15u) == 0 && (off >> 4) + n16 <= a.pool_units;
    if (mode == KVC_MODE_RAW)
        ok = ok && n16 == (uint32_t)(E >> 3);
    else if (mode == KVC_MODE_INT8)
        ok = ok && n16 == (uint32_t)(E >> 4);
    else if (mode == KVC_MODE_DELTA || mode == KVC_MODE_RLE || mode == KVC_MODE_PACK)
        ok = ok && n16 * 16u >= (uint32_t)hdr && n16 < (uint32_t)(E >> 4);
    else
        ok = false;
    if (!ok) {
        zero_page(dst, a.g);
        return false;
    }
    const uint8_t* pl = a.pool + off;
    if (mode == KVC_MODE_RAW) {  // stored-uncompressed bypass
        for (uint32_t o = lane; o < n16; o += 64)
            *reinterpret_cast<uint4*>(dst + elem_off(a.g, (int)o * 8)) = reinterpret_cast<const uint4*>(pl)[o];
        return true;
    }
    if (mode == KVC_MODE_INT8) {
#pragma unroll
        for (int p = 0; p < MAXP; ++p) {
            const int e0 = p * 512 + lane * 8;
            if (e0 < E) {
                const uint2 v = *reinterpret_cast<const uint2*>(pl + e0);
                int q[8];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    q[k] = (int)(v.x >> (8 * k));
                    q[4 + k] = (int)(v.y >> (8 * k));
                }
                *reinterpret_cast<uint4*>(dst + elem_off(a.g, e0)) = dequant8(q, s);
            }
        }
        return true;
    }
    // modes 2/3: stage the payload in LDS
    const uint8_t* stage8 = reinterpret_cast<const uint8_t*>(stage);
    for (uint32_t o = lane; o < n16; o += 64) reinterpret_cast<uint4*>(stage)[o] = reinterpret_cast<const uint4*>(pl)[o];
    wave_sync();
    // header: code of every group -> body offset by a prefix sum over body sizes
    uint32_t run = 0;
    bool bad = false;
    for (int g0 = 0; g0 < G; g0 += 64) {
        const int gi = g0 + lane;
        uint32_t c = 0;
        if (gi < G) {
            const uint32_t byte = stage8[gi >> 1];
            c = (gi & 1) ? (byte >> 4) : (byte & 15u);
            if (c > 9 || (mode == KVC_MODE_DELTA && (c == 0 || c == 9))) bad = true;
        }
        const uint32_t size = (c == 0) ? 0u : (c == 9 ? 1u : 4u * c);
        const uint32_t incl = wave_incl_scan_dpp(size);
        if (gi < G) ginfo[gi] = ((run + incl - size) << 4) | c;
        run += (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
    }
    if (__any(bad) || (((uint32_t)hdr + run + 15u) >> 4) != n16) {
        zero_page(dst, a.g);
        return false;
    }
    wave_sync();
    uint32_t row_carry = 0;  // prefix of the row that continues from the pass before
#pragma unroll
    for (int p = 0; p < MAXP; ++p) {
        if (p * 512 < E) {
            const int e0 = p * 512 + lane * 8;
            const bool act = e0 < E;
            uint32_t c = 0, goff = 0;
            if (act) {
                const uint32_t gi = ginfo[p * 16 + (lane >> 2)];
                c = gi & 15u;
                goff = gi >> 4;
            }
            uint32_t u[8];
            if (c >= 1 && c <= 8) {
                const uint32_t B = (uint32_t)hdr + goff + (uint32_t)(lane & 3) * c;
                const uint32_t sh = (B & 3u) * 8u;
                const uint32_t* p0 = stage + (B >> 2);
                const uint32_t d0 = p0[0], d1 = p0[1], d2 = p0[2];
                const uint32_t lo = __builtin_amdgcn_alignbit(d1, d0, sh);  // (d1 : d0) >> sh, sh a multiple of 8 below 32
                const uint32_t hi = __builtin_amdgcn_alignbit(d2, d1, sh);
                const uint32_t mid = shr_nibbles(lo, hi, c);  // values 4..7 start at bit 4c
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    u[k] = __builtin_amdgcn_ubfe(lo, (uint32_t)k * c, c);
                    u[4 + k] = __builtin_amdgcn_ubfe(mid, (uint32_t)k * c, c);
                }
            } else {
                const uint32_t v = (c == 9) ? stage8[hdr + goff] : 0u;
#pragma unroll
                for (int k = 0; k < 8; ++k) u[k] = v;
            }
            // undo zig-zag, prefix sum along the channel index (mod 256)
            int q[8];
            int acc = 0;
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                acc += (int)(u[k] >> 1) ^ -(int)(u[k] & 1u);
                q[k] = acc;
            }
            const uint32_t incl = row_incl_scan_u32((uint32_t)acc, lane_in_row(a.g, (uint32_t)(p * 64 + lane)), row_carry);
            row_carry = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
            const int before = (int)(incl - (uint32_t)acc);
            if (mode == KVC_MODE_PACK) {  // values are the codes themselves: undo the in-lane sums
#pragma unroll
                for (int k = 7; k > 0; --k) q[k] -= q[k - 1];
            } else {
#pragma unroll
                for (int k = 0; k < 8; ++k) q[k] += before;
            }
            if (act) *reinterpret_cast<uint4*>(dst + elem_off(a.g, e0)) = dequant8(q, s);
        }
    }
    return true;
}

template <int MAXP, int PPW>
__global__ __launch_bounds__(kThreads) void k_decompress(DecodeArgs a) {
    __shared__ __align__(16) uint32_t s_stage[kWavesPerWG][Slot<MAXP>::kWords];
    __shared__ uint32_t s_ginfo[kWavesPerWG][MAXP * 16];
    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t t0 = ((int64_t)task_block_index<1>() * kWavesPerWG + wave) * PPW;
    TaskPos pos = task_pos(t0, a.g.ppb);
    for (int i = 0; i < PPW; ++i) {
        const DecTask task = resolve_dec_task(a, t0 + i, pos);
        task_advance(pos, a.g.ppb);
        if (task.kind == 2) zero_page(task.dst, a.g);
        if (task.kind == 1 && !decode_page<MAXP>(a, task.desc_idx, task.dst, s_stage[wave], s_ginfo[wave])) {
            if (lane == 0) atomicOr(&a.st->status, KVC_ST_CORRUPT);
        }
        wave_sync();
    }
}

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
// to transfer is ready at once, the others when their last transfer completes.  One workgroup.
__global__ __launch_bounds__(256) void k_window_build(WindowArgs w) {
    __shared__ uint32_t s_cnt[4];
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const long long now = max(wall_clock64(), 1ll);
    uint32_t base = 0;  // queue entries so far (workgroup-uniform)
    for (int l = 0; l < w.n_layers_call; ++l) {
        uint32_t in_layer = 0;
        for (int c0 = 0; c0 < w.per_layer; c0 += 256) {
            const int i = c0 + (int)threadIdx.x;
            const bool live = i < w.per_layer && w.fetch[(int64_t)l * w.per_layer + i] >= 0;
            const uint64_t m = __builtin_amdgcn_ballot_w64(live);
            if (lane == 0) s_cnt[wave] = (uint32_t)__builtin_popcountll(m);
            __syncthreads();
            uint32_t before = 0, all = 0;
            for (int k = 0; k < 4; ++k) {
                before += k < wave ? s_cnt[k] : 0u;
                all += s_cnt[k];
            }
            if (live) w.queue[base + in_layer + before + __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u))] = l * w.per_layer + i;
            in_layer += all;
            __syncthreads();
        }
        if (threadIdx.x == 0) {
            w.pending[l] = (int32_t)in_layer;
            w.notify[w.layer_begin + l] = in_layer ? 0ll : now;
        }
        base += in_layer;
    }
    if (threadIdx.x == 0) {
        const unsigned int engines = min(base, (uint32_t)w.omega);
        w.hdr->n_issued = base;
        w.hdr->engines = engines;
        // entries per turn: long queues space out the bookkeeping, short ones keep every engine busy
        w.hdr->chunk = engines ? min(max(base / (4u * engines), 1u), 8u) : 1u;
        w.hdr->ticket = 0;
        w.hdr->done = 0;
        w.notify[w.n_layers] = now;                       // window opened
        w.notify[w.n_layers + 1] = (long long)base;       // transfers issued
        w.notify[w.n_layers + 2] = (long long)engines;    // engines at work: the bound on blocks in flight
        w.notify[w.n_layers + 3] = base ? 0ll : now;      // all complete
    }
}

// Transfer engines of the window for the generic page geometries: see window_next.
template <int MAXP>
__global__ __launch_bounds__(kThreads) void k_decompress_window(DecodeArgs a, WindowArgs w) {
    __shared__ __align__(16) uint32_t s_stage[kWavesPerWG][Slot<MAXP>::kWords];
    __shared__ uint32_t s_ginfo[kWavesPerWG][MAXP * 16];
    __shared__ uint32_t s_turn[2];
    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    WindowTurn none;
    none.first = none.count = 0;
    WindowTurn turn = window_next(w, s_turn, none);
    while (turn.count) {
        for (uint32_t i = 0; i < turn.count; ++i) {
            const int32_t slot = __builtin_amdgcn_readfirstlane(w.queue[turn.first + i]);
            for (int pg = wave; pg < a.g.ppb; pg += kWavesPerWG) {
                TaskPos pos;
                pos.blk = slot;
                pos.pg = pg;
                const DecTask task = resolve_dec_task(a, (int64_t)slot * a.g.ppb + pg, pos);
                if (task.kind == 2) zero_page(task.dst, a.g);
                if (task.kind == 1 && !decode_page<MAXP>(a, task.desc_idx, task.dst, s_stage[wave], s_ginfo[wave])) {
                    if (lane == 0) atomicOr(&a.st->status, KVC_ST_CORRUPT);
                }
                wave_sync();
            }
        }
        turn = window_next(w, s_turn, turn);
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

// geometries served by the specialised kernels of kvc_fast.h
const FastKernels* fast_kernels(int N, int d) {
    using Lookup = const FastKernels* (*)(int, int);
    static const Lookup groups[kFastGroups] = {fast_kernels_group0, fast_kernels_group1, fast_kernels_group2, fast_kernels_group3,
                                               fast_kernels_group4, fast_kernels_group5, fast_kernels_group6, fast_kernels_group7};
    for (Lookup f : groups)
        if (const FastKernels* k = f(N, d)) return k;
    return nullptr;
}

static inline unsigned grid_for(int64_t n_pages, int ppw) {
    const int64_t per_wg = (int64_t)kWavesPerWG * ppw;
    return (unsigned)((n_pages + per_wg - 1) / per_wg);
}

hipError_t launch_compress(const EncodeArgs& a, hipStream_t s) {
    if (a.n_pages == 0) return hipSuccess;
    if (const FastKernels* f = fast_kernels(a.g.N, a.g.d)) return f->compress(a, s);
    constexpr int PPW = 4;
    const dim3 grid(grid_for(a.n_pages, PPW)), block(kThreads);
    if (a.g.E <= 512) return launch_kernel(k_compress<1, PPW>, grid, block, s, a);
    if (a.g.E <= 2048) return launch_kernel(k_compress<4, PPW>, grid, block, s, a);
    return launch_kernel(k_compress<8, 2>, dim3(grid_for(a.n_pages, 2)), block, s, a);
}

hipError_t launch_decompress(const DecodeArgs& a, hipStream_t s) {
    if (a.n_pages == 0) return hipSuccess;
    if (const FastKernels* f = fast_kernels(a.g.N, a.g.d)) return f->decompress(a, s);
    constexpr int PPW = 4;
    const dim3 grid(grid_for(a.n_pages, PPW)), block(kThreads);
    if (a.g.E <= 512) return launch_kernel(k_decompress<1, PPW>, grid, block, s, a);
    if (a.g.E <= 2048) return launch_kernel(k_decompress<4, PPW>, grid, block, s, a);
    return launch_kernel(k_decompress<8, PPW>, grid, block, s, a);
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
    return launch_kernel(k_window_build, dim3(1), dim3(256), s, w);
}

// At most omega workgroups, one block in flight each; the queue may turn out shorter than the grid, in
// which case the surplus workgroups leave at their first look.
hipError_t launch_decompress_window(const DecodeArgs& a, const WindowArgs& w, int32_t omega, hipStream_t s) {
    if (w.n_now <= 0) return hipSuccess;
    const unsigned grid = (unsigned)std::min<int64_t>(omega, w.n_now);
    if (const FastKernels* f = fast_kernels(a.g.N, a.g.d)) return f->decompress_window(a, w, grid, s);
    const dim3 block(kThreads);
    if (a.g.E <= 512) return launch_kernel(k_decompress_window<1>, dim3(grid), block, s, a, w);
    if (a.g.E <= 2048) return launch_kernel(k_decompress_window<4>, dim3(grid), block, s, a, w);
    return launch_kernel(k_decompress_window<8>, dim3(grid), block, s, a, w);
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
