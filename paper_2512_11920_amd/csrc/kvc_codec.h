// The codec kernels, specialised at compile time for the page shape: D channels (any multiple of 32 up to
// 256) and NP = 1..8 passes of 512 elements.  Two kinds of shape: pages that are a whole number of passes
// (N = NP * 512 / D tokens; 16 x 128 FP16, D = 128 and NP = 4, is the paper's 4 KB page and the shape the
// tuning was done on), where every quantity is a constant and no lane is ever inactive, and -- PARTIAL --
// pages of any other token count that needs NP passes, where the element count is read at run time and the
// last pass is short.  This file holds the templates; kvc_codec.hip instantiates them.
//
// Lane mapping: one wave per page, passes of 512 elements, a lane owns 8 consecutive channels (one 128-bit
// access), a packet group is a quad of lanes, a token row is D/8 neighbouring lanes (one 16-lane DPP row at
// D = 128).  Every cross-lane step is a DPP operation, the per-group statistics (max, width, run test) and
// the offset scans are done on quads.  When D does not divide 512 (96, 160, 192, 224) a token row may begin
// in one pass and end in the next: the delta step and its inverse then carry one value from pass to pass.
// Written plainly the codec is bound by vector-ALU issue long before HBM bandwidth; the instruction count
// per element is kept low enough here that the memory system is the limit.
//
// Encode: Algorithm 2 of the paper (scaling, quantize, delta, run-length encode).
// Decode: Section 3.5.3 (undo run-length coding, prefix sum, dequantize; bypass for raw pages).
#pragma once
#include "kvc_device.h"

namespace kvc {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef unsigned short ushort2v __attribute__((ext_vector_type(2)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));

// Non-temporal hints for the page-sized streams (encoder input, decoder output): measured 4-7 % faster.
#ifndef KVC_NT_LOAD
#define KVC_NT_LOAD 1
#endif
#ifndef KVC_NT_STORE
#define KVC_NT_STORE 1
#endif
#ifndef KVC_NT_POOL
#define KVC_NT_POOL 0
#endif

// 128-bit global accesses of streamed data (each byte is touched once)
__device__ __forceinline__ uint4 load_stream(const uint4* p) {
#if KVC_NT_LOAD
    const uint4v v = __builtin_nontemporal_load(reinterpret_cast<const uint4v*>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
#else
    return *p;
#endif
}
__device__ __forceinline__ void store_stream(uint4* p, const uint4& v) {
#if KVC_NT_STORE
    uint4v w;
    w.x = v.x; w.y = v.y; w.z = v.z; w.w = v.w;
    __builtin_nontemporal_store(w, reinterpret_cast<uint4v*>(p));
#else
    *p = v;
#endif
}

// Compile-time shape of a page of NP passes with D channels per token.  PARTIAL: the page has fewer
// than NP * 512 elements (more than (NP - 1) * 512); kE, kN, kGroups and kHdr are then upper bounds and
// the run-time values come from page_extent().
template <int D, int NP, bool PARTIAL = false>
struct Page {
    static_assert(D % 32 == 0 && D >= 32 && D <= 256 && NP >= 1 && NP <= 8 && (PARTIAL || (NP * 512) % D == 0), "page shape");
    static constexpr int kD = D;
    static constexpr bool kPartial = PARTIAL;
    static constexpr int kE = NP * 512;       // elements
    static constexpr int kN = kE / D;         // tokens
    static constexpr int kPasses = NP;        // passes of 512 elements
    static constexpr int kGroups = NP * 16;   // packet groups of 32
    static constexpr int kHdr = NP * 8;       // header bytes, 4 bits per group
    static constexpr int kLpr = D / 8;        // lanes per token row
    static constexpr bool kAligned = 512 % D == 0;  // a token row never continues into the next pass
    static constexpr int kRowsPerPass = 512 / D;    // (whole rows; exact when kAligned)
    static constexpr int kRounds = (NP + 1) / 2;    // rounds of 64 lanes x 16 bytes that cover a payload (< kE bytes)
    static constexpr bool kChan = !PARTIAL && kN == 16 && (D == 64 || D == 128 || D == 256);  // mode 5 is built for these pages
};

// Extent of a page: elements, header bytes (4 bits per group of 32, rounded up to a byte) and the number
// of lanes that hold data in the last pass.  Constants unless P::kPartial.  A token row is a multiple of
// four lanes, so a packet group (a quad) and a row are either all data or all beyond the page.
struct Extent {
    uint32_t E, hdr, last;
};
template <class P>
__device__ __forceinline__ Extent page_extent(const Geometry& g) {
    Extent x;
    if (P::kPartial) {
        x.E = (uint32_t)g.E;
        x.hdr = (((uint32_t)g.E >> 5) + 1u) >> 1;
        x.last = ((uint32_t)g.E >> 3) - (uint32_t)(P::kPasses - 1) * 64u;
    } else {
        x.E = P::kE;
        x.hdr = P::kHdr;
        x.last = 64u;
    }
    return x;
}
// does this lane hold data in pass p (p a constant after unrolling: true at compile time except in the
// last pass of a partial page)
template <class P>
__device__ __forceinline__ bool lane_live(const Extent& x, int p) {
    return !P::kPartial || p < P::kPasses - 1 || (uint32_t)lane_id() < x.last;
}

// Where a lane sits in pass 0: token row and position inside the row, both in lanes of 8 channels, and
// the byte offset of its 16 bytes inside the page (row-major deal, and the deal of mode 5).
struct LanePos {
    uint32_t row0, col0, off0, off0_chan;
};
template <class P>
__device__ __forceinline__ LanePos lane_pos(const Geometry& g) {
    const uint32_t lane = (uint32_t)lane_id();
    LanePos lp;
    lp.row0 = lane / P::kLpr;
    lp.col0 = lane % P::kLpr;
    lp.off0 = (lp.row0 * (uint32_t)g.row_stride + lp.col0 * 8u) * 2u;
    lp.off0_chan = P::kD == 64 ? (((lane >> 5) * 8u + (lane & 3u)) * (uint32_t)g.row_stride + ((lane >> 2) & 7u) * 8u) * 2u
                               : ((lane & 3u) * (uint32_t)g.row_stride + (lane >> 2) * 8u) * 2u;
    return lp;
}
// ... and in pass p (p is a constant after unrolling): 64 * p lanes further on.
template <class P>
__device__ __forceinline__ uint32_t pass_col(const LanePos& lp, int p) {
    const uint32_t c = lp.col0 + (uint32_t)((p * 64) % P::kLpr);
    return (!P::kAligned && c >= (uint32_t)P::kLpr) ? c - P::kLpr : c;
}
template <class P>
__device__ __forceinline__ uint32_t pass_row(const LanePos& lp, int p) {
    const uint32_t wrap = (!P::kAligned && lp.col0 + (uint32_t)((p * 64) % P::kLpr) >= (uint32_t)P::kLpr) ? 1u : 0u;
    return lp.row0 + (uint32_t)((p * 64) / P::kLpr) + wrap;
}

// Values of the encoder's SCHEME parameter below zero: the mode is read per page at run time, from modes
// 0..4, or from 0..5 (only built for the page shapes that have mode 5).
constexpr int kSchemeRowMajor = -1;
constexpr int kSchemeAny = -2;

constexpr float kMagic = 12582912.0f;  // 1.5 * 2^23: adding it rounds to an integer, ties to even
constexpr uint32_t kMagicBits = 0x4B400000u;

__device__ __forceinline__ uint32_t pk_max_u16(uint32_t a, uint32_t b) {
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(ushort2v, a),
                                                                 __builtin_bit_cast(ushort2v, b)));
}

// Quantize step on 8 FP16 values: bits of (x * s_inv + M_k), M_k = 1.5*2^23 + 256*k.  The fused
// multiply-add rounds the exact product once, to an integer, ties to even; the low byte of the result
// is q (two's complement).  The per-element bias 256*k makes every difference of neighbouring results
// positive: bits(t_k) - bits(t_{k-1}) = q_k - q_{k-1} + 256.
__device__ __forceinline__ void quantize8_bits(const uint4& raw, float s_inv, uint32_t t[8]) {
    const half8 h = __builtin_bit_cast(half8, raw);
#pragma unroll
    for (int k = 0; k < 8; ++k) t[k] = __float_as_uint(__builtin_fmaf((float)h[k], s_inv, kMagic + 256.0f * (float)k));
}

// Two ways of dealing a page's 128-bit pieces (one token, eight channels = one octet) to the lanes.
// Row-major (CHAN = false): piece number p*64 + lane in pass p.  Channel-pair mode 5 (CHAN = true):
// at D = 128 or 256 lane 4*l + r takes, in pass p, token 4*(p mod 4) + r of octet 16*(p div 4) + l, so
// that the four lanes of a quad hold the 16 tokens of one octet over four passes; at D = 64 (eight octets,
// two passes) lane 32*h + 4*l + r takes token 8*h + 4*p + r of octet l, so that a quad and its partner 32
// lanes away hold the 16 tokens of one octet between them.
template <class P, bool CHAN>
__device__ __forceinline__ int piece_index(int p, int lane) {  // position in row-major piece order
    if (!CHAN) return p * 64 + lane;
    if (P::kD == 64) return (8 * (lane >> 5) + 4 * p + (lane & 3)) * P::kLpr + ((lane >> 2) & 7);
    return (4 * (p & 3) + (lane & 3)) * P::kLpr + 16 * (p >> 2) + (lane >> 2);
}

// plain INT8 payload: codes as bytes, row-major
template <class P, bool CHAN>
__device__ __forceinline__ void store_codes(const uint4 (&raw)[P::kPasses], float s_inv, const Extent& x, uint32_t* stage) {
    constexpr int NP = P::kPasses;
    const int lane = lane_id();
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        if (!lane_live<P>(x, p)) continue;
        uint32_t t[8];
        quantize8_bits(raw[p], s_inv, t);
        uint2 v;
        v.x = __builtin_amdgcn_perm(__builtin_amdgcn_perm(t[3], t[2], 0x0c0c0400u), __builtin_amdgcn_perm(t[1], t[0], 0x0c0c0400u), 0x05040100u);
        v.y = __builtin_amdgcn_perm(__builtin_amdgcn_perm(t[7], t[6], 0x0c0c0400u), __builtin_amdgcn_perm(t[5], t[4], 0x0c0c0400u), 0x05040100u);
        reinterpret_cast<uint2*>(stage)[piece_index<P, CHAN>(p, lane)] = v;
    }
}

// Table of the 8-bit wrap + zig-zag map, indexed by delta + 256 (delta in [-254, 254]).
__device__ __forceinline__ void fill_zigzag_lut(uint8_t* lut) {
    for (int i = threadIdx.x; i < 512; i += blockDim.x) {
        const uint32_t b = (uint32_t)(i - 256) & 0xFFu;
        lut[i] = (uint8_t)(((b << 1) ^ (0u - (b >> 7))) & 0xFFu);
    }
}

// t7 of the lane to the left within the token row; row starts receive `first`.  `carry` is the value
// of lane 63 in the pass before, for a row that continues across the pass boundary (!P::kAligned only).
template <class P>
__device__ __forceinline__ uint32_t left_neighbour(const LanePos& lp, int p, uint32_t first, uint32_t v, uint32_t carry) {
    constexpr int LPR = P::kLpr;
    if (P::kAligned) {
        if (LPR == 16) return dpp<0x111>(first, v);  // row_shr:1, lane 0 of a DPP row keeps `first`
        if (LPR < 16) {
            const uint32_t x = dpp<0x111>(first, v);
            return (lane_id() & (LPR - 1)) == 0 ? first : x;
        }
        const uint32_t x = dpp<0x138>(first, v);  // wave_shr:1 crosses the 16-lane rows
        return (lane_id() & 31) == 0 ? first : x;
    }
    const uint32_t x = dpp<0x138>(carry, v);  // lane 0 has no source lane and keeps `carry`
    return pass_col<P>(lp, p) == 0 ? first : x;
}

// Inclusive prefix sum over the lanes of a token row in pass p.  `carry` is the value this function
// returned at lane 63 in the pass before, for a row that began there (!P::kAligned only).
template <class P>
__device__ __forceinline__ uint32_t row_incl_scan(const LanePos& lp, int p, uint32_t v, uint32_t carry) {
    constexpr int LPR = P::kLpr;
    if (P::kAligned) {
        if (LPR == 16) return row16_incl_scan_dpp(v);
        if (LPR == 32) {
            v = row16_incl_scan_dpp(v);
            return v + dpp<0x142, 0xA>(0, v);  // odd DPP rows add the total of the row before
        }
        const int r = lane_id() & (LPR - 1);
        uint32_t t = dpp<0x111>(0, v);
        v += r >= 1 ? t : 0u;
        t = dpp<0x112>(0, v);
        v += r >= 2 ? t : 0u;
        if (LPR == 4) return v;
        t = dpp<0x114>(0, v);
        return v + (r >= 4 ? t : 0u);
    }
    // rows of LPR lanes begin anywhere: prefix over the whole wave, minus its value just before the
    // row's first lane; a row that began in the pass before adds what it had collected there
    const uint32_t S = wave_incl_scan_dpp(v);
    const int lane = lane_id();
    const int start = lane - (int)pass_col<P>(lp, p);  // first lane of this lane's row (< 0: in the pass before)
    const uint32_t before = (uint32_t)__builtin_amdgcn_ds_bpermute((start > 0 ? start - 1 : 0) << 2, (int)S);
    return start > 0 ? S - before : (start < 0 ? S + carry : S);
}

// Second half of a pass: body offsets, header bits, packing, LDS write.  RUNS = some group of this
// pass may be a run packet (is_run is then meaningful), else every group is literal or all-zero.
template <class P, bool RUNS>
__device__ __forceinline__ void encode_tail(const uint32_t (&u)[8], uint32_t c, uint32_t size, bool is_run, uint32_t qi,
                                            int p, bool live, uint32_t& run, uint32_t* stage, DevState* st) {
    (void)st;  // only the bounds-checking build reads it
    const uint32_t incl = quad_incl_scan_dpp(size);
    const uint32_t off = run + incl - size;  // byte offset of this group's body
    run += (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
    // header: group j of this pass has its code in the quad's lanes; lane 4j+i contributes bit i,
    // so the ballot is the 8 header bytes of the pass (even group in the low nibble)
    const uint64_t hb = __builtin_amdgcn_ballot_w64(((c >> qi) & 1u) != 0);
    if (P::kPartial && p == P::kPasses - 1) {
        // a short page's header ends where its first body begins: bytes, each written by the first lane
        // of the two groups it describes
        const uint32_t lane = (uint32_t)lane_id();
        if (live && (lane & 7u) == 0)
            reinterpret_cast<uint8_t*>(stage)[8 * p + (lane >> 3)] = (uint8_t)(lane < 32 ? (uint32_t)hb >> lane : (uint32_t)(hb >> 32) >> (lane - 32));
    } else if (lane_id() == 0) {
        stage[2 * p] = (uint32_t)hb;
        stage[2 * p + 1] = (uint32_t)(hb >> 32);
    }
    // body: this lane's 8 values are bytes [qi*c, qi*c + c) of the group's little-endian bit string
    uint2 W = pack8_bits(u, c);
    uint32_t B = off + __umul24(qi, c);
    if (RUNS && is_run) {
        W = make_uint2(qi == 0 ? u[0] : 0u, 0u);
        B = off;
    }
    uint32_t* p0 = stage + (B >> 2);
    KVC_CHECK(st, c <= 9 && (B >> 2) + 2 < (uint32_t)Slot<P::kPasses>::kWords && B >= (uint32_t)(P::kPartial ? 8 * (P::kPasses - 1) + 1 : P::kHdr));
    uint32_t d0, d1, d2;
    shl_bytes(W, B, d0, d1, d2);
    atomicOr(p0, d0);
    atomicOr(p0 + 1, d1);
    if (d2) atomicOr(p0 + 2, d2);
}

// One packet group per quad of lanes: each lane brings 8 of its 32 values.  Group statistics over
// the quad (max -> width, run test), then the tail.  p = index of the group's set of 16 (a pass).
template <class P>
__device__ __forceinline__ void encode_groups(const uint32_t (&u)[8], bool RLE, uint32_t c_min, uint32_t qi, int p, bool live,
                                              uint32_t& run, uint32_t* stage, DevState* st) {
    // per-group statistics over the quad of lanes
    uint32_t gmax = max(max(u[0], u[1]), u[2]);
    gmax = max(max(gmax, u[3]), u[4]);
    gmax = max(max(gmax, u[5]), u[6]);
    gmax = max(gmax, u[7]);
    gmax = max(gmax, dpp<0xB1>(0, gmax));
    gmax = max(gmax, dpp<0x4E>(0, gmax));
    // bit length of the group maximum (0 for 0): exponent of its float value
    uint32_t c = max((uint32_t)__builtin_amdgcn_frexp_expf((float)gmax), c_min);
    if (P::kPartial && !live) c = 0;  // a group beyond the page: no header bits, no body (its values are zeros)
    const uint32_t size = c << 2;
    bool cand_any = false;
    uint32_t x = 0;
    if (RLE) {
        // run packet: all 32 values equal and non-zero.  Cheap necessary test first.
        x = (u[0] ^ gmax) | (u[7] ^ gmax);
        cand_any = __builtin_amdgcn_ballot_w64(x == 0 && gmax != 0) != 0;
    }
    if (RLE && cand_any) {
        uint32_t y = x;
#pragma unroll
        for (int k = 1; k < 7; ++k) y |= u[k] ^ gmax;
        y |= dpp<0xB1>(0, y);
        y |= dpp<0x4E>(0, y);
        const bool is_run = (y == 0) && (gmax != 0);
        encode_tail<P, true>(u, is_run ? 9u : c, is_run ? 1u : size, is_run, qi, p, live, run, stage, st);
    } else {
        encode_tail<P, false>(u, c, size, false, qi, p, live, run, stage, st);
    }
}

// Byte offset, inside a page, of the 16 bytes a lane handles in pass p, as a wave-uniform part plus a
// per-lane part that stays in 32 bits (the layout setter bounds the row stride): a page access is then a
// wave-uniform 64-bit base plus a 32-bit lane offset.  Row-major deal: lane l of pass p holds token row
// (64p + l) / (D/8), channels 8 * ((64p + l) mod (D/8)) .. +7; with contiguous rows a pass is one 1 KB
// run.  When D divides 512 the lane part is the same in every pass.  Mode 5 (CHAN, see piece_index):
// lane 4l + r takes token 4 (p mod 4) + r of octet 16 (p div 4) + l.
template <class P, bool CHAN>
__device__ __forceinline__ int64_t pass_base_off(const Geometry& g, int p) {
    if (CHAN) return (int64_t)(p & 3) * 4 * g.row_stride * 2 + (P::kD == 64 ? 0 : (p >> 2) * 256);
    return (int64_t)((p * 64) / P::kLpr) * g.row_stride * 2;  // the whole rows before the pass
}
template <class P, bool CHAN>
__device__ __forceinline__ uint32_t pass_lane_off(const Geometry& g, const LanePos& lp, int p) {
    if (CHAN) return lp.off0_chan;
    if (P::kAligned) return lp.off0;
    const uint32_t c = lp.col0 + (uint32_t)((p * 64) % P::kLpr);  // the pass begins this far into a row
    const bool wrap = c >= (uint32_t)P::kLpr;
    return ((lp.row0 + (wrap ? 1u : 0u)) * (uint32_t)g.row_stride + (wrap ? c - P::kLpr : c) * 8u) * 2u;
}

template <class P, bool CHAN>
__device__ __forceinline__ void load_page(const EncodeArgs& a, const EncTask& task, const LanePos& lp,
                                          uint4 (&raw)[P::kPasses]) {
    const char* src = reinterpret_cast<const char*>(a.cache) + wave_uniform((int64_t)task.src_off * 2);
    const Extent x = page_extent<P>(a.g);
#pragma unroll
    for (int p = 0; p < P::kPasses; ++p) {
        raw[p] = make_uint4(0u, 0u, 0u, 0u);  // lanes beyond a short page hold zeros
        if (lane_live<P>(x, p))
            raw[p] = load_stream(reinterpret_cast<const uint4*>(src + pass_base_off<P, CHAN>(a.g, p) + pass_lane_off<P, CHAN>(a.g, lp, p)));
    }
}

// Mode 5: the packets of a page whose 128-bit pieces were dealt to the lanes as piece_index<P, true> says;
// every group holds one pair of neighbouring channels over the 16 tokens.
template <class P>
__device__ __forceinline__ void pack_channel_pairs(const uint4 (&raw)[P::kPasses], float s_inv, uint32_t& run, uint32_t* stage,
                                                   const uint8_t* lut, DevState* st) {
    static_assert(P::kChan, "mode 5 is built for 16-token pages of 64, 128 or 256 channels");
    constexpr int NP = P::kPasses;
    const int lane = lane_id();
    const uint32_t qi = (uint32_t)lane & 3u;
    if constexpr (P::kD == 64) {
        // Eight octets: a lane holds tokens 8h + r and 8h + 4 + r of its octet (two passes), its partner 32
        // lanes away the other eight tokens' share.  Of the octet's four channel pairs the lane packs pairs h
        // and 2 + h (group sets 0 and 1), the partner the other two; each hands the other the four values it
        // holds of the other's pair.  Value index inside a packet: 2 * (token div 4) + (channel mod 2), token
        // div 4 = 2h + p.
        static_assert(NP == 2, "sixteen tokens of eight octets are two passes");
        const bool hi = lane >= 32;
        uint32_t uu[2][8];
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            uint32_t t[8];
            quantize8_bits(raw[p], s_inv, t);
#pragma unroll
            for (int k = 0; k < 8; ++k) uu[p][k] = lut[t[k] - (kMagicBits + 256u * (uint32_t)k - 256u)];
        }
#pragma unroll
        for (int sset = 0; sset < 2; ++sset) {
            uint32_t u[8];
#pragma unroll
            for (int p = 0; p < 2; ++p)
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    const uint32_t lo_pair = uu[p][4 * sset + e], hi_pair = uu[p][4 * sset + 2 + e];  // pairs 2 sset, 2 sset + 1
                    const uint32_t mine = hi ? hi_pair : lo_pair;
                    const uint32_t got = (uint32_t)__builtin_amdgcn_ds_bpermute((lane ^ 32) << 2, (int)(hi ? lo_pair : hi_pair));
                    u[2 * p + e] = hi ? got : mine;
                    u[4 + 2 * p + e] = hi ? mine : got;
                }
            encode_groups<P>(u, true, 0u, qi, sset, true, run, stage, st);
        }
    } else {
        // Sixteen or 32 octets: the four passes of a run of 16 octets are quantized and mapped first; group
        // set j of the run then takes channels 2j, 2j + 1 of each of them: the quad's 32 values are one
        // channel pair over the 16 tokens.
#pragma unroll
        for (int h = 0; h < NP / 4; ++h) {
            uint32_t uu[4][8];
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                uint32_t t[8];
                quantize8_bits(raw[4 * h + p], s_inv, t);
#pragma unroll
                for (int k = 0; k < 8; ++k) uu[p][k] = lut[t[k] - (kMagicBits + 256u * (uint32_t)k - 256u)];
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                uint32_t u[8];
#pragma unroll
                for (int m = 0; m < 8; ++m) u[m] = uu[m >> 1][2 * j + (m & 1)];
                encode_groups<P>(u, true, 0u, qi, 4 * h + j, true, run, stage, st);
            }
        }
    }
}

// Encode one page (already in registers) into the LDS slot `stage`.  The requested mode is the
// compile-time SCHEME when that is >= 0 (one mode for the whole launch: its branches fold away), else
// the wave-uniform run-time value: any of modes 0..4 (SCHEME -1), or any of 0..5 (SCHEME -2, built for
// the page shapes that have mode 5; the page must then have been loaded in the deal of its mode).
template <class P, int SCHEME>
__device__ __forceinline__ PageResult encode_page(const uint4 (&raw)[P::kPasses], const LanePos& lp, const Extent& x, int scheme_rt,
                                                 uint32_t* stage, const uint8_t* lut, DevState* st) {
    const int scheme = SCHEME >= 0 ? SCHEME : scheme_rt;
    constexpr int kE = P::kE, NP = P::kPasses;
    constexpr bool kMayChan = SCHEME == KVC_MODE_CHAN || SCHEME == kSchemeAny;
    const bool chan = SCHEME == KVC_MODE_CHAN || (SCHEME == kSchemeAny && scheme == KVC_MODE_CHAN);
    const bool RLE = scheme != KVC_MODE_DELTA;  // zero-run and run packets (modes 3 and 4)
    const bool no_delta = scheme == KVC_MODE_PACK;
    const uint32_t c_min = RLE ? 0u : 1u;  // without run packets an all-zero group is a 1-bit literal
    const int lane = lane_id();
    const uint32_t qi = (uint32_t)lane & 3u;

    // scaling: max |x| on the FP16 bit patterns, two per dword
    uint32_t m2 = 0;
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        m2 = pk_max_u16(m2, raw[p].x & 0x7FFF7FFFu);
        m2 = pk_max_u16(m2, raw[p].y & 0x7FFF7FFFu);
        m2 = pk_max_u16(m2, raw[p].z & 0x7FFF7FFFu);
        m2 = pk_max_u16(m2, raw[p].w & 0x7FFF7FFFu);
    }
    const uint32_t m = wave_max_dpp(max(m2 & 0xFFFFu, m2 >> 16));
    PageResult r;
    if (scheme == KVC_MODE_RAW || m >= 0x7C00u) {  // requested, or NaN/Inf present: bypass
        r.n16 = x.E >> 3;
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
    auto codes_to_stage = [&]() {  // the plain INT8 payload, from whichever deal the lanes hold
        if constexpr (kMayChan) {
            if (chan) {
                store_codes<P, true>(raw, s_inv, x, stage);
                return;
            }
        }
        store_codes<P, false>(raw, s_inv, x, stage);
    };
    if (scheme == KVC_MODE_INT8) {
        codes_to_stage();
        r.n16 = x.E >> 4;
        r.mode = KVC_MODE_INT8;
        return r;
    }
    // bodies are OR-ed into the slot, and the zero padding is part of the payload
#pragma unroll
    for (int z = 0; z < P::kRounds; ++z)
        if (kE % 1024 == 0 || lane + 64 * z < kE / 16) reinterpret_cast<uint4*>(stage)[lane + 64 * z] = make_uint4(0, 0, 0, 0);
    wave_sync();

    uint32_t run = x.hdr;  // payload bytes so far (wave-uniform)
    bool packed_by_pairs = false;
    if constexpr (kMayChan) {
        if (chan) {
            pack_channel_pairs<P>(raw, s_inv, run, stage, lut, st);
            packed_by_pairs = true;
        }
    }
    if (!packed_by_pairs) {
        uint32_t carry = kMagicBits - 256u;  // last value of the pass before, for a row that continues
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            uint32_t t[8];
            quantize8_bits(raw[p], s_inv, t);
            // delta along the channel index, plus 256; the first column of a token row has no left
            // neighbour and is kept verbatim (q - 0).  Then wrap + zig-zag by table.
            uint32_t u[8];
            if (no_delta) {  // mode 4: the table is indexed by q + 256
#pragma unroll
                for (int k = 0; k < 8; ++k) u[k] = lut[t[k] - (kMagicBits + 256u * (uint32_t)k - 256u)];
            } else {
                const uint32_t prev = left_neighbour<P>(lp, p, kMagicBits - 256u, t[7] - 2048u, carry);
                if (!P::kAligned) carry = (uint32_t)__builtin_amdgcn_readlane((int)(t[7] - 2048u), 63);
                KVC_CHECK(st, t[0] - prev < 512u && t[1] - t[0] < 512u && t[7] - t[6] < 512u);
                u[0] = lut[t[0] - prev];
#pragma unroll
                for (int k = 1; k < 8; ++k) u[k] = lut[t[k] - t[k - 1]];
            }
            const bool live = lane_live<P>(x, p);
            if (P::kPartial && p == NP - 1) {  // lanes beyond the page hold no values
#pragma unroll
                for (int k = 0; k < 8; ++k) u[k] = live ? u[k] : 0u;
            }
            encode_groups<P>(u, RLE, c_min, qi, p, live, run, stage, st);
        }
    }
    const uint32_t n = (run + 15u) & ~15u;
    wave_sync();
    if (n >= x.E) {  // packing did not beat plain INT8
        codes_to_stage();
        r.n16 = x.E >> 4;
        r.mode = KVC_MODE_INT8;
    } else {
        r.n16 = n >> 4;
        r.mode = (uint32_t)scheme;
    }
    return r;
}

// Encode the page held in `raw` (if the task is live) into LDS slot `slot` and note its result.
template <class P, int SCHEME, int SLOTS>
__device__ __forceinline__ void encode_into_slot(const EncodeArgs& a, const uint4 (&raw)[P::kPasses], const LanePos& lp, const EncTask& task,
                                                 int slot, uint32_t* stage, const uint8_t* lut, EncBook<SLOTS>& book) {
    PageResult r;
    r.n16 = 0;
    r.mode = KVC_MODE_INVALID;
    r.scale = 0.0f;
    if (task.desc_idx >= 0) r = encode_page<P, SCHEME>(raw, lp, page_extent<P>(a.g), task.scheme, stage, lut, a.st);
    if (lane_id() == 0) {
        book.n16[slot] = r.n16;
        book.mode[slot] = r.mode;
        book.scale[slot] = r.scale;
        book.desc[slot] = task.desc_idx;
        book.srcoff[slot] = task.src_off;
    }
}

#ifndef KVC_PPW5
#define KVC_PPW5 3
#endif
#ifndef KVC_PPW6
#define KVC_PPW6 3
#endif
#ifndef KVC_PPW7
#define KVC_PPW7 2
#endif
#ifndef KVC_PPW8
#define KVC_PPW8 2
#endif
#ifndef KVC_RING5
#define KVC_RING5 3
#endif
#ifndef KVC_RING6
#define KVC_RING6 3
#endif
#ifndef KVC_RING7
#define KVC_RING7 2
#endif
#ifndef KVC_ENC_WAVES_LONG
#define KVC_ENC_WAVES_LONG 4
#endif
#ifndef KVC_ENC_MIN_WAVES
#define KVC_ENC_MIN_WAVES 4
#endif
#ifndef KVC_ENC_WAVES_1KB
#define KVC_ENC_WAVES_1KB 8
#endif

// Pages a wave holds in registers at once: while one is encoded the loads of the others are in flight.
// Measured best with the ring as long as the wave's whole share (all loads issued up front, about 16 KB
// per wave, no loop) for pages of up to four passes; a page is 4 registers per pass, so longer pages
// take turns in fewer sets, and at eight passes a second page in registers costs occupancy and gains
// nothing.
// The run-time-scheme instantiation needs more registers for itself: from six passes on it keeps one page.
constexpr int enc_ring_max(int np, int scheme) {
    return np <= 2 ? 8 : np <= 3 ? 5 : np <= 4 ? 4 : np <= 5 ? KVC_RING5 : (np == 6 && scheme >= 0) ? KVC_RING6 : (np == 7 && scheme >= 0) ? KVC_RING7 : 1;
}

// (four waves per SIMD is what the LDS slots allow anyway: keep every instantiation within 128 VGPRs; the
// channel-pair encoder at D = 256 holds 32 mapped values beside the page and runs better with three, and
// so do the run-time-scheme encoders of seven- and eight-pass pages whose rows cross passes or whose last
// pass may be short, which would spill at four)
template <class P, int SCHEME>
constexpr int enc_min_waves() {
    return ((P::kD == 256 && (SCHEME == KVC_MODE_CHAN || SCHEME == kSchemeAny)) || (P::kPasses >= 7 && (!P::kAligned || P::kPartial) && SCHEME < 0)) ? 3 : KVC_ENC_MIN_WAVES;
}
template <class P, int WAVES, int PPW, int SCHEME>
__global__ __launch_bounds__(WAVES * 64) __attribute__((amdgpu_waves_per_eu(enc_min_waves<P, SCHEME>()))) void k_compress(EncodeArgs a) {
    constexpr int kSlots = WAVES * PPW;
    constexpr int NP = P::kPasses;
    constexpr int kMaxMode = SCHEME == kSchemeAny ? KVC_MODE_CHAN : KVC_MODE_PACK;  // what a per-block request may ask for
    constexpr int kRing = enc_ring_max(NP, SCHEME) < PPW ? enc_ring_max(NP, SCHEME) : PPW;
    static_assert(PPW % kRing == 0, "the loop handles pages in groups of kRing");
    __shared__ __align__(16) uint32_t s_stage[kSlots][Slot<NP>::kWords];
    __shared__ EncBook<kSlots> s_book;
    __shared__ uint8_t s_lut[512];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    fill_zigzag_lut(s_lut);
    __syncthreads();
    const int64_t t0 = ((int64_t)task_block_index<0>() * WAVES + wave) * PPW;
    TaskPos pos = task_pos(t0, a.g.ppb);
    const LanePos lp = lane_pos<P>(a.g);
    const int slot0 = wave * PPW;
    // the deal of the page to the lanes follows the mode requested for it
    auto load = [&](const EncTask& task, uint4 (&raw)[NP]) {
        if constexpr (SCHEME == kSchemeAny) {
            if (task.scheme == KVC_MODE_CHAN)
                load_page<P, true>(a, task, lp, raw);
            else
                load_page<P, false>(a, task, lp, raw);
        } else {
            load_page<P, SCHEME == KVC_MODE_CHAN>(a, task, lp, raw);
        }
    };
    if (kRing > 1) {
        // The register sets take turns (the inner loop is unrolled, so every index is a constant):
        // nothing is copied between them.
        EncTask t[kRing];
        uint4 r[kRing][NP];
#pragma unroll
        for (int j = 0; j < kRing - 1; ++j) {
            if (j > 0) task_advance(pos, a.g.ppb);
            t[j] = resolve_enc_task(a, t0 + j, pos, kMaxMode);
            if (t[j].desc_idx >= 0) load(t[j], r[j]);
        }
#pragma unroll 1
        for (int i = 0; i < PPW; i += kRing) {
#pragma unroll
            for (int j = 0; j < kRing; ++j) {
                constexpr int kAhead = kRing - 1;
                const int nb = (j + kAhead) % kRing;
                task_advance(pos, a.g.ppb);
                t[nb] = resolve_enc_task(a, i + j + kAhead < PPW ? t0 + i + j + kAhead : a.n_pages, pos, kMaxMode);  // past the end: no task
                if (t[nb].desc_idx >= 0) load(t[nb], r[nb]);
                encode_into_slot<P, SCHEME>(a, r[j], lp, t[j], slot0 + i + j, s_stage[slot0 + i + j], s_lut, s_book);
            }
        }
    } else {
#pragma unroll 1
        for (int i = 0; i < PPW; ++i) {
            const EncTask task = resolve_enc_task(a, t0 + i, pos, kMaxMode);
            task_advance(pos, a.g.ppb);
            uint4 raw[NP];
            if (task.desc_idx >= 0) load(task, raw);
            encode_into_slot<P, SCHEME>(a, raw, lp, task, slot0 + i, s_stage[slot0 + i], s_lut, s_book);
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) reserve_pool_span<kSlots>(a, s_book);
    __syncthreads();
#pragma unroll 1
    for (int i = 0; i < PPW; ++i) emit_page<kSlots>(a, s_book, slot0 + i, s_stage[slot0 + i]);
}

// ---------------------------------------------------------------------------------- decode

// dequantize: x = fp16(fp32(q) * s).  b = (q + 128) mod 256 sits in the low byte of pb; the fused
// b*s - 128*s rounds q*s once to binary32 (128*s is exact), then one rounding to FP16.
__device__ __forceinline__ uint4 dequant8_biased(const uint32_t pb[8], float s, float neg128s) {
    half2v h[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        h[k].x = (_Float16)__builtin_fmaf((float)(pb[2 * k] & 0xFFu), s, neg128s);
        h[k].y = (_Float16)__builtin_fmaf((float)(pb[2 * k + 1] & 0xFFu), s, neg128s);
    }
    return make_uint4(__builtin_bit_cast(uint32_t, h[0]), __builtin_bit_cast(uint32_t, h[1]),
                      __builtin_bit_cast(uint32_t, h[2]), __builtin_bit_cast(uint32_t, h[3]));
}

// This lane's 8 values of its quad's packet in group set p, read from the staged payload: the bits
// above each value's sign flag (hb) and the flag as 0 / -1 (sg): delta = hb ^ sg.
template <int NP>
__device__ __forceinline__ void unpack8(const DecodeArgs& a, const uint32_t* stage, const uint32_t* ginfo, int p, bool special, uint32_t hdr,
                                        uint32_t (&hb)[8], int (&sg)[8]) {
    (void)hdr;
    (void)a;  // only the bounds-checking build reads it
    const int lane = lane_id();
    const uint32_t qi = (uint32_t)lane & 3u;
    const uint32_t gi = ginfo[p * 16 + (lane >> 2)];
    uint32_t c = gi & 15u;
    const uint32_t goff = gi >> 4;
    uint32_t B = goff + qi * c;
    if (special && c == 9) B = goff;
    const uint32_t sh = (B & 3u) << 3;
    const uint32_t* p0 = stage + (B >> 2);
    KVC_CHECK(a.st, (B >> 2) + 2 < (uint32_t)Slot<NP>::kWords && B >= hdr);  // bodies start after the header bytes
    const uint32_t d0 = p0[0], d1 = p0[1], d2 = p0[2];
    uint32_t lo = __builtin_amdgcn_alignbit(d1, d0, sh);
    uint32_t hi = __builtin_amdgcn_alignbit(d2, d1, sh);
    if (special) {
        if (c == 9) {  // run packet: the body byte, 32 times
            lo = __builtin_amdgcn_perm(lo, lo, 0u);
            hi = lo;
            c = 8;
        } else if (c == 0) {  // zero-run packet
            lo = 0;
            hi = 0;
            c = 1;
        }
    }
    const uint32_t mid = shr_nibbles(lo, hi, c);  // values 4..7 start at bit 4c
    // value k sits at bits [k*c, k*c + c); delta = (u >> 1) ^ -(u & 1) taken straight from the fields
    const uint32_t w1 = c - 1u;
    const uint32_t o1 = c, o2 = c << 1, o3 = o2 + c;
    hb[0] = __builtin_amdgcn_ubfe(lo, 1u, w1), sg[0] = __builtin_amdgcn_sbfe((int)lo, 0u, 1u);
    hb[1] = __builtin_amdgcn_ubfe(lo, o1 + 1u, w1), sg[1] = __builtin_amdgcn_sbfe((int)lo, o1, 1u);
    hb[2] = __builtin_amdgcn_ubfe(lo, o2 + 1u, w1), sg[2] = __builtin_amdgcn_sbfe((int)lo, o2, 1u);
    hb[3] = __builtin_amdgcn_ubfe(lo, o3 + 1u, w1), sg[3] = __builtin_amdgcn_sbfe((int)lo, o3, 1u);
    hb[4] = __builtin_amdgcn_ubfe(mid, 1u, w1), sg[4] = __builtin_amdgcn_sbfe((int)mid, 0u, 1u);
    hb[5] = __builtin_amdgcn_ubfe(mid, o1 + 1u, w1), sg[5] = __builtin_amdgcn_sbfe((int)mid, o1, 1u);
    hb[6] = __builtin_amdgcn_ubfe(mid, o2 + 1u, w1), sg[6] = __builtin_amdgcn_sbfe((int)mid, o2, 1u);
    hb[7] = __builtin_amdgcn_ubfe(mid, o3 + 1u, w1), sg[7] = __builtin_amdgcn_sbfe((int)mid, o3, 1u);
}

// A page on its way through the decoder: the descriptor's fields, the outcome of its validation and,
// for the packed modes, the payload as it arrives from the pool (16 bytes per lane and round).
template <class P>
struct DecPage {
    uint64_t off;
    float s;
    uint32_t n16, mode;
    bool ok;
    uint4 pay[P::kRounds];
};

template <class P>
__device__ __forceinline__ bool is_packed_mode(uint32_t mode) {
    return mode == KVC_MODE_DELTA || mode == KVC_MODE_RLE || mode == KVC_MODE_PACK || (P::kChan && mode == KVC_MODE_CHAN);
}

// Take the descriptor apart, validate it against the pool and the page geometry, and start the
// payload loads of a packed page.  Nothing here waits for those loads.
template <class P>
__device__ __forceinline__ DecPage<P> dec_open(const DecodeArgs& a, uint4 dw) {
    const Extent x = page_extent<P>(a.g);
    const int lane = lane_id();
    DecPage<P> pg;
    pg.off = (uint64_t)dw.x | ((uint64_t)dw.y << 32);
    pg.s = __uint_as_float(dw.z);
    pg.n16 = dw.w & 0xFFFFu;
    pg.mode = (dw.w >> 16) & 0xFFu;
    bool ok = (pg.off & 15u) == 0 && (pg.off >> 4) + pg.n16 <= a.pool_units;
    if (pg.mode == KVC_MODE_RAW)
        ok = ok && pg.n16 == x.E >> 3;
    else if (pg.mode == KVC_MODE_INT8)
        ok = ok && pg.n16 == x.E >> 4;
    else if (is_packed_mode<P>(pg.mode))
        ok = ok && pg.n16 * 16u >= x.hdr && pg.n16 < x.E >> 4;
    else
        ok = false;
    pg.ok = ok;
#pragma unroll
    for (int z = 0; z < P::kRounds; ++z) pg.pay[z] = make_uint4(0u, 0u, 0u, 0u);
    if (ok && is_packed_mode<P>(pg.mode)) {
        const uint4* pl4 = reinterpret_cast<const uint4*>(a.pool + pg.off);
#pragma unroll
        for (int z = 0; z < P::kRounds; ++z) {
#if KVC_NT_POOL
            if ((uint32_t)lane + 64 * z < pg.n16) pg.pay[z] = load_stream(pl4 + lane + 64 * z);
#else
            if ((uint32_t)lane + 64 * z < pg.n16) pg.pay[z] = pl4[lane + 64 * z];
#endif
        }
    }
    return pg;
}

// Decode an opened page into dst.  false = validation failed, dst zeroed.
template <class P>
__device__ __forceinline__ bool dec_finish(const DecodeArgs& a, const DecPage<P>& pg, uint16_t* __restrict__ dst,
                                           uint32_t* stage, uint32_t* ginfo) {
    constexpr int NP = P::kPasses, kG = P::kGroups;
    const Extent x = page_extent<P>(a.g);
    const int lane = lane_id();
    const float s = pg.s;
    const uint32_t n16 = pg.n16, mode = pg.mode;
    char* dst_b = reinterpret_cast<char*>(a.out) + wave_uniform((int64_t)(dst - a.out) * 2);  // wave-uniform page base
    const LanePos lp = lane_pos<P>(a.g);
    if (!pg.ok) {
        zero_page(dst, a.g);
        return false;
    }
    const uint4* pl4 = reinterpret_cast<const uint4*>(a.pool + pg.off);
    if (mode == KVC_MODE_RAW) {  // stored-uncompressed bypass
#pragma unroll
        for (int p = 0; p < NP; ++p)
            if (lane_live<P>(x, p)) *reinterpret_cast<uint4*>(dst_b + pass_base_off<P, false>(a.g, p) + pass_lane_off<P, false>(a.g, lp, p)) = pl4[p * 64 + lane];
        return true;
    }
    const float neg128s = -128.0f * s;
    if (mode == KVC_MODE_INT8) {
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            if (!lane_live<P>(x, p)) continue;
            const uint2 v = reinterpret_cast<const uint2*>(pl4)[p * 64 + lane];
            uint32_t pb[8];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                pb[k] = ((v.x >> (8 * k)) + 128u);
                pb[4 + k] = ((v.y >> (8 * k)) + 128u);
            }
            store_stream(reinterpret_cast<uint4*>(dst_b + pass_base_off<P, false>(a.g, p) + pass_lane_off<P, false>(a.g, lp, p)), dequant8_biased(pb, s, neg128s));
        }
        return true;
    }
    // packed modes: stage the payload in LDS (fewer than kE/16 16-byte units)
    {
        uint4* st4 = reinterpret_cast<uint4*>(stage);
#pragma unroll
        for (int z = 0; z < P::kRounds; ++z)
            if ((uint32_t)lane + 64 * z < n16) st4[lane + 64 * z] = pg.pay[z];
    }
    wave_sync();
    // header: a lane takes the code of group g (64 groups per round); body offsets are a prefix sum of
    // body sizes
    uint32_t total = x.hdr;
    bool bad = false, special = false;
#pragma unroll
    for (int g0 = 0; g0 < kG; g0 += 64) {
        const int g = g0 + lane;
        const bool in_slot = kG % 64 == 0 || g < kG;                         // the group has an entry in ginfo
        const bool live = P::kPartial ? (uint32_t)g < (x.E >> 5) : in_slot;  // ... and exists in this page
        const uint32_t c_own = live ? (stage[g >> 3] >> ((g & 7) << 2)) & 15u : 1u;
        const uint32_t size_own = !live ? 0u : (c_own == 9) ? 1u : (c_own << 2);
        const uint32_t incl = wave_incl_scan_dpp(size_own);
        // (a group beyond a short page: a one-bit literal at the payload's end, read but never stored)
        if (in_slot) ginfo[g] = ((total + incl - size_own) << 4) | c_own;
        total += (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
        bad = bad || c_own > 9 || (mode == KVC_MODE_DELTA && (c_own == 0 || c_own == 9));
        special = special || c_own == 0 || c_own == 9;
    }
    special = __builtin_amdgcn_ballot_w64(special) != 0;  // any zero-run / run packet in the page
    if (__builtin_amdgcn_ballot_w64(bad) != 0 || ((total + 15u) >> 4) != n16) {
        zero_page(dst, a.g);
        return false;
    }
    wave_sync();
    if constexpr (P::kChan && P::kD == 64) {
        if (mode == KVC_MODE_CHAN) {
            // Mode 5 with eight octets (see the encoder): group set s holds, for this lane, pair 2s + h of its
            // octet over all 16 tokens; the lane's own tokens are values 4h .. 4h + 3 of the packet, the
            // partner's the other four.  The biased codes of a set are kept as bytes, two dwords per set; the
            // lane hands the partner the dword with the partner's tokens and receives the partner's pair for
            // its own tokens.
            const bool hi = lane >= 32;
            uint32_t pair_lo[2], pair_hi[2];  // per set: the dwords of pairs 2s and 2s + 1 for this lane's tokens
#pragma unroll
            for (int sset = 0; sset < 2; ++sset) {
                uint32_t hb[8];
                int sg[8];
                unpack8<NP>(a, stage, ginfo, sset, special, x.hdr, hb, sg);
                uint32_t b[8];
#pragma unroll
                for (int m = 0; m < 8; ++m) b[m] = (hb[m] ^ (uint32_t)sg[m]) + 128u;
                const uint32_t w0 = __builtin_amdgcn_perm(__builtin_amdgcn_perm(b[3], b[2], 0x0c0c0400u), __builtin_amdgcn_perm(b[1], b[0], 0x0c0c0400u), 0x05040100u);
                const uint32_t w1 = __builtin_amdgcn_perm(__builtin_amdgcn_perm(b[7], b[6], 0x0c0c0400u), __builtin_amdgcn_perm(b[5], b[4], 0x0c0c0400u), 0x05040100u);
                const uint32_t own = hi ? w1 : w0;  // values 4h .. 4h + 3: this lane's tokens
                const uint32_t got = (uint32_t)__builtin_amdgcn_ds_bpermute((lane ^ 32) << 2, (int)(hi ? w0 : w1));
                pair_lo[sset] = hi ? got : own;  // pair 2s: packed by the lower half's lane
                pair_hi[sset] = hi ? own : got;  // pair 2s + 1: packed by the upper half's lane
            }
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                uint32_t pb[8];
#pragma unroll
                for (int k = 0; k < 8; ++k)  // channel k = pair k / 2 = 2 (k / 4) + (k / 2) % 2, value 2p + k % 2 of the dword
                    pb[k] = (((k >> 1) & 1) ? pair_hi[k >> 2] : pair_lo[k >> 2]) >> (8 * (2 * p + (k & 1)));
                store_stream(reinterpret_cast<uint4*>(dst_b + pass_base_off<P, true>(a.g, p) + pass_lane_off<P, true>(a.g, lp, p)),
                             dequant8_biased(pb, s, neg128s));
            }
            return true;
        }
    } else if (P::kChan && mode == KVC_MODE_CHAN) {
        // Mode 5: of a run of 16 octets, group set j holds channels 2j, 2j + 1 of the lane's octet,
        // tokens 4p + (lane & 3) for p = 0..3 (value 2p + e of the packet = pass p, channel 2j + e).  The
        // biased codes of a set are kept as bytes, so that pass p then finds its eight codes at fixed
        // byte positions.
#pragma unroll
        for (int h = 0; h < NP / 4; ++h) {
            uint32_t packed[4][2];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                uint32_t hb[8];
                int sg[8];
                unpack8<NP>(a, stage, ginfo, 4 * h + j, special, x.hdr, hb, sg);
                uint32_t b[8];
#pragma unroll
                for (int m = 0; m < 8; ++m) b[m] = (hb[m] ^ (uint32_t)sg[m]) + 128u;
                packed[j][0] = __builtin_amdgcn_perm(__builtin_amdgcn_perm(b[3], b[2], 0x0c0c0400u), __builtin_amdgcn_perm(b[1], b[0], 0x0c0c0400u), 0x05040100u);
                packed[j][1] = __builtin_amdgcn_perm(__builtin_amdgcn_perm(b[7], b[6], 0x0c0c0400u), __builtin_amdgcn_perm(b[5], b[4], 0x0c0c0400u), 0x05040100u);
            }
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                uint32_t pb[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const int m = 2 * p + (k & 1);  // value index inside group set k / 2
                    pb[k] = packed[k >> 1][m >> 2] >> (8 * (m & 3));
                }
                store_stream(reinterpret_cast<uint4*>(dst_b + pass_base_off<P, true>(a.g, 4 * h + p) + pass_lane_off<P, true>(a.g, lp, 4 * h + p)),
                             dequant8_biased(pb, s, neg128s));
            }
        }
        return true;
    }
    uint32_t carry = 0;  // what a row that continues from the pass before had summed up there
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        uint32_t hb[8];  // bits above the sign flag
        int sg[8];       // 0 or -1 from the sign flag
        unpack8<NP>(a, stage, ginfo, p, special, x.hdr, hb, sg);
        uint32_t pb[8];
        if (mode == KVC_MODE_PACK) {  // no delta step was taken: the fields are the codes
#pragma unroll
            for (int k = 0; k < 8; ++k) pb[k] = (hb[k] ^ (uint32_t)sg[k]) + 128u;
        } else {
            // prefix sum along the channel index: in the lane first (each step is one xor-add), then
            // the lanes of the token row before this one
            uint32_t pre[8];
            pre[0] = hb[0] ^ (uint32_t)sg[0];
#pragma unroll
            for (int k = 1; k < 8; ++k) pre[k] = (hb[k] ^ (uint32_t)sg[k]) + pre[k - 1];
            const uint32_t tot = pre[7];
            const uint32_t incl = row_incl_scan<P>(lp, p, tot, carry);
            if (!P::kAligned) carry = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
            const uint32_t base = incl - tot + 128u;  // +128: biased codes, see dequant8_biased
#pragma unroll
            for (int k = 0; k < 8; ++k) pb[k] = pre[k] + base;
        }
        if (lane_live<P>(x, p))
            store_stream(reinterpret_cast<uint4*>(dst_b + pass_base_off<P, false>(a.g, p) + pass_lane_off<P, false>(a.g, lp, p)), dequant8_biased(pb, s, neg128s));
    }
    return true;
}

template <class P, int WAVES, int PPW>
__global__ __launch_bounds__(WAVES * 64) void k_decompress(DecodeArgs a) {
    __shared__ __align__(16) uint32_t s_stage[WAVES][Slot<P::kPasses>::kWords];
    __shared__ uint32_t s_ginfo[WAVES][P::kGroups];
    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t t0 = ((int64_t)task_block_index<1>() * WAVES + wave) * PPW;
    TaskPos pos = task_pos(t0, a.g.ppb);
    // A page's memory chain is ids -> descriptor -> payload, each a full trip to HBM.  The wave walks
    // it for all of its PPW pages side by side: every descriptor load is issued before the first is
    // looked at, then every payload load before the first page is decoded.
    DecTask task[PPW];
    uint4 dw[PPW];
    DecPage<P> pg[PPW];
#pragma unroll
    for (int i = 0; i < PPW; ++i) {
        task[i] = resolve_dec_task(a, t0 + i, pos);
        task_advance(pos, a.g.ppb);
        if (task[i].kind == 1) dw[i] = reinterpret_cast<const uint4*>(a.desc)[task[i].desc_idx];
    }
#pragma unroll
    for (int i = 0; i < PPW; ++i)
        if (task[i].kind == 1) pg[i] = dec_open<P>(a, dw[i]);
#pragma unroll
    for (int i = 0; i < PPW; ++i) {
        if (task[i].kind == 2) zero_page(task[i].dst, a.g);
        if (task[i].kind == 1 && !dec_finish<P>(a, pg[i], task[i].dst, s_stage[wave], s_ginfo[wave])) {
            if (lane == 0) atomicOr(&a.st->status, KVC_ST_CORRUPT);
        }
        wave_sync();
    }
}

// Transfer engines of the prefetch window (Algorithm 1: at most Omega_max transfers outstanding): a
// workgroup takes the next issued block from the queue, its waves decode the block's pages, and the
// completion is reported before the next block is taken.
// (pages of up to four passes whose rows do not cross passes: held within 128 VGPRs, so that four waves fit a SIMD)
template <class P, int WAVES>
__global__ __launch_bounds__(WAVES * 64) __attribute__((amdgpu_waves_per_eu(P::kPasses <= 4 && P::kAligned ? 4 : 1))) void k_decompress_window(DecodeArgs a, WindowArgs w) {
    __shared__ __align__(16) uint32_t s_stage[WAVES][Slot<P::kPasses>::kWords];
    __shared__ uint32_t s_ginfo[WAVES][P::kGroups];
    __shared__ uint32_t s_turn[2];
    __shared__ int32_t s_q[WAVES][2][64];
    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int ppb = a.g.ppb;
    if (blockIdx.x >= w.hdr->engines) return;  // the window was opened for fewer engines than the grid holds
    WindowTurn none;
    none.first = none.count = 0;
    WindowTurn turn = window_next(w, s_turn, none);
    while (turn.count) {
      // the turn's queue entries (at most 64) and the pool blocks they name, fetched one per lane and parked
      // in the wave's row of LDS: two trips to memory per turn instead of two per block
      if ((uint32_t)lane < turn.count) {
          const int32_t slot_l = w.queue[turn.first + lane];
          s_q[wave][0][lane] = slot_l;
          s_q[wave][1][lane] = a.pool_ids[slot_l];
      }
      wave_sync();
      for (uint32_t i = 0; i < turn.count; ++i) {
        const int32_t slot = __builtin_amdgcn_readfirstlane(s_q[wave][0][i]);
        const int32_t pb = __builtin_amdgcn_readfirstlane(s_q[wave][1][i]);
        // a wave takes the block's pages wave, wave + WAVES, ... four at a time: all four descriptor loads
        // are issued before the first is looked at, then all payload loads before the first page is decoded
        constexpr int kSide = 4;
        for (int pg0 = wave; pg0 < ppb; pg0 += kSide * WAVES) {
            DecTask task[kSide];
            uint4 dw[kSide];
            DecPage<P> dp[kSide];
#pragma unroll
            for (int j = 0; j < kSide; ++j) {
                const int pg = pg0 + j * WAVES;
                task[j].kind = 0;  // past the block: no task
                if (pg < ppb) task[j] = place_dec_task(a, pb, slot, pg, false);
                if (task[j].kind == 1) dw[j] = reinterpret_cast<const uint4*>(a.desc)[task[j].desc_idx];
            }
#pragma unroll
            for (int j = 0; j < kSide; ++j)
                if (task[j].kind == 1) dp[j] = dec_open<P>(a, dw[j]);
#pragma unroll
            for (int j = 0; j < kSide; ++j) {
                if (task[j].kind == 2) zero_page(task[j].dst, a.g);
                if (task[j].kind == 1 && !dec_finish<P>(a, dp[j], task[j].dst, s_stage[wave], s_ginfo[wave])) {
                    if (lane == 0) atomicOr(&a.st->status, KVC_ST_CORRUPT);
                }
                wave_sync();
            }
        }
      }
      turn = window_next(w, s_turn, turn);
    }
}

// Launch shapes by page size (NP passes of 1 KB): waves per workgroup, pages per wave.
constexpr int kCodecWaves = 4;
// large calls: about 64 KB of input per workgroup and one pool-cursor atomic for it
constexpr int enc_ppw_large(int np) { return np == 1 ? 64 / KVC_ENC_WAVES_1KB : np == 2 ? 8 : np == 3 ? 5 : np == 4 ? 4 : np == 5 ? KVC_PPW5 : np == 6 ? KVC_PPW6 : np == 7 ? KVC_PPW7 : KVC_PPW8; }
// waves per encoder workgroup in large calls
// (one-pass pages: eight waves share the workgroup's 64 slots, so that six waves instead of four fit a SIMD
// beside the LDS the slots take: 0.41 -> 0.51 of HBM peak at 16 x 32; two-pass pages lose by the same change)
constexpr int enc_waves_large(int np) { return np >= 5 ? KVC_ENC_WAVES_LONG : np == 1 ? KVC_ENC_WAVES_1KB : 4; }
// A small call (a decode step's offload of a few blocks) is latency: one page per wave (more only for
// the smallest pages), so the pages are encoded side by side instead of several in a row.  The cursor
// then takes an atomic per four pages, which only a large call would feel.
constexpr int enc_ppw_small(int np) { return np == 1 ? 4 : np == 2 ? 2 : 1; }
// a page of one or two passes is too small to cover its own memory chain: a wave walks several side by side
constexpr int dec_ppw(int np) { return np == 1 ? 4 : np == 2 ? 2 : 1; }
// calls of at most this many pages take the low-latency launch shape
#ifndef KVC_ENC_SMALL_PAGES
#define KVC_ENC_SMALL_PAGES 2048
#endif

inline dim3 page_grid(int64_t n_pages, int ppw, int waves = kCodecWaves) {
    const int64_t per_wg = (int64_t)waves * ppw;
    return dim3((unsigned)((n_pages + per_wg - 1) / per_wg));
}

// The host side of one page shape: picks the instantiation and launches it.
template <int D, int NP, bool PARTIAL>
struct ShapeOps {
    using P = Page<D, NP, PARTIAL>;

    template <int SCHEME>
    static hipError_t compress_scheme(const EncodeArgs& a, hipStream_t s) {
        const dim3 block(kCodecWaves * 64);
        if (a.n_pages <= KVC_ENC_SMALL_PAGES)
            return launch_kernel(k_compress<P, kCodecWaves, enc_ppw_small(NP), SCHEME>, page_grid(a.n_pages, enc_ppw_small(NP)), block, s, a);
        constexpr int W = enc_waves_large(NP);
        return launch_kernel(k_compress<P, W, enc_ppw_large(NP), SCHEME>, page_grid(a.n_pages, enc_ppw_large(NP), W), dim3(W * 64), s, a);
    }

    static hipError_t compress(const EncodeArgs& a, hipStream_t s) {
        // the full scheme of Algorithm 2 for every block is the common launch and gets its own
        // instantiation; any other request (another mode, or one mode per block) reads it at run time,
        // and so do all requests for pages with a short last pass
        if constexpr (PARTIAL) {
            return a.scheme == KVC_MODE_CHAN ? hipErrorInvalidValue : compress_scheme<kSchemeRowMajor>(a, s);
        } else {
            if (a.block_scheme == nullptr && a.scheme == KVC_MODE_RLE) return compress_scheme<KVC_MODE_RLE>(a, s);
            if (a.block_scheme == nullptr && a.scheme == KVC_MODE_CHAN) {
                // channel-pair groups: its own instantiations (another deal of the page to the lanes)
                if constexpr (P::kChan)
                    return compress_scheme<KVC_MODE_CHAN>(a, s);
                else
                    return hipErrorInvalidValue;
            }
            // one mode per block: where the shape has mode 5, the instantiation that can also deal a page by channel pairs
            if constexpr (P::kChan) {
                if (a.block_scheme != nullptr) return compress_scheme<kSchemeAny>(a, s);
            }
            return compress_scheme<kSchemeRowMajor>(a, s);
        }
    }

    static hipError_t decompress(const DecodeArgs& a, hipStream_t s) {
        return launch_kernel(k_decompress<P, kCodecWaves, dec_ppw(NP)>, page_grid(a.n_pages, dec_ppw(NP)), dim3(kCodecWaves * 64), s, a);
    }

    static hipError_t decompress_window(const DecodeArgs& a, const WindowArgs& w, unsigned grid, hipStream_t s) {
        return launch_kernel(k_decompress_window<P, kCodecWaves>, dim3(grid), dim3(kCodecWaves * 64), s, a, w);
    }

    // engines the current device holds at once: a larger grid would only queue workgroups behind the
    // resident ones, which keep taking turns until the queue is empty
    static int window_capacity() {
        int dev = 0, cus = 0, per_cu = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_decompress_window<P, kCodecWaves>, kCodecWaves * 64, 0) != hipSuccess) {
            (void)hipGetLastError();
            return 0;  // unknown: no cap
        }
        return cus * per_cu;
    }

    static constexpr ShapeKernels kTable = {D, NP, PARTIAL, &compress, &decompress, &decompress_window, &window_capacity};
};

}  // namespace
}  // namespace kvc
