/*
 * kvc_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * A plain, slow, one-page-at-a-time CPU statement of the KV-cache codec of
 * CXL-SpecKV (Section 3.5.2, Algorithm 2 "KV-Cache Compression", and its inverse,
 * Section 3.5.3), in the concrete byte format this repository calls KVC-1.  It exists
 * so that the GPU library can be checked against something that was written from the
 * paper and can be read against it by eye.  Only tests, the smoke check and the
 * cpu_baseline leg of the benchmark may call it.  It shares no code with the GPU path.
 *
 * Algorithm 2 in order:
 *   scaling       s = max|X| / 127                       (Alg. 2, "Scaling" step)
 *   quantize      q = round(x * s^-1)  in [-127,127]      (Alg. 2, inner loop over j,i)
 *   delta         delta[j][i] = q[j][i] - q[j][i-1], i>=2 (Alg. 2, "Delta encoding" loop)
 *   RLE           D_RLE = RunLengthEncode({delta})        (Alg. 2, last step)
 *   output        < s, D_RLE >
 * Inverse (Section 3.5.3): undo RLE, prefix-sum the deltas, multiply by s, emit FP16;
 * pages that were stored uncompressed bypass all of it.
 *
 * Where the paper leaves the byte format open, the readings are:
 *   - the quantize line's trailing "* 127" repeats the 127 already inside s; q = round(x/s);
 *   - a page is N tokens x d channels of one KV head (16 x 128 FP16 = the paper's 4 KB page);
 *   - s and s^-1 are IEEE binary32 quotients; rounding is to nearest, ties to even, of the
 *     exact product x * s^-1;
 *   - the first column has no left neighbour: delta[j][0] = q[j][0];
 *   - deltas wrap to 8 bits (exact on decode since |q| <= 127) and are zig-zag mapped to
 *     unsigned u;
 *   - RunLengthEncode works on groups of 32 consecutive u (row-major): a group of 32
 *     zeros is a zero-run packet (no body), 32 equal non-zero values are a run packet
 *     (1 byte), anything else a literal packet bit-packed at the width of its largest u;
 *   - a page with a NaN/Inf is stored raw (the bypass path); a page whose packed form is
 *     not smaller than its plain INT8 form is stored as plain INT8.
 * Two modes go beyond Algorithm 2 and are marked as extensions where they are defined: mode 4 packs
 * the codes without the delta step, mode 5 packs them in groups of one channel pair over 16 tokens.
 *
 * Floating point: the paper fixes FP16 in/out and INT8 codes; everything else here is
 * binary64 or exact integer arithmetic, except s and s^-1 which are binary32 by the
 * reading above (they are stored / define the codes).
 *
 * Pins: every function below is checked against something other than itself (FP16 conversions
 * exhaustively against a library, scale and codes by exact rational arithmetic, the bit format
 * against an independent big-integer statement, hand-worked pages, brute force on tiny pages,
 * closed forms for sizes).  Parity unpinned: the compression ratio the paper reports (3.2x, band
 * 2.5-4.0) and its accuracy figures depend on real KV caches and cannot be pinned here; the
 * ratio function itself is a sum over descriptors and is pinned by its closed forms.
 *
 * Build: gcc -O2 -std=c11 -ffp-contract=off -fPIC -shared -pthread (no -ffast-math).
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define KVO_MODE_RAW 0
#define KVO_MODE_INT8 1
#define KVO_MODE_DELTA 2
#define KVO_MODE_RLE 3
#define KVO_MODE_PACK 4 /* extension, not in Alg. 2: INT8 codes zig-zag mapped and packed as in mode 3, no delta step */
#define KVO_MODE_CHAN 5 /* extension: mode 4 with the stream regrouped by channel pair (16-token pages only) */
#define KVO_MODE_INVALID 0xFF

#define KVO_OK 0
#define KVO_ERR_ARG (-1)
#define KVO_ERR_CORRUPT (-2)
#define KVO_ERR_SPACE (-3)

/* 16-byte page descriptor: where the payload is, its scale, its size, how it was stored. */
typedef struct {
    uint64_t off;  /* byte offset of the payload in the pool, multiple of 16 */
    float scale;   /* s of Alg. 2 (0 for raw and all-zero pages) */
    uint16_t n16;  /* payload size in 16-byte units, zero padding included */
    uint8_t mode;  /* KVO_MODE_* */
    uint8_t rsvd;  /* 0 */
} kvo_desc;

/* ---------------------------------------------------------------- FP16 <-> real */

/* Value of an IEEE binary16 bit pattern: (-1)^sign * 2^(e-15) * (1 + m/1024), subnormals
 * 2^-14 * m/1024.  Every binary16 value is exactly representable in binary32. */
float kvo_half_to_float(uint16_t h) {
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1F;
    int m = h & 0x3FF;
    double v;
    if (e == 0)
        v = ldexp((double)m, -24);
    else if (e == 31)
        v = m ? (double)NAN : (double)INFINITY;
    else
        v = ldexp((double)(m + 1024), e - 25);
    return (float)(sign ? -v : v);
}

/* Nearest binary16 to a finite real, ties to even; magnitudes that round past the
 * largest finite value (65504) become infinity.  Done from the definition: pick the
 * binade, divide by its spacing, round to an integer with nearbyint (the C default
 * rounding direction is to-nearest-even). */
uint16_t kvo_float_to_half(float f) {
    uint16_t sign = signbit(f) ? 0x8000u : 0u;
    double a = fabs((double)f);
    if (isnan(a)) return (uint16_t)(sign | 0x7E00u);
    if (isinf(a)) return (uint16_t)(sign | 0x7C00u);
    if (a < ldexp(1.0, -14)) {
        /* subnormal range, spacing 2^-24; a result of 1024 is the smallest normal */
        double m = nearbyint(ldexp(a, 24));
        return (uint16_t)(sign | (uint16_t)m);
    }
    int ex;
    (void)frexp(a, &ex); /* a = fr * 2^ex, fr in [0.5,1) */
    int e = ex - 1;      /* a in [2^e, 2^(e+1)) */
    double m = nearbyint(ldexp(a, 10 - e)); /* in [1024, 2048] */
    if (m == 2048.0) {
        m = 1024.0;
        e += 1;
    }
    if (e > 15) return (uint16_t)(sign | 0x7C00u);
    return (uint16_t)(sign | (uint16_t)((e + 15) << 10) | (uint16_t)((int)m - 1024));
}

size_t kvo_pad16(size_t n) { return (n + 15u) & ~(size_t)15u; }

/* ---------------------------------------------------------------- Alg. 2, step by step */

/* Scaling and quantize steps.  Returns 1 if the page holds a NaN or Inf (then nothing
 * else is written), else 0 with *s, *s_inv and q[0..E) filled. */
int kvo_quantize_page(const uint16_t* x, int E, float* s, float* s_inv, int8_t* q) {
    float amax = 0.0f;
    for (int i = 0; i < E; ++i) {
        if ((x[i] & 0x7C00u) == 0x7C00u) return 1;
        float a = fabsf(kvo_half_to_float(x[i]));
        if (a > amax) amax = a;
    }
    if (amax == 0.0f) {
        *s = 0.0f;
        *s_inv = 0.0f;
    } else {
        *s = amax / 127.0f;  /* binary32 division */
        *s_inv = 1.0f / *s;  /* binary32 division */
    }
    for (int i = 0; i < E; ++i) {
        /* 11-bit times 24-bit significand: the product is exact in binary64 */
        double p = (double)kvo_half_to_float(x[i]) * (double)*s_inv;
        double r = nearbyint(p);
        if (r > 127.0 || r < -127.0) abort(); /* cannot happen: |x| <= amax */
        q[i] = (int8_t)r;
    }
    return 0;
}

/* The zig-zag map 0,-1,1,-2,... -> 0,1,2,3,... of an 8-bit signed value (-128 -> 255), written as its two
 * cases so that no negative value is ever shifted. */
static uint8_t zigzag8(int v) { return (uint8_t)(v >= 0 ? 2 * v : -2 * v - 1); }

/* Delta step along the channel index, first column verbatim, wrapped to 8 bits, then
 * the zig-zag map. */
void kvo_delta_zigzag(const int8_t* q, int N, int d, uint8_t* u) {
    for (int j = 0; j < N; ++j) {
        for (int i = 0; i < d; ++i) {
            int left = (i == 0) ? 0 : q[j * d + i - 1];
            int8_t delta = (int8_t)(uint8_t)((q[j * d + i] - left) & 0xFF);
            u[j * d + i] = zigzag8(delta);
        }
    }
}

/* Mode 4 (an extension beyond Algorithm 2, for data without correlation along the channel index, where
 * differencing only widens the values): the zig-zag map applied to the codes themselves. */
void kvo_zigzag_codes(const int8_t* q, int E, uint8_t* u) {
    for (int i = 0; i < E; ++i) {
        u[i] = zigzag8(q[i]);
    }
}

/* Mode 5 (an extension beyond Algorithm 2, for 16-token pages): the codes of mode 4, but put into the
 * stream so that a group of 32 holds one pair of neighbouring channels over all 16 tokens.  KV channels
 * differ in scale far more than the tokens of one channel do, so such a group packs at the width its own
 * channels need instead of the width of the widest of 32 neighbouring channels.
 * Element (token t, channel c) sits in octet o = c / 8 of the channels, pair j = (c / 2) mod 4 of that
 * octet.  The octets are taken in runs of W = min(16, d / 8); inside a run the groups are ordered by
 * pair index first: g = ((o div W) * 4 + j) * W + o mod W, and the element goes to position
 * k = (t mod 4) * 8 + (t div 4) * 2 + (c mod 2) of its group.  (The order inside a group and of the
 * groups is free as far as the ratio goes; this one lets a GPU lane that holds tokens t, t+4, t+8, t+12
 * of one octet emit whole bytes, sixteen octets at a time.) */
/* The group formula fills the page's groups exactly once each only when the channel octets make whole
 * runs of W: d / 8 <= 16 (one run) or d / 8 a multiple of 16.  Other channel counts (160, 192, 224) have
 * no mode 5. */
static int chan_geometry_ok(int N, int d) { return N == 16 && (d / 8 <= 16 || (d / 8) % 16 == 0); }

static int chan_group(int c, int d) {
    int o = c / 8, j = (c / 2) % 4;
    int W = d / 8 < 16 ? d / 8 : 16;
    return ((o / W) * 4 + j) * W + o % W;
}

void kvo_zigzag_codes_by_channel(const int8_t* q, int d, uint8_t* u) {
    for (int t = 0; t < 16; ++t)
        for (int c = 0; c < d; ++c) {
            int g = chan_group(c, d);
            int k = (t % 4) * 8 + (t / 4) * 2 + (c % 2);
            u[32 * g + k] = zigzag8(q[t * d + c]);
        }
}

static int bit_length(unsigned v) {
    int n = 0;
    while (v) {
        ++n;
        v >>= 1;
    }
    return n;
}

/* RunLengthEncode over groups of 32.  out must hold ceil(G/2) + 32*G bytes.
 * with_runs = 0 gives the "INT8 + Delta" ablation scheme (literal packets only).
 * Returns the unpadded byte count. */
size_t kvo_rle_pack(const uint8_t* u, int E, int with_runs, uint8_t* out) {
    int G = E / 32;
    size_t hdr = (size_t)(G + 1) / 2;
    memset(out, 0, hdr);
    size_t pos = hdr;
    for (int g = 0; g < G; ++g) {
        const uint8_t* ug = u + 32 * g;
        unsigned umax = 0;
        int all_equal = 1;
        for (int k = 0; k < 32; ++k) {
            if (ug[k] > umax) umax = ug[k];
            if (ug[k] != ug[0]) all_equal = 0;
        }
        int code;
        if (with_runs && umax == 0) {
            code = 0; /* zero-run packet: no body */
        } else if (with_runs && all_equal) {
            code = 9; /* run packet: one byte */
            out[pos++] = ug[0];
        } else {
            int w = bit_length(umax);
            if (w == 0) w = 1;
            code = w;
            memset(out + pos, 0, (size_t)(4 * w));
            for (int k = 0; k < 32; ++k)
                for (int b = 0; b < w; ++b) {
                    int bit = (ug[k] >> b) & 1;
                    int p = k * w + b;
                    out[pos + (size_t)(p >> 3)] |= (uint8_t)(bit << (p & 7));
                }
            pos += (size_t)(4 * w);
        }
        out[g >> 1] |= (uint8_t)((g & 1) ? (code << 4) : code);
    }
    return pos;
}

/* Encode one page.  payload must hold 2*E bytes.  scheme = requested mode 0..5 (5: N = 16 and d <= 128 or a
 * multiple of 128 only).
 * Fills desc (off left at 0) and returns the padded payload size in bytes, or <0. */
int64_t kvo_encode_page(const uint16_t* x, int N, int d, int scheme, uint8_t* payload, kvo_desc* desc) {
    if (N < 1 || d < 32 || d % 32 != 0 || scheme < 0 || scheme > 5) return KVO_ERR_ARG;
    if (scheme == KVO_MODE_CHAN && !chan_geometry_ok(N, d)) return KVO_ERR_ARG;
    int E = N * d;
    desc->off = 0;
    desc->rsvd = 0;
    float s = 0.0f, s_inv = 0.0f;
    int8_t* q = (int8_t*)malloc((size_t)E);
    int nonfinite = kvo_quantize_page(x, E, &s, &s_inv, q);
    if (scheme == KVO_MODE_RAW || nonfinite) {
        memcpy(payload, x, (size_t)E * 2);
        desc->scale = 0.0f;
        desc->mode = KVO_MODE_RAW;
        desc->n16 = (uint16_t)(E * 2 / 16);
        free(q);
        return (int64_t)E * 2;
    }
    size_t int8_bytes = kvo_pad16((size_t)E);
    size_t n = 0;
    int mode = scheme;
    if (scheme != KVO_MODE_INT8) {
        uint8_t* u = (uint8_t*)malloc((size_t)E);
        uint8_t* tmp = (uint8_t*)malloc((size_t)E / 64 + 1 + (size_t)E);
        if (scheme == KVO_MODE_PACK)
            kvo_zigzag_codes(q, E, u);
        else if (scheme == KVO_MODE_CHAN)
            kvo_zigzag_codes_by_channel(q, d, u);
        else
            kvo_delta_zigzag(q, N, d, u);
        size_t raw_n = kvo_rle_pack(u, E, scheme != KVO_MODE_DELTA, tmp);
        n = kvo_pad16(raw_n);
        if (n >= int8_bytes) {
            mode = KVO_MODE_INT8; /* packing did not beat plain INT8 */
        } else {
            memcpy(payload, tmp, raw_n);
            memset(payload + raw_n, 0, n - raw_n);
        }
        free(u);
        free(tmp);
    }
    if (mode == KVO_MODE_INT8) {
        memcpy(payload, q, (size_t)E);
        memset(payload + E, 0, int8_bytes - (size_t)E);
        n = int8_bytes;
    }
    desc->scale = s;
    desc->mode = (uint8_t)mode;
    desc->n16 = (uint16_t)(n / 16);
    free(q);
    return (int64_t)n;
}

/* Recover the INT8 codes of a page stored in mode 1 to 5. */
int kvo_decode_codes(const uint8_t* payload, size_t nbytes, int mode, int N, int d, int8_t* q) {
    int E = N * d, G = E / 32;
    if (mode == KVO_MODE_INT8) {
        if (nbytes != kvo_pad16((size_t)E)) return KVO_ERR_CORRUPT;
        memcpy(q, payload, (size_t)E);
        return KVO_OK;
    }
    if (mode != KVO_MODE_DELTA && mode != KVO_MODE_RLE && mode != KVO_MODE_PACK && mode != KVO_MODE_CHAN) return KVO_ERR_CORRUPT;
    if (mode == KVO_MODE_CHAN && !chan_geometry_ok(N, d)) return KVO_ERR_CORRUPT;
    const int runs = mode != KVO_MODE_DELTA; /* zero-run and run packets allowed */
    size_t hdr = (size_t)(G + 1) / 2;
    if (nbytes < hdr) return KVO_ERR_CORRUPT;
    /* the encoder stores a page whose packed form is not smaller than its INT8 form as INT8 (the fallback
     * step of kvo_encode_page), so no valid packed page is that large */
    if (nbytes >= kvo_pad16((size_t)E)) return KVO_ERR_CORRUPT;
    size_t pos = hdr;
    uint8_t* u = (uint8_t*)malloc((size_t)E);
    for (int g = 0; g < G; ++g) {
        int code = (g & 1) ? (payload[g >> 1] >> 4) : (payload[g >> 1] & 0xF);
        uint8_t* ug = u + 32 * g;
        if (code == 0 && runs) {
            memset(ug, 0, 32);
        } else if (code == 9 && runs) {
            if (pos + 1 > nbytes) goto corrupt;
            memset(ug, payload[pos], 32);
            pos += 1;
        } else if (code >= 1 && code <= 8) {
            int w = code;
            if (pos + (size_t)(4 * w) > nbytes) goto corrupt;
            for (int k = 0; k < 32; ++k) {
                unsigned v = 0;
                for (int b = 0; b < w; ++b) {
                    int p = k * w + b;
                    v |= (unsigned)((payload[pos + (size_t)(p >> 3)] >> (p & 7)) & 1) << b;
                }
                ug[k] = (uint8_t)v;
            }
            pos += (size_t)(4 * w);
        } else {
            goto corrupt;
        }
    }
    if (kvo_pad16(pos) != nbytes) goto corrupt;
    if (mode == KVO_MODE_CHAN) { /* undo the regrouping and the zig-zag map; there was no delta step */
        for (int t = 0; t < 16; ++t)
            for (int c = 0; c < d; ++c) {
                unsigned uu = u[32 * chan_group(c, d) + (t % 4) * 8 + (t / 4) * 2 + (c % 2)];
                q[t * d + c] = (int8_t)((int)(uu >> 1) ^ -(int)(uu & 1));
            }
        free(u);
        return KVO_OK;
    }
    /* undo zig-zag, then (modes 2, 3) the prefix sum along the channel index, wrapped to 8 bits */
    for (int j = 0; j < N; ++j) {
        int acc = 0;
        for (int i = 0; i < d; ++i) {
            unsigned uu = u[j * d + i];
            int delta = (int)(uu >> 1) ^ -(int)(uu & 1);
            if (mode == KVO_MODE_PACK) acc = 0;
            acc = (int8_t)(uint8_t)((acc + delta) & 0xFF);
            q[j * d + i] = (int8_t)acc;
        }
    }
    free(u);
    return KVO_OK;
corrupt:
    free(u);
    return KVO_ERR_CORRUPT;
}

/* Decode one page: out gets E FP16 bit patterns.  On error out is zero-filled. */
int kvo_decode_page(const uint8_t* payload, const kvo_desc* desc, int N, int d, uint16_t* out) {
    int E = N * d;
    size_t nbytes = (size_t)desc->n16 * 16;
    if (desc->mode == KVO_MODE_RAW) {
        if (nbytes != (size_t)E * 2) goto bad;
        memcpy(out, payload, nbytes);
        return KVO_OK;
    }
    {
        int8_t* q = (int8_t*)malloc((size_t)E);
        int rc = kvo_decode_codes(payload, nbytes, desc->mode, N, d, q);
        if (rc != KVO_OK) {
            free(q);
            goto bad;
        }
        for (int i = 0; i < E; ++i) {
            float r = (float)q[i] * desc->scale; /* binary32 multiply */
            out[i] = kvo_float_to_half(r);       /* then one rounding to binary16 */
        }
        free(q);
        return KVO_OK;
    }
bad:
    memset(out, 0, (size_t)E * 2);
    return KVO_ERR_CORRUPT;
}

/* ---------------------------------------------------------------- whole-batch drivers */

typedef struct {
    const uint16_t* x;
    int64_t p0, p1;
    int N, d, scheme;
    uint8_t* buf;     /* this worker's payloads, back to back */
    uint64_t used;
    kvo_desc* desc;   /* global descriptor array; off is worker-relative until fixed */
    int rc;
} enc_job;

static void* enc_worker(void* arg) {
    enc_job* j = (enc_job*)arg;
    size_t E = (size_t)j->N * (size_t)j->d;
    j->used = 0;
    j->rc = KVO_OK;
    for (int64_t p = j->p0; p < j->p1; ++p) {
        int64_t n = kvo_encode_page(j->x + (size_t)p * E, j->N, j->d, j->scheme, j->buf + j->used, &j->desc[p]);
        if (n < 0) {
            j->rc = (int)n;
            return NULL;
        }
        j->desc[p].off = j->used;
        j->used += (uint64_t)n;
    }
    return NULL;
}

/* Encode n_pages pages, payloads placed back to back in page order starting at pool[0].
 * Threads take contiguous page ranges; the result does not depend on n_threads.
 * Returns bytes used, or <0 (KVO_ERR_SPACE if the pool is too small). */
int64_t kvo_compress_pages(const uint16_t* x, int64_t n_pages, int N, int d, int scheme, uint8_t* pool,
                           uint64_t pool_bytes, kvo_desc* desc, int n_threads) {
    if (n_pages < 0 || n_threads < 1) return KVO_ERR_ARG;
    if (n_threads > n_pages) n_threads = n_pages > 0 ? (int)n_pages : 1;
    size_t E = (size_t)N * (size_t)d;
    enc_job* jobs = (enc_job*)calloc((size_t)n_threads, sizeof(enc_job));
    pthread_t* th = (pthread_t*)calloc((size_t)n_threads, sizeof(pthread_t));
    for (int t = 0; t < n_threads; ++t) {
        enc_job* j = &jobs[t];
        j->x = x;
        j->p0 = n_pages * t / n_threads;
        j->p1 = n_pages * (t + 1) / n_threads;
        j->N = N;
        j->d = d;
        j->scheme = scheme;
        j->desc = desc;
        j->buf = (uint8_t*)malloc((size_t)(j->p1 - j->p0) * E * 2 + 16);
        if (n_threads == 1)
            enc_worker(j);
        else
            pthread_create(&th[t], NULL, enc_worker, j);
    }
    int64_t total = 0;
    int rc = KVO_OK;
    for (int t = 0; t < n_threads; ++t) {
        enc_job* j = &jobs[t];
        if (n_threads > 1) pthread_join(th[t], NULL);
        if (j->rc != KVO_OK) rc = j->rc;
        if (rc == KVO_OK) {
            if ((uint64_t)total + j->used > pool_bytes) {
                rc = KVO_ERR_SPACE;
            } else {
                memcpy(pool + total, j->buf, j->used);
                for (int64_t p = j->p0; p < j->p1; ++p) desc[p].off += (uint64_t)total;
                total += (int64_t)j->used;
            }
        }
        free(j->buf);
    }
    free(jobs);
    free(th);
    return rc == KVO_OK ? total : rc;
}

typedef struct {
    const uint8_t* pool;
    uint64_t pool_bytes;
    const kvo_desc* desc;
    const int64_t* page_ids; /* NULL = identity */
    int64_t p0, p1;
    int N, d;
    uint16_t* out;
    int64_t n_bad;
} dec_job;

static void* dec_worker(void* arg) {
    dec_job* j = (dec_job*)arg;
    size_t E = (size_t)j->N * (size_t)j->d;
    j->n_bad = 0;
    for (int64_t p = j->p0; p < j->p1; ++p) {
        const kvo_desc* ds = &j->desc[j->page_ids ? j->page_ids[p] : p];
        uint16_t* o = j->out + (size_t)p * E;
        if (ds->off % 16 != 0 || ds->off + (uint64_t)ds->n16 * 16 > j->pool_bytes) {
            memset(o, 0, E * 2);
            j->n_bad++;
            continue;
        }
        if (kvo_decode_page(j->pool + ds->off, ds, j->N, j->d, o) != KVO_OK) j->n_bad++;
    }
    return NULL;
}

/* Decode n_pages pages into out[n_pages][N][d]; output page p comes from descriptor
 * page_ids[p] (or p).  Returns the number of pages that failed to decode (zero-filled). */
int64_t kvo_decompress_pages(const uint8_t* pool, uint64_t pool_bytes, const kvo_desc* desc, const int64_t* page_ids,
                             int64_t n_pages, int N, int d, uint16_t* out, int n_threads) {
    if (n_pages < 0 || n_threads < 1) return KVO_ERR_ARG;
    if (n_threads > n_pages) n_threads = n_pages > 0 ? (int)n_pages : 1;
    dec_job* jobs = (dec_job*)calloc((size_t)n_threads, sizeof(dec_job));
    pthread_t* th = (pthread_t*)calloc((size_t)n_threads, sizeof(pthread_t));
    for (int t = 0; t < n_threads; ++t) {
        dec_job* j = &jobs[t];
        j->pool = pool;
        j->pool_bytes = pool_bytes;
        j->desc = desc;
        j->page_ids = page_ids;
        j->p0 = n_pages * t / n_threads;
        j->p1 = n_pages * (t + 1) / n_threads;
        j->N = N;
        j->d = d;
        j->out = out;
        if (n_threads == 1)
            dec_worker(j);
        else
            pthread_create(&th[t], NULL, dec_worker, j);
    }
    int64_t bad = 0;
    for (int t = 0; t < n_threads; ++t) {
        if (n_threads > 1) pthread_join(th[t], NULL);
        bad += jobs[t].n_bad;
    }
    free(jobs);
    free(th);
    return bad;
}
