// A client of libkvc's C ABI that uses nothing but the HIP runtime and include/kvc.h: no Python, no
// torch.  It builds a seeded FP16 cache on the host, runs compress -> stats -> decompress ->
// gather-decompress through the library and checks what holds without an oracle:
//   * every page is stored in the requested mode or one of its fall-backs, sizes add up;
//   * the reconstruction error bound of the quantizer (Algorithm 2, scaling and quantize steps):
//     |x - xhat| <= amax/254 * (1 + 2^-14) + half an FP16 ulp of xhat;
//   * gather-decompress through a block table returns the same blocks as the plain decompress.
// Exit status 0 = all checks passed; it prints one line per step.
#include <hip/hip_runtime_api.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "kvc.h"

#define HIP_OK(call)                                                                 \
    do {                                                                             \
        hipError_t e_ = (call);                                                      \
        if (e_ != hipSuccess) {                                                      \
            std::printf("HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__); \
            return 2;                                                                \
        }                                                                            \
    } while (0)
#define KVC_OK_OR_FAIL(call)                                                  \
    do {                                                                      \
        int r_ = (call);                                                      \
        if (r_ != KVC_OK) {                                                   \
            std::printf("%s -> %d (%s)\n", #call, r_, kvc_strerror(r_));      \
            return 3;                                                         \
        }                                                                     \
    } while (0)

static float half_to_float(uint16_t h) {
    const uint32_t sign = (uint32_t)(h >> 15) << 31, exp = (h >> 10) & 31u, man = h & 1023u;
    float v;
    if (exp == 0)
        v = std::ldexp((float)man, -24);
    else if (exp == 31)
        v = man ? NAN : INFINITY;
    else
        v = std::ldexp((float)(man | 1024u), (int)exp - 25);
    return sign ? -v : v;
}

static uint16_t float_to_half(float f) {  // round to nearest even; inputs here stay in the normal range
    uint32_t x;
    std::memcpy(&x, &f, 4);
    const uint32_t sign = (x >> 16) & 0x8000u;
    int32_t exp = (int32_t)((x >> 23) & 255u) - 127 + 15;
    uint32_t man = x & 0x7FFFFFu;
    if (exp <= 0) return (uint16_t)sign;
    if (exp >= 31) return (uint16_t)(sign | 0x7BFFu);
    uint32_t h = ((uint32_t)exp << 10) | (man >> 13);
    const uint32_t rest = man & 0x1FFFu;
    if (rest > 0x1000u || (rest == 0x1000u && (h & 1u))) ++h;
    return (uint16_t)(sign | h);
}

static uint32_t lcg(uint32_t& s) {
    s = s * 1664525u + 1013904223u;
    return s;
}

static float gauss(uint32_t& s) {  // Box-Muller on two uniform draws
    const float u1 = ((lcg(s) >> 8) + 1) * (1.0f / 16777217.0f), u2 = (lcg(s) >> 8) * (1.0f / 16777216.0f);
    return std::sqrt(-2.0f * std::log(u1)) * std::cos(6.28318530718f * u2);
}

int main() {
    const int N = 16, d = 128, ppb = 8, n_blocks = 512;  // 4096 pages of 4 KB
    const int E = N * d;
    const size_t n_pages = (size_t)n_blocks * ppb, n_elem = n_pages * E;
    std::vector<uint16_t> h_x(n_elem);
    uint32_t seed = 20251211u;
    std::vector<float> chan(d);
    for (size_t p = 0; p < n_pages; ++p) {
        if (p % ppb == 0)
            for (int i = 0; i < d; ++i) chan[i] = std::exp(0.5f * gauss(seed));
        for (int j = 0; j < N; ++j)
            for (int i = 0; i < d; ++i) h_x[p * E + j * d + i] = float_to_half(gauss(seed) * chan[i]);
    }
    for (int i = 0; i < E; ++i) h_x[5 * (size_t)E + i] = 0;  // an all-zero page
    h_x[9 * (size_t)E + 77] = 0x7C00;                        // a page with +Inf: stored RAW

    uint16_t *d_x = nullptr, *d_out = nullptr, *d_g = nullptr;
    uint8_t* d_pool = nullptr;
    kvc_desc* d_desc = nullptr;
    const uint64_t pool_bytes = n_elem * 2 + 4096;
    HIP_OK(hipMalloc((void**)&d_x, n_elem * 2));
    HIP_OK(hipMalloc((void**)&d_out, n_elem * 2));
    HIP_OK(hipMalloc((void**)&d_pool, pool_bytes));
    HIP_OK(hipMalloc((void**)&d_desc, n_pages * sizeof(kvc_desc)));
    HIP_OK(hipMemcpy(d_x, h_x.data(), n_elem * 2, hipMemcpyHostToDevice));
    HIP_OK(hipMemset(d_out, 0xFF, n_elem * 2));

    kvc_config cfg;
    cfg.tokens_per_block = N;
    cfg.head_dim = d;
    cfg.pages_per_block = ppb;
    cfg.scheme = KVC_MODE_RLE;
    kvc_ctx* ctx = nullptr;
    KVC_OK_OR_FAIL(kvc_create(&ctx, &cfg));
    KVC_OK_OR_FAIL(kvc_bind_pool(ctx, d_pool, pool_bytes, d_desc, n_pages));
    KVC_OK_OR_FAIL(kvc_reset_pool(ctx, nullptr));
    KVC_OK_OR_FAIL(kvc_compress_blocks(ctx, d_x, n_blocks, nullptr, nullptr, n_blocks, nullptr));
    kvc_stats_t st;
    KVC_OK_OR_FAIL(kvc_stats(ctx, &st, nullptr));
    const uint64_t stored = st.pages[0] + st.pages[1] + st.pages[2] + st.pages[3] + st.pages[4] + st.pages[5];
    std::printf("compress: %llu pages (raw %llu, int8 %llu, rle %llu), pool %llu bytes, ratio %.3f\n",
                (unsigned long long)stored, (unsigned long long)st.pages[0], (unsigned long long)st.pages[1],
                (unsigned long long)st.pages[3], (unsigned long long)st.pool_bytes_used,
                (double)(n_elem * 2) / (double)(st.payload_bytes + 16 * stored));
    if (stored != n_pages || st.pages[0] != 1 || st.pages[2] != 0 || st.pages[4] != 0 || st.pages[5] != 0 || st.pages_invalid != 0 ||
        st.status != 0 || st.payload_bytes != st.pool_bytes_used) {
        std::printf("unexpected statistics\n");
        return 4;
    }

    KVC_OK_OR_FAIL(kvc_decompress_blocks(ctx, d_out, n_blocks, nullptr, nullptr, n_blocks, nullptr));
    std::vector<uint16_t> h_out(n_elem);
    HIP_OK(hipMemcpy(h_out.data(), d_out, n_elem * 2, hipMemcpyDeviceToHost));
    size_t worst_page = 0;
    double worst = 0.0;
    for (size_t p = 0; p < n_pages; ++p) {
        const uint16_t* x = &h_x[p * E];
        const uint16_t* y = &h_out[p * E];
        if (p == 9) {  // RAW page: bit-exact
            if (std::memcmp(x, y, (size_t)E * 2) != 0) {
                std::printf("RAW page differs\n");
                return 5;
            }
            continue;
        }
        float amax = 0.0f;
        for (int i = 0; i < E; ++i) amax = std::fmax(amax, std::fabs(half_to_float(x[i])));
        for (int i = 0; i < E; ++i) {
            const float xv = half_to_float(x[i]), yv = half_to_float(y[i]);
            const float ay = std::fabs(yv);
            const float ulp = ay >= 6.103515625e-05f ? std::ldexp(1.0f, std::ilogb(ay) - 10) : 5.9604644775390625e-08f;
            const double bound = (double)amax / 254.0 * (1.0 + 1.0 / 16384.0) + 0.5 * ulp;
            const double err = std::fabs((double)xv - (double)yv);
            if (err > bound) {
                std::printf("page %zu element %d: |%g - %g| = %g exceeds %g\n", p, i, xv, yv, err, bound);
                return 6;
            }
            if (bound > 0 && err / bound > worst) {
                worst = err / bound;
                worst_page = p;
            }
        }
    }
    std::printf("decompress: error bound holds on all %zu pages (tightest: %.3f of the bound, page %zu)\n", n_pages, worst,
                worst_page);

    // gather: 4 sequences x 8 predicted logical blocks over a reversed block table, one layer
    const int n_seq = 4, k = 8, max_blocks = n_blocks / n_seq;
    std::vector<int32_t> h_bt((size_t)n_seq * max_blocks), h_pred((size_t)n_seq * k);
    for (int s = 0; s < n_seq; ++s)
        for (int b = 0; b < max_blocks; ++b) h_bt[(size_t)s * max_blocks + b] = n_blocks - 1 - (s * max_blocks + b);
    for (int s = 0; s < n_seq; ++s)
        for (int j = 0; j < k; ++j) h_pred[(size_t)s * k + j] = (int32_t)(lcg(seed) % (uint32_t)max_blocks);
    int32_t *d_bt = nullptr, *d_pred = nullptr;
    const size_t g_elem = (size_t)n_seq * k * ppb * E;
    HIP_OK(hipMalloc((void**)&d_bt, h_bt.size() * 4));
    HIP_OK(hipMalloc((void**)&d_pred, h_pred.size() * 4));
    HIP_OK(hipMalloc((void**)&d_g, g_elem * 2));
    HIP_OK(hipMemcpy(d_bt, h_bt.data(), h_bt.size() * 4, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(d_pred, h_pred.data(), h_pred.size() * 4, hipMemcpyHostToDevice));
    KVC_OK_OR_FAIL(kvc_gather_decompress(ctx, d_g, d_bt, max_blocks, d_pred, n_seq, k, 1, n_blocks, nullptr));
    KVC_OK_OR_FAIL(kvc_stats(ctx, &st, nullptr));
    std::vector<uint16_t> h_g(g_elem);
    HIP_OK(hipMemcpy(h_g.data(), d_g, g_elem * 2, hipMemcpyDeviceToHost));
    for (int s = 0; s < n_seq; ++s)
        for (int j = 0; j < k; ++j) {
            const int pool_block = h_bt[(size_t)s * max_blocks + h_pred[(size_t)s * k + j]];
            if (std::memcmp(&h_g[((size_t)s * k + j) * ppb * E], &h_out[(size_t)pool_block * ppb * E], (size_t)ppb * E * 2) != 0) {
                std::printf("gather: sequence %d prediction %d differs from block %d\n", s, j, pool_block);
                return 7;
            }
        }
    std::printf("gather-decompress: %d blocks equal to the plain decompress\n", n_seq * k);

    // a host-visible error: more blocks than the descriptor table holds
    if (kvc_compress_blocks(ctx, d_x, n_blocks + 1, nullptr, nullptr, n_blocks + 1, nullptr) != KVC_ERR_ARG) {
        std::printf("oversized call was not rejected\n");
        return 8;
    }
    kvc_destroy(ctx);
    (void)hipFree(d_x);
    (void)hipFree(d_out);
    (void)hipFree(d_g);
    (void)hipFree(d_pool);
    (void)hipFree(d_desc);
    (void)hipFree(d_bt);
    (void)hipFree(d_pred);
    std::printf("abi client ok\n");
    return 0;
}
