/* Runs the CPU oracle (oracle/kvc_oracle.c, compiled into this program with AddressSanitizer and
 * UndefinedBehaviorSanitizer) over cases a test writes to a file, and writes what the oracle returned.
 * Test infrastructure only.  File format, little-endian, repeated until end of input:
 *   int32 kind (1 = encode then decode, 2 = decode only), N, d, scheme, n_pages, n_threads; int64 pool_bytes
 *   kind 1: uint16 x[n_pages][N][d]
 *   kind 2: kvo_desc desc[n_pages]; uint8 pool[pool_bytes]
 * Output per record: int64 used (kind 1; pool_bytes for kind 2), int64 bad; kind 1 also desc[n_pages] and
 * pool[used]; then uint16 out[n_pages][N][d]. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    uint64_t off;
    float scale;
    uint16_t n16;
    uint8_t mode, rsvd;
} desc_t;

int64_t kvo_compress_pages(const uint16_t* x, int64_t n_pages, int N, int d, int scheme, uint8_t* pool, uint64_t pool_bytes,
                           desc_t* desc, int n_threads);
int64_t kvo_decompress_pages(const uint8_t* pool, uint64_t pool_bytes, const desc_t* desc, const int64_t* page_ids,
                             int64_t n_pages, int N, int d, uint16_t* out, int n_threads);

static void must(int ok, const char* what) {
    if (!ok) {
        fprintf(stderr, "oracle_san_driver: %s\n", what);
        exit(2);
    }
}

int main(int argc, char** argv) {
    must(argc == 3, "usage: oracle_san_driver <cases> <results>");
    FILE* in = fopen(argv[1], "rb");
    FILE* out = fopen(argv[2], "wb");
    must(in && out, "cannot open files");
    int32_t h[6];
    int n_records = 0;
    while (fread(h, sizeof h, 1, in) == 1) {
        int64_t pool_bytes;
        must(fread(&pool_bytes, 8, 1, in) == 1, "truncated header");
        const int kind = h[0], N = h[1], d = h[2], scheme = h[3], n_threads = h[5];
        const int64_t n = h[4];
        const size_t E = (size_t)N * (size_t)d;
        desc_t* desc = (desc_t*)calloc((size_t)n + 1, sizeof(desc_t));
        uint16_t* dec = (uint16_t*)calloc((size_t)n * E + 1, 2);
        uint8_t* pool;
        int64_t used;
        if (kind == 1) {
            uint16_t* x = (uint16_t*)malloc((size_t)n * E * 2 + 2);
            must(fread(x, 2, (size_t)n * E, in) == (size_t)n * E, "truncated pages");
            /* exactly the capacity the encoder may need, so that one byte too many is caught */
            const size_t cap = (size_t)n * E * 2;
            pool = (uint8_t*)malloc(cap + 1);
            used = kvo_compress_pages(x, n, N, d, scheme, pool, cap, desc, n_threads);
            must(used >= 0, "compress failed");
            free(x);
        } else {
            must(fread(desc, sizeof(desc_t), (size_t)n, in) == (size_t)n, "truncated descriptors");
            pool = (uint8_t*)malloc((size_t)pool_bytes + 1);
            must(fread(pool, 1, (size_t)pool_bytes, in) == (size_t)pool_bytes, "truncated pool");
            used = pool_bytes;
        }
        const int64_t bad = kvo_decompress_pages(pool, (uint64_t)used, desc, NULL, n, N, d, dec, n_threads);
        fwrite(&used, 8, 1, out);
        fwrite(&bad, 8, 1, out);
        if (kind == 1) {
            fwrite(desc, sizeof(desc_t), (size_t)n, out);
            fwrite(pool, 1, (size_t)used, out);
        }
        fwrite(dec, 2, (size_t)n * E, out);
        free(desc);
        free(dec);
        free(pool);
        ++n_records;
    }
    fclose(in);
    must(fclose(out) == 0, "write failed");
    printf("oracle_san_driver: %d records\n", n_records);
    return 0;
}
