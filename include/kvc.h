/*
 * kvc.h -- C ABI of libkvc: the KV-cache page codec of CXL-SpecKV for one AMD MI355X (gfx950).
 *
 * The library encodes paged FP16 K/V blocks into a compressed pool when they are offloaded
 * (the paper's Compression Engine, Section 3.5.2, Algorithm 2) and decodes pool blocks back into
 * a paged FP16 buffer when they are prefetched (Decompression Engine, Section 3.5.3; the
 * scatter-gather fetch through a translation table of Section 3.4.2, Algorithm 1).  The remote
 * (CXL) tier of the paper is a second buffer in the same GPU's HBM.
 *
 * Geometry.  A PAGE is N tokens x d channels of one KV head, FP16, row-major (N*d*2 bytes; 16 x 128
 * gives the paper's 4 KB page).  Any N >= 1 and any d that is a multiple of 32 up to 256 with N*d <= 4096 is
 * accepted.  The kernels are compiled per channel count and page length; pages that are a whole number of
 * 512-element passes with N in {8, 16, 32} (every d at N = 16) have instantiations of their own, other token
 * counts run on ones that read N at run time (a little slower).  A BLOCK is `pages_per_block` pages (all KV
 * heads, or K and V of all heads, of one 16-token block).  A cache buffer is FP16 [n_blocks][ppb][N][d] unless
 * kvc_set_cache_layout gives other strides.
 *
 * Compressed form of a page = one 16-byte descriptor (kvc_desc) + a payload of n16*16 bytes in
 * the pool.  Payload by mode:
 *   0 RAW    the N*d*2 input bytes unchanged (requested, or the page holds a NaN/Inf);
 *   1 INT8   q[j][i] = round_half_even(x * (1/s)), s = max|X|/127 (binary32), N*d bytes;
 *   2 DELTA  q differenced along i (first column verbatim), wrapped to 8 bits, zig-zag mapped to
 *            u, cut into groups of 32; header of one 4-bit code per group (group g in byte g/2,
 *            even g in the low nibble) followed by the group bodies; code w in 1..8 = literal
 *            packet, 4*w bytes, u_k in bits [k*w,(k+1)*w) of the little-endian bit string;
 *   3 RLE    as 2, plus code 0 = 32 zeros (no body) and code 9 = 32 copies of one byte (1 byte);
 *   4 PACK   as 3 with u = zig-zag of q itself, no differencing (for data without correlation
 *            along the channel index; not part of the paper's algorithm);
 *   5 CHAN   as 4 with the values regrouped so that a group holds one pair of neighbouring channels
 *            over the 16 tokens of the page (see KVC_MODE_CHAN below; N = 16, d = 64, 128 or 256 only; not part
 *            of the paper's algorithm);
 *   payloads are zero-padded to 16 bytes; a mode-2/3/4/5 page whose payload would not be smaller
 *   than its INT8 payload is stored as mode 1.
 * Decoding yields fp16(fp32(q) * s), one binary32 multiply and one round-to-nearest-even.
 *
 * Memory.  Every data pointer below is DEVICE memory allocated and owned by the caller; the
 * library owns only the host-side context and a small device state block (pool cursor, sticky
 * status).  `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *
 * Asynchrony and errors.  compress / decompress / gather only enqueue kernels.  They return 0 or a
 * negative KVC_ERR_* for faults the host can see (nothing is enqueued then).  Faults only the
 * device can see set sticky KVC_ST_* bits: the page gets mode 0xFF (compress) or is zero-filled
 * (decompress); kvc_stats() reports them.  Block ids < 0 mean "skip this block".
 * Calls on one context that overlap on different streams race on the pool cursor; serialise them.
 * A context belongs to the device that was current in kvc_create; calls made with another device
 * current return KVC_ERR_ARG.  A context is not thread-safe: one host thread at a time.
 * The data calls (compress, decompress, gather, prefetch, reset) launch kernels only: no allocation, no
 * memset, no synchronisation, so a stream that is being captured into a HIP graph may record them.
 * One data call handles at most 2^26 - 4 pages (blocks * pages_per_block; 256 GiB of 4 KB pages: the
 * largest launch of 256-thread workgroups, one wave per page, that stays below 2^32 threads); more is
 * KVC_ERR_ARG.
 */
#ifndef KVC_H
#define KVC_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define KVC_OK 0
#define KVC_ERR_ARG (-1)          /* bad argument (null pointer, size out of range) */
#define KVC_ERR_NOT_BOUND (-2)    /* kvc_bind_pool has not been called */
#define KVC_ERR_HIP (-3)          /* a HIP runtime call failed */
#define KVC_ERR_POOL_FULL (-4)    /* reported by kvc_stats: at least one page did not fit */
#define KVC_ERR_CORRUPT (-5)      /* reported by kvc_stats: bad descriptor, payload or index */
#define KVC_ERR_UNSUPPORTED (-6)  /* geometry the kernels are not built for */
#define KVC_ERR_TOO_LARGE (-7)    /* the call exceeds the library's static workspace */

#define KVC_MODE_RAW 0
#define KVC_MODE_INT8 1
#define KVC_MODE_DELTA 2
#define KVC_MODE_RLE 3
#define KVC_MODE_PACK 4 /* extension beyond Algorithm 2: as 3 without the delta step (u = zigzag(q)) */
/* Extension beyond Algorithm 2, for 16-token pages: the packets of mode 4 over groups that hold one
 * pair of neighbouring channels across the 16 tokens, so that each pair packs at its own width.
 * With o = c / 8 the channel's octet, j = (c / 2) mod 4 its pair inside the octet and W = min(16, d / 8),
 * element (t, c) goes to group ((o div W) * 4 + j) * W + o mod W, position
 * (t mod 4) * 8 + (t div 4) * 2 + c mod 2.  Compress produces it, and decompress reads it, for
 * tokens_per_block = 16 and head_dim 64, 128 or 256 only. */
#define KVC_MODE_CHAN 5
#define KVC_MODE_INVALID 0xFF

#define KVC_ST_POOL_FULL 1u  /* a page did not fit into the pool */
#define KVC_ST_CORRUPT 2u    /* descriptor/payload failed validation on decode */
#define KVC_ST_BAD_INDEX 4u  /* a block id or table entry pointed outside its buffer */

typedef struct kvc_ctx kvc_ctx; /* opaque host object */

/* Page descriptor, 16 bytes, little-endian.  The paper's output <s, D_RLE> (Algorithm 2) is
 * {scale, payload at off}. */
typedef struct {
    uint64_t off;  /* byte offset of the payload in the pool, multiple of 16 */
    float scale;   /* s; 0 for RAW and all-zero pages */
    uint16_t n16;  /* payload bytes / 16, padding included */
    uint8_t mode;  /* KVC_MODE_* */
    uint8_t rsvd;  /* 0 */
} kvc_desc;

typedef struct {
    int32_t tokens_per_block; /* N >= 1 */
    int32_t head_dim;         /* d: a multiple of 32, 32..256;  N*d <= 4096 */
    int32_t pages_per_block;  /* ppb >= 1 */
    int32_t scheme;           /* mode requested from compress: 0..5 (5: N = 16, d = 64, 128 or 256 only, else KVC_ERR_UNSUPPORTED) */
} kvc_config;

typedef struct {
    uint64_t pool_bytes_used; /* bytes handed out by the pool cursor (capped at the pool size) */
    uint64_t pages[6];        /* bound descriptors per mode 0..5 */
    uint64_t pages_invalid;   /* bound descriptors with mode 0xFF (never written, or did not fit) */
    uint64_t payload_bytes;   /* sum of n16*16 over descriptors of mode 0..5 */
    uint32_t status;          /* OR of KVC_ST_* since the last kvc_reset_pool */
    uint32_t rsvd;
} kvc_stats_t;

/* Create / destroy a context.  kvc_create allocates the device state block on the current device. */
int kvc_create(kvc_ctx** out, const kvc_config* cfg);
void kvc_destroy(kvc_ctx* ctx);

/* Change the mode compress requests (0..5, with the geometry limit of mode 5); takes effect for later calls. */
int kvc_set_scheme(kvc_ctx* ctx, int32_t scheme);

/* Layout of the FP16 cache buffers read by compress and written by decompress / gather / prefetch,
 * in FP16 elements: element (token j, channel i) of page p of block b is at
 * b*block_stride + p*page_stride + j*row_stride + i.  Default (and all three = 0): contiguous pages,
 * row_stride = d, page_stride = N*d, block_stride = ppb*N*d.  Example: a [block][token][head][d] cache has
 * row_stride = H*d, page_stride = d, block_stride = N*H*d.  Strides are multiples of 8 (128-bit
 * accesses), row_stride >= d.  n_cache_blocks / n_out_blocks then count blocks of block_stride
 * elements; the caller guarantees the buffer covers the last block's last row. */
int kvc_set_cache_layout(kvc_ctx* ctx, int64_t block_stride, int64_t page_stride, int64_t row_stride);

/* Attach the compressed pool (pool_bytes, 16-byte aligned, any multiple of 16) and the descriptor
 * table (n_desc_pages entries; page p of pool block b is entry b*ppb + p).  Both caller-owned.
 * Either may also be pinned, device-mapped host memory (hipHostMalloc): the pool then sits behind
 * the host link, the closest single-GPU analogue of the paper's remote tier.  Pageable host
 * pointers are refused with KVC_ERR_ARG. */
int kvc_bind_pool(kvc_ctx* ctx, void* d_pool, uint64_t pool_bytes, kvc_desc* d_desc, uint64_t n_desc_pages);

/* Cursor = 0, status = 0, every descriptor = INVALID.  Enqueues fill kernels only. */
int kvc_reset_pool(kvc_ctx* ctx, void* stream);

/* Resume on a pool that was filled earlier: the cursor continues at used_bytes (a multiple of 16, at most
 * the pool size; the value kvc_stats reported as pool_bytes_used when the pool was saved), the status is
 * cleared, the descriptors are left as they are.  A pool, its descriptor table and that one number are a
 * complete checkpoint of the compressed tier: copy them back into buffers of the same sizes, bind them to
 * a context of the same geometry, call this, and compress, decompress and gather go on as before.
 * Enqueues one small kernel. */
int kvc_restore_pool(kvc_ctx* ctx, uint64_t used_bytes, void* stream);

/* Algorithm 2 over n blocks.  Block i is read from cache block src[i] (NULL: i) and stored as pool
 * block pool[i] (NULL: i).  d_cache: FP16 [n_cache_blocks][ppb][N][d].  Space comes from a bump
 * cursor; placement order inside the pool is unspecified, descriptors say where each page is.
 * Re-compressing into an occupied pool block leaks its old span until kvc_reset_pool. */
int kvc_compress_blocks(kvc_ctx* ctx, const void* d_cache, int64_t n_cache_blocks, const int32_t* d_src_block_ids,
                        const int32_t* d_pool_block_ids, int32_t n, void* stream);

/* As kvc_compress_blocks, with the requested mode given per block: d_block_scheme[i] in 0..5 where the
 * geometry has mode 5 (N = 16, d = 64, 128 or 256), else 0..4; higher values are read as the highest.
 * It applies to block i of the call.  This is the mechanism behind the paper's
 * layer-wise algorithm selection (Sections 3.1 (vi) and 3.6.3); the selection policy is the caller's. */
int kvc_compress_blocks_mixed(kvc_ctx* ctx, const void* d_cache, int64_t n_cache_blocks, const int32_t* d_src_block_ids,
                              const int32_t* d_pool_block_ids, const uint8_t* d_block_scheme, int32_t n, void* stream);

/* Inverse (Section 3.5.3) over n blocks: pool block pool[i] (NULL: i) is decoded into output block
 * dst[i] (NULL: i) of d_cache_out, FP16 [n_out_blocks][ppb][N][d]. */
int kvc_decompress_blocks(kvc_ctx* ctx, void* d_cache_out, int64_t n_out_blocks, const int32_t* d_pool_block_ids,
                          const int32_t* d_dst_block_ids, int32_t n, void* stream);

/* Prefetch fetch of Algorithm 1: for every layer l, sequence s and j < k, logical block
 * pred[s][j] is translated through block_table[s][.] to a pool block of that layer
 * (l*pool_blocks_per_layer + entry) and decoded into output block (l*n_seq + s)*k + j of d_out,
 * FP16 [n_layers*n_seq*k][ppb][N][d].  d_block_table: int32 [n_seq][max_blocks]; d_pred: int32
 * [n_seq][k].  pred < 0 or a table entry < 0 skips the block; values beyond their range set
 * KVC_ST_BAD_INDEX and zero-fill the block. */
int kvc_gather_decompress(kvc_ctx* ctx, void* d_out, const int32_t* d_block_table, int32_t max_blocks,
                          const int32_t* d_pred, int32_t n_seq, int32_t k, int32_t n_layers,
                          int64_t pool_blocks_per_layer, void* stream);

/* Speculative prefetch of Algorithm 1 into a double-buffered L2 prefetch buffer (Section 3.3.1), for
 * layers [layer_begin, layer_end) of one decode step; the token predictor is outside (d_pred is given).
 *   d_l2    FP16 [2][n_layers*n_seq*k][ppb][N][d]: two halves; this call fills half `fill_half`, the
 *           other half is what the previous step filled (and what attention may be reading).  Under
 *           kvc_set_cache_layout a slot is a block of that layout: slot i of half h starts at element
 *           (h*n_layers*n_seq*k + i) * block_stride.
 *   d_tags  int32 [2][n_layers*n_seq*k]: pool block held by every slot, -1 = empty (kvc_prefetch_reset).
 *   d_fetch int32 [n_layers*n_seq*k], out: pool block decoded into slot (l,s,j) by this call, or -1.
 *   d_loc   int32 [n_layers*n_seq*k], out: where the consumer finds predicted block (l,s,j):
 *           half*n_slots + slot (>= 0), -2 = resident in the GPU-local cache (logical block >=
 *           d_l1_first_block[s]; pass NULL for no L1), -1 = no block (pred < 0, table entry < 0, or an
 *           index out of range, which also sets KVC_ST_BAD_INDEX).
 * For every (layer, sequence) the k predictions are taken in order: translate through the block
 * table; if the pool block is in L1, in any slot of the other half, in a slot of this half already
 * settled in this step, or already in its own slot j, nothing is fetched (the residency test
 * "A_phys not in L1 u L2"); otherwise slot j of this half is claimed and the block decoded into it.
 * Stale slots are never cleared, only overwritten (lazy invalidation, Section 3.4.3).
 * k <= 32.  Calls for disjoint layer ranges may run on different streams (layer l+1, l+2 prefetch while layer l
 * computes, Section 3.4.4); calls for the same layers must be ordered. */
/* Slot policy of kvc_prefetch_layers.  0 (default): as described above, prediction j uses slot j
 * (Algorithm 1's L2[i]).  1: slot reuse -- a block wanted by this step that already sits in ANY slot of
 * either half stays there, and a block in neither half is decoded into the lowest slot of the half being
 * filled whose content this step does not want; d_fetch is then indexed by destination slot.  A window
 * sliding over consecutive blocks then transfers one block per new block instead of k. */
int kvc_set_prefetch_policy(kvc_ctx* ctx, int32_t policy);
int kvc_prefetch_reset(kvc_ctx* ctx, int32_t* d_tags, int32_t n_seq, int32_t k, int32_t n_layers, void* stream);
int kvc_prefetch_layers(kvc_ctx* ctx, void* d_l2, int32_t* d_tags, int32_t* d_fetch, int32_t* d_loc,
                        const int32_t* d_block_table, int32_t max_blocks, const int32_t* d_pred,
                        const int32_t* d_l1_first_block, int32_t n_seq, int32_t k, int32_t n_layers, int32_t layer_begin,
                        int32_t layer_end, int64_t pool_blocks_per_layer, int32_t fill_half, void* stream);

/* kvc_prefetch_layers with Algorithm 1's outstanding-request window (WaitCompletion over at most
 * Omega_max concurrent transfers; Section 3.4.2 gives the paper's controller a window of 16): the
 * transfers the planner issues are queued in issue order (layer, sequence, slot) and carried out by at
 * most `omega` transfer engines (workgroups), each holding one block in flight and taking the next queue
 * entry when its block is complete.  omega >= 1; a small omega leaves most of the GPU to the computation
 * the prefetch hides behind, a large one approaches kvc_prefetch_layers.  Plan arrays (tags, fetch, loc)
 * and buffer contents are those of kvc_prefetch_layers.
 *   d_notify  int64 [n_layers + 4], device, out.  Entry l (layers of the call only): 0 while transfers
 *             of layer l are outstanding, then the device's wall clock (hipDeviceAttributeWallClockRate
 *             ticks, never 0) at which its last transfer completed -- the ready notification a consumer
 *             may poll or wait for; a layer that needed no transfer is stamped when the window opens.
 *             [n_layers] = clock when the window opened, [n_layers+1] = transfers issued by the call,
 *             [n_layers+2] = transfer engines the call put to work: at most omega, at most one per transfer
 *             issued, at most what the GPU holds at once (1,024 to 2,048 on MI355X, by page shape), and
 *             beyond 256 only while each engine has at least eight transfers; no more blocks than that are
 *             ever in flight,
 *             [n_layers+3] = 0 until every transfer of the call has completed, then that clock value.
 *   d_work    device workspace of at least kvc_prefetch_window_workspace(n_blocks, n_layers_call) bytes,
 *             256-byte aligned, n_blocks = (layer_end - layer_begin) * n_seq * k, n_layers_call =
 *             layer_end - layer_begin; caller-owned, contents meaningless between calls.  Calls that
 *             overlap in time need workspaces and notify arrays of their own.
 * A call over no slots (layer_begin = layer_end, n_seq = 0 or k = 0) does nothing. */
uint64_t kvc_prefetch_window_workspace(int64_t n_blocks, int32_t n_layers_call);
/* Rate of the clock the d_notify stamps count, in kHz, on the current device (KVC_ERR_HIP if the query fails). */
int kvc_wall_clock_khz(int32_t* khz);
int kvc_prefetch_layers_window(kvc_ctx* ctx, void* d_l2, int32_t* d_tags, int32_t* d_fetch, int32_t* d_loc,
                               const int32_t* d_block_table, int32_t max_blocks, const int32_t* d_pred,
                               const int32_t* d_l1_first_block, int32_t n_seq, int32_t k, int32_t n_layers,
                               int32_t layer_begin, int32_t layer_end, int64_t pool_blocks_per_layer, int32_t fill_half,
                               int32_t omega, int64_t* d_notify, void* d_work, uint64_t work_bytes, void* stream);

/* kvc_prefetch_layers_window for callers that cannot allocate and have no workspace to pass: code under
 * HIP graph capture, tight serving loops, harnesses that forbid allocation.  The window's queue lives in
 * a static device array inside the library (about 260 KB per GPU, held from library load until the
 * process ends), so one call covers at most 65,536 slots ((layer_end - layer_begin) * n_seq * k) and at
 * most 1,024 layers; more returns KVC_ERR_TOO_LARGE and enqueues nothing.  The call itself allocates and
 * frees nothing and only launches kernels (the array is cleared by them, not by a memset).  Results are
 * those of kvc_prefetch_layers_window.  Every call on one GPU, from any context, shares the one array:
 * calls that overlap in time on a GPU (different streams, or different contexts) race on it; order them. */
int kvc_prefetch_layers_window_static(kvc_ctx* ctx, void* d_l2, int32_t* d_tags, int32_t* d_fetch, int32_t* d_loc,
                                      const int32_t* d_block_table, int32_t max_blocks, const int32_t* d_pred,
                                      const int32_t* d_l1_first_block, int32_t n_seq, int32_t k, int32_t n_layers,
                                      int32_t layer_begin, int32_t layer_end, int64_t pool_blocks_per_layer,
                                      int32_t fill_half, int32_t omega, int64_t* d_notify, void* stream);

/* Reduce the descriptor table and read the device state.  The only call that synchronises
 * (on `stream`).  Returns KVC_ERR_POOL_FULL / KVC_ERR_CORRUPT if the matching status bit is set
 * (out is filled either way), else 0. */
int kvc_stats(kvc_ctx* ctx, kvc_stats_t* out, void* stream);

const char* kvc_strerror(int code);

/* ---- Verification and measurement hooks -------------------------------------------------------
 * The calls below are not steps of the codec path and no codec call depends on them.  They exist so
 * that a test can check the encoder's scale arithmetic exhaustively, so that a benchmark can time a
 * plain copy with the codec's access shape on the same device, through the same library, and so that it
 * can record the clocks the runtime reports beside the bandwidth it measures. */

/* Shader clock, memory clock (both kHz) and memory bus width (bits) of the current device, as
 * hipDeviceGetAttribute reports them; any pointer may be NULL.  KVC_ERR_HIP if a query fails. */
int kvc_device_clocks(int32_t* shader_khz, int32_t* memory_khz, int32_t* memory_bus_bits);

/* The scaling step of Algorithm 2 on its own: for n page maxima given as FP16 bit patterns (sign
 * ignored) write s = amax / 127 and s_inv = 1 / s as the encoder computes them (binary32); 0, Inf
 * and NaN give 0 for both.  All three arrays are device memory.  The encoder does not use IEEE
 * division instructions for these quotients; this call lets a test compare its arithmetic with
 * plain division for every possible maximum. */
int kvc_page_scales(const uint16_t* d_amax, float* d_scale, float* d_scale_inv, uint64_t n, void* stream);

/* dst[0..nbytes) = src[0..nbytes), a wavefront per contiguous 4 KB with 128-bit loads and stores;
 * nbytes a multiple of 16 and at most 2^38 - 4096 (else KVC_ERR_ARG); both pointers device memory, 16-byte
 * aligned, not overlapping.  The bandwidth yardstick the codec kernels are compared with. */
int kvc_copy_bytes(void* d_dst, const void* d_src, uint64_t nbytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* KVC_H */
