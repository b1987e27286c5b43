/*
 * kvc.h -- C ABI of the MI355X (gfx950) KV-cache compress / decompress library.
 *
 * The library implements the quantizer Q and codec C stages of the KVServe compression
 * pipeline BS = C(Q(T(X))) (paper section 5.1) and their inverses, as they run at the
 * two ends of a KV movement (section 4: Prefill -> Compression -> Communication ->
 * Decompression -> Decode).  A *strategy* (section 5.1: the choice of modules and their
 * parameters) is fixed for a whole request (section 3.1) and applied to that request's
 * K and V tensors; the result is one self-contained payload whose byte size V_p defines
 * the compression ratio cr = V / V_p (section 3.1).
 *
 * Conventions, for every entry point:
 *  - plain C types only; pointers are HOST pointers unless the comment says DEVICE;
 *  - the caller owns every buffer; the library allocates no device memory and, apart from
 *    launching kernels on the caller's stream, performs no device synchronisation (the one
 *    host-to-device copy of the library is in kvc_workspace_init);
 *  - all device pointers must be 16-byte aligned; strides are in elements (2 bytes);
 *  - errors the host can see are returned (negative kvc_status) before anything is
 *    launched; errors only the device can see (bad block-table entry, corrupt payload)
 *    are written to the caller's status words and never cause out-of-bounds accesses;
 *  - head_dim must be 128 (the kernels map 16 lanes x 8 channels onto one token row);
 *  - layers * kv_heads <= 2^20 and tokens <= 2^32, so that no byte count comes near 2^63;
 *  - inputs must be finite; +0 and -0 are both reconstructed as +0.
 */
#ifndef KVC_H
#define KVC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    KVC_OK = 0,
    KVC_ERR_ARG = -1,          /* null pointer, misalignment, non-positive size, bad enum    */
    KVC_ERR_UNSUPPORTED = -2,  /* valid in the format but not built (head_dim != 128, ...)   */
    KVC_ERR_CAPACITY = -3,     /* payload / workspace / plan limit too small                 */
    KVC_ERR_FORMAT = -4,       /* payload header is not a KVC1 header or is inconsistent      */
    KVC_ERR_MISMATCH = -5,     /* payload does not belong to this plan                        */
    KVC_ERR_DEVICE = -6        /* a HIP call failed                                           */
} kvc_status;

/* device-side status bits (OR-ed into the caller's int32 status word of a request) */
enum {
    KVC_DEV_BAD_BLOCK = 1,     /* block-table entry outside [0, num_phys_blocks)              */
    KVC_DEV_BAD_HEADER = 2,    /* payload header does not match the plan / request            */
    KVC_DEV_BAD_CHUNK = 4,     /* coder directory or chunk body inconsistent                  */
    KVC_DEV_BAD_TABLE = 8,     /* code-length table is not a complete prefix code             */
    KVC_DEV_SCAN_TIMEOUT = 16  /* internal: chunk-offset scan gave up waiting                 */
};

enum { KVC_F16 = 1, KVC_BF16 = 2 };
enum { KVC_CODEC_NONE = 0, KVC_CODEC_HUFF8 = 1 };

/*
 * The knobs a controller selects (section 5.1, "Quantizer": bit width, granularity and
 * mixed precision; "Codec"; section 7.1: KIVI = asymmetric 2-bit).
 *   bits_k / bits_v : 2, 3, 4, 8, or 16 (16 = the tensor travels unchanged: the bypass case)
 *   group_k         : tokens per K group (K is quantized per channel): 32, 64 or 128
 *   group_v         : channels per V group (V is quantized per token): 32, 64 or 128
 *   codec           : lossless stage over the packed code bytes (needs bits < 16)
 *   transform       : stage T (section 5.1, the Hadamard rotation listed among the transformer
 *                     modules): 0 none, KVC_T_HADAMARD = every head_dim-long row of K and of V
 *                     is replaced by H x / 8 before the quantizer and decompression applies
 *                     H x / 16 to the reconstructed row (H = Walsh-Hadamard matrix of order 128
 *                     in natural order; fp32 butterflies with strides 1, 2, ..., 64; results
 *                     rounded to the tensor type); KVC_T_DELTA = the difference from an anchor
 *                     token (named in section 5.1 with a reference to CacheGen): the tokens of a
 *                     head form runs of anchor_period tokens, the first token of a run is its
 *                     anchor and travels unchanged (16 bits per element) in the payload's
 *                     auxiliary section, after the coder's tables or the width tables, K anchors
 *                     then V anchors; every row is quantized as row - anchor row of its run and
 *                     decompression returns reconstructed difference + anchor (an anchor row is
 *                     its stored copy); a difference or sum is the exact value rounded once to
 *                     the tensor type and limited to its finite range.  A tensor stored unchanged
 *                     (16 bits) is not transformed by either
 *   anchor_period   : KVC_T_DELTA only: 8, 16, 32, 64 or 128 tokens; 0 otherwise
 *   head_bits_k/v   : optional per-head bit widths (section 5.1: mixed precision at head
 *                     granularity; the mechanism behind MixHQ, which keeps the heads that matter
 *                     at a high precision and gives the others very few bits).  HOST arrays of
 *                     layers * kv_heads bytes, index layer * kv_heads + head, values 2, 3, 4 or
 *                     8; NULL = one width for the whole tensor.  A tensor with a table has
 *                     bits_k (bits_v) = 0.  kvc_plan copies the tables.  The codes of the heads
 *                     follow each other in (layer, head) order, each with its own width; the
 *                     tables travel in the payload's auxiliary section (K table, then V table).
 *                     Which head gets which width is the caller's choice.  With a codec the chunks
 *                     of a tensor are ordered by width (2, 3, 4, 8), then by (layer, head, chunk),
 *                     and every width has its own code table (docs/FORMAT.md).
 *                     A plan with tables needs a workspace (kvc_workspace_size) that has been
 *                     through kvc_workspace_init.
 * Every group carries two fp16 values (scale, zero): the 32 bits per group that cap
 * 2-bit / group-32 at 16/(2+1) = 5.33x (section 7.3).
 */
#define KVC_T_NONE 0
#define KVC_T_HADAMARD 1
#define KVC_T_DELTA 2

typedef struct {
    uint8_t bits_k, bits_v;
    uint16_t group_k, group_v;
    uint8_t codec, transform;
    uint16_t anchor_period;
    const uint8_t *head_bits_k, *head_bits_v;
} kvc_strategy;

typedef struct {
    uint8_t dtype;                       /* KVC_F16 or KVC_BF16 (input and output type)      */
    int32_t layers, kv_heads, head_dim;
} kvc_model;

/*
 * One request's KV in device memory.  Element (l, h, t, d) of K lives at
 *   k + l*stride_layer + h*stride_head + tok(t) + d
 *   tok(t) = t*stride_token                                         when block_table == NULL
 *          = block_table[t / block_tokens]*stride_block
 *            + (t % block_tokens)*stride_token                      otherwise (paged)
 * and likewise for V from v.  A contiguous [layer][kv][head][token][dim] cache is
 *   v = k + heads*tokens*dim, stride_layer = 2*heads*tokens*dim, stride_head = tokens*dim,
 *   stride_token = dim;
 * a vLLM-style pool [layer][kv][phys_block][block_tokens][head][dim] is
 *   stride_head = dim, stride_token = heads*dim, stride_block = block_tokens*heads*dim.
 * block_table (DEVICE, ceil(tokens/block_tokens) int32 entries) is shared by all layers;
 * block_tokens must be a power of two.  For kvc_decompress the same struct names the
 * destination (k, v are written), which may use a different block table than the sender.
 */
typedef struct {
    void *k, *v;                         /* DEVICE */
    int64_t tokens;
    int64_t stride_layer, stride_head, stride_token, stride_block;
    const int32_t *block_table;          /* DEVICE or NULL */
    int32_t block_tokens, num_phys_blocks;
} kvc_request;

typedef struct kvc_plan_s kvc_plan_t;      /* opaque, host memory */

/*
 * A plan is one profile in the sense of section 3.1: the strategy chosen for a request when its
 * KV movement begins and held for the whole request, together with the model shape it applies to.
 * Validates the (model, strategy) pair and fixes the limits the workspace is sized for
 * (max_tokens per request, max_batch requests per call).  Returns KVC_OK and a plan in *out
 * (host memory, release with kvc_plan_free), KVC_ERR_ARG for a value outside the format,
 * KVC_ERR_UNSUPPORTED for one the format has and this build does not run; *out = NULL on error.
 * Touches no device.  The plan copies the width tables; a plan may be used by one thread at a time.
 */
int kvc_plan(const kvc_model *model, const kvc_strategy *strategy, int64_t max_tokens,
             int32_t max_batch, kvc_plan_t **out);
void kvc_plan_free(kvc_plan_t *plan);

/*
 * Payload bytes of a request of `tokens` tokens: V_p of section 3.1.  Without the codec
 * the value is exact (*is_exact = 1):
 *   128 + a16(4*L*H*ceil(T/group_k)*D) + a16(4*L*H*T*D/group_v)
 *       + a16(L*H*T*D*bits_k/8) + a16(L*H*T*D*bits_v/8),      a16 = round up to 16
 * (plus the auxiliary section: L*H bytes per width table, and with KVC_T_DELTA
 * 2*L*H*ceil(T/anchor_period)*D bytes of anchor rows per transformed tensor);
 * with it, the value is the capacity the caller must provide (every chunk stored raw,
 * plus tables and directory) and the true size is reported by kvc_compress.
 */
int kvc_payload_size(const kvc_plan_t *plan, int64_t tokens, uint64_t *bytes, int *is_exact);

/* Bytes of DEVICE scratch kvc_compress / kvc_decompress need (may be 0). */
size_t kvc_workspace_size(const kvc_plan_t *plan);

/*
 * Plans with per-head width tables (section 5.1, head-wise mixed precision) keep a device image
 * of the tables in the first kvc_table_bytes(plan) bytes of the workspace.  kvc_workspace_init
 * writes it: one copy from pageable HOST memory on `hip_stream`, which may block the host until
 * the copy is staged and cannot be captured into a graph.  Call it once per (plan, workspace)
 * before the first kvc_compress / kvc_decompress, and again only if something else has written
 * those bytes; the calls themselves leave them alone.  For plans without tables both functions
 * do nothing (0 bytes).  Returns KVC_OK, KVC_ERR_ARG (null or misaligned workspace) or
 * KVC_ERR_DEVICE.
 */
size_t kvc_table_bytes(const kvc_plan_t *plan);
int kvc_workspace_init(const kvc_plan_t *plan, void *workspace, void *hip_stream);

/*
 * Compress n requests (n <= max_batch, each tokens <= max_tokens) with the plan's strategy.
 *   payload      DEVICE buffer; request i's payload starts at payload + payload_off[i]
 *   payload_off  HOST, n+1 ascending multiples of 16; payload_off[i+1]-payload_off[i] must
 *                be >= kvc_payload_size(tokens_i)
 *   out_bytes    DEVICE, n x uint64: the true payload size of each request
 *   dev_status   DEVICE, n x int32: KVC_DEV_* bits (zeroed by the call, then OR-ed)
 *   workspace    DEVICE, kvc_workspace_size bytes (may be NULL when that is 0)
 *   hip_stream   hipStream_t the kernels are enqueued on (NULL = default stream)
 * Each payload is independent of the others in the batch (the profile is fixed per
 * request, section 3.1) and identical to compressing that request alone.
 */
int kvc_compress(const kvc_plan_t *plan, const kvc_request *reqs, int32_t n, void *payload,
                 const uint64_t *payload_off, uint64_t *out_bytes, int32_t *dev_status,
                 void *workspace, void *hip_stream);

/*
 * kvc_compress for callers that cannot allocate device memory and have no workspace to hand in:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments and results as kvc_compress, without the workspace: the coder's scratch (histograms,
 * code tables, work-order counter, chunk-offset scan state) lives in a static device array of
 * KVC_STATIC_WORKSPACE_BYTES inside the library, one copy per GPU, held until the process ends.
 * The call allocates nothing and clears what must start from zero itself.
 *   - the stream must belong to the current device;
 *   - plans whose kvc_workspace_size exceeds KVC_STATIC_WORKSPACE_BYTES are refused with
 *     KVC_ERR_CAPACITY (4 MiB covers the lossless stage up to layers * kv_heads *
 *     ceil(max_tokens / 128) * max_batch = 250,000 chunks per tensor, e.g. 80 x 8 x 32768 x 1);
 *   - plans with per-head width tables are refused with KVC_ERR_UNSUPPORTED (their tables live
 *     in a caller workspace);
 *   - all calls on one GPU share the array: two calls that overlap in time on one GPU (different
 *     streams or threads) race; calls in stream order on one stream do not.
 */
#define KVC_STATIC_WORKSPACE_BYTES (4u << 20)
int kvc_compress_static(const kvc_plan_t *plan, const kvc_request *reqs, int32_t n, void *payload,
                        const uint64_t *payload_off, uint64_t *out_bytes, int32_t *dev_status,
                        void *hip_stream);

/*
 * The decompression stage at the receiving end of a KV movement (section 4: ... Communication ->
 * Decompression -> Decode), the inverse of BS = C(Q(T(X))) (section 5.1): rebuild K and V of n
 * requests into dst[i] (DEVICE; the layout, contiguous or paged, may differ from the sender's).
 *   payload / payload_off   as for kvc_compress; payload_off[i+1]-payload_off[i] must cover the
 *                           payload (without the codec: kvc_payload_size; with it: at least the
 *                           part before the code sections; the device checks the rest)
 *   dst[i].tokens           must equal the payload's token count
 *   dev_status, workspace, hip_stream   as for kvc_compress
 * The device checks each header (and width table) against the plan and sets KVC_DEV_BAD_HEADER,
 * writing nothing for that request, on a mismatch; a damaged table, directory or chunk sets
 * KVC_DEV_BAD_TABLE / KVC_DEV_BAD_CHUNK and the affected chunks are not written.  Host-visible
 * errors (KVC_ERR_ARG, KVC_ERR_CAPACITY) are returned before anything is launched.
 * Reconstruction: x^ = round(code*scale + zero) in the model dtype, then the inverse of stage T.
 */
int kvc_decompress(const kvc_plan_t *plan, const void *payload, const uint64_t *payload_off,
                   const kvc_request *dst, int32_t n, int32_t *dev_status, void *workspace,
                   void *hip_stream);

/*
 * The bitstream BS of section 5.1 describes itself: decode a 128-byte payload header held in
 * HOST memory into the model shape and strategy that produced it.  sections[10] receives five
 * (offset, bytes) pairs: K meta, V meta, coder tables+directory, K codes, V codes.
 * Any output pointer may be NULL.  Returns KVC_ERR_FORMAT for a bad magic, version or
 * field combination.
 */
int kvc_payload_inspect(const void *header128, kvc_model *model, kvc_strategy *strategy,
                        int64_t *tokens, uint64_t *total_bytes, uint64_t *sections);

/* Host-side check of a block table held in HOST memory (every entry in range). */
int kvc_check_block_table(const int32_t *table, int64_t entries, int32_t num_phys_blocks);

/*
 * Measurement hook, for benchmarks only.  While an array of `capacity` hipEvent_t handles (HOST
 * array, owned by the caller) is installed in a plan, every kvc_compress / kvc_decompress with
 * that plan records, per request and on the call's stream, four events: before the set-up work
 * (for the first request of a call: before anything the call enqueues), before the K pass,
 * between the K and V passes, and after the V pass (short requests of one call share their launches
 * and then share these moments).  Returns the number of events recorded since the previous call;
 * NULL uninstalls.  The state lives in the plan.
 */
int kvc_trace(kvc_plan_t *plan, void **hip_events, int32_t capacity);

/*
 * Measurement aid, for benchmarks only: moves bytes in the access shape of a tensor pass with no
 * arithmetic, so that a benchmark can put what the memory system gives to this pattern
 * beside the published HBM peak (the path is bound by HBM bandwidth: every element is read once
 * and written once in the other form, sections 3.1 and 5.1 give the two directions).
 *   mode 0  the compress direction: one wave per 128 token rows reads 128 x 256 bytes from `src`
 *           (four serial passes of 32 rows, 16 bytes per lane and access) and writes
 *           128 x payload_row_bytes to `dst`
 *   mode 1  the decompress direction: the same with the two sides exchanged
 *   rows               token rows of 256 bytes (a multiple of 128)
 *   payload_row_bytes  bytes per row on the payload side: a multiple of 16 in [16, 256]
 * `src` and `dst` are DEVICE buffers owned by the caller, 16-byte aligned, of rows x 256 and
 * rows x payload_row_bytes bytes (mode 0; exchanged for mode 1).  Enqueued on `hip_stream`.
 * Returns KVC_OK, KVC_ERR_ARG, KVC_ERR_CAPACITY (more than 2^32 chunks) or KVC_ERR_DEVICE.
 */
int kvc_stream_probe(int mode, const void *src, void *dst, int64_t rows, int32_t payload_row_bytes,
                     void *hip_stream);

/*
 * Device self-test of the quantizer's arithmetic shortcuts (stage Q of section 5.1 fixes the
 * results; the kernels reach them with cheaper instruction sequences).  Each count is the
 * number of inputs, over the whole domain a shortcut is used on, for which it differs from
 * the plain IEEE operation; every count must be zero.
 *   counts[0..3]  min((max - min) / (2^b - 1), 65504) for b = 2, 3, 4, 8: all floats >= 0 and +infinity
 *   counts[4]     1 / scale: all positive finite fp16 scales
 *   counts[5]     x - zero read from a packed fp16 pair: all pairs of finite fp16 values
 *   counts[6]     float -> byte with insertion: round-to-nearest-even, all floats in [0, 255]
 * `counts` is DEVICE memory, KVC_SELFTEST_COUNTS 64-bit words, 8-byte aligned, owned by the
 * caller; it is cleared and filled on `stream` (asynchronous: synchronize before reading).
 * Returns KVC_OK, KVC_ERR_ARG for a null pointer, KVC_ERR_DEVICE if a launch failed.
 */
#define KVC_SELFTEST_COUNTS 8
int kvc_selftest(uint64_t *counts, void *stream);

/*
 * Analytic selection among measured profiles (section 6.1).  Host functions, no GPU work.
 * A profile is the triple of section 3.1 as this library measures it: cr = V / V_p and the
 * encode / decode throughputs in bytes of uncompressed KV per second (any consistent unit).
 *   kvc_profile_throughput : s_p, the harmonic combination 1 / (1/s_enc + 1/s_dec)
 *   kvc_benefit_threshold  : B*_p = (1 - 1/cr_p) s_p (Eq. 5): the profile shortens the transfer
 *                            exactly when the effective bandwidth is below it (Theorem 1)
 *   kvc_policy_build       : the piecewise policy of Theorem 2, the lower envelope over
 *                            x = 1/B of cost_p(x) = 1/s_p + x/cr_p (Eq. 6) together with
 *                            cost(x) = x for an uncompressed transfer.  Writes *count segments
 *                            ordered by x_from (the first starts at 0); segment i is optimal for
 *                            x in [x_from_i, x_from_(i+1)); profile -1 = do not compress.
 *                            Profiles that are never optimal do not appear.  Returns
 *                            KVC_ERR_CAPACITY (with *count set) if the table is too small
 *                            (n + 1 entries always suffice), KVC_ERR_ARG for a profile with a
 *                            non-positive or non-finite field.
 *   kvc_policy_lookup      : O(log n) look-up for a bandwidth (same unit as the throughputs):
 *                            the optimal profile and its two neighbours on the envelope, the
 *                            candidate set the paper hands to its online stage.
 * All arrays are host memory owned by the caller.
 */
typedef struct {
    double cr, s_enc, s_dec;
} kvc_profile;

typedef struct {
    double x_from;
    int32_t profile;
} kvc_policy_segment;

double kvc_profile_throughput(const kvc_profile *p);
double kvc_benefit_threshold(const kvc_profile *p);
int kvc_policy_build(const kvc_profile *profiles, int32_t n, kvc_policy_segment *table, int32_t capacity,
                     int32_t *count);
int kvc_policy_lookup(const kvc_policy_segment *table, int32_t count, double bandwidth, int32_t *profile,
                      int32_t *toward_more_bandwidth, int32_t *toward_less_bandwidth);

const char *kvc_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif
