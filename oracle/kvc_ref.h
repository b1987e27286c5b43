/*
 * kvc_ref.h -- CPU oracle for the KV-cache compress / decompress path.
 *
 * TEST INFRASTRUCTURE ONLY.  This is a plain, slow, single-threaded restatement of
 * what the path computes; it exists so that the GPU library can be checked against
 * something that can be read against the paper by eye.  It shares no code, header,
 * table or constant with the GPU library and must never be called by it.
 *
 * What the paper fixes (KVServe, section 5.1 and section 7.3): the payload is
 * BS = C(Q(T(X))): an optional transform T, a quantizer Q, a lossless codec C.
 * Q is asymmetric (a zero point as well as a scale), fine-grained grouped with
 * per-group metadata, K grouped along tokens per channel and V along channels per
 * token, 2 or 4 bits typical, with two 16-bit metadata values per group (which is
 * what limits 2-bit / group-32 to 16/(2+32/32) = 5.33x).  Everything below that
 * level -- formula, rounding, bit order, payload layout, the entropy coder -- is
 * not given by the paper; the readings taken here are listed in the header comment
 * of each function.
 *
 * Pins (tests/test_oracle_*.py): payload-size closed form and the 5.33x limit;
 * half-step error bound and brute-force nearest level in float64; min -> code 0,
 * max -> top code; constant group exact; offset invariance (asymmetry); identity at
 * 16 bits; exhaustive pack/unpack; hand-written packed byte strings; K/V transpose
 * duality; paged == contiguous; Kraft equality, length limit, entropy bound and
 * round trip for the coder; number-format conversions against numpy; the transforms against
 * their float64 definitions (matrix product; exact difference rounded once) and against
 * transform-free payloads of tensors transformed beforehand.
 * Parity unpinned by the paper itself: the exact operation order of the quantizer
 * (two rounded fp32 operations), the tie rule, the payload byte layout and the
 * choice of entropy coder.  They are pinned only by the invariants above.
 */
#ifndef KVC_REF_H
#define KVC_REF_H

#include <stdint.h>
#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { REF_OK = 0, REF_ERR_ARG = -1, REF_ERR_UNSUPPORTED = -2, REF_ERR_CAPACITY = -3,
       REF_ERR_FORMAT = -4, REF_ERR_MISMATCH = -5 };

enum { REF_F16 = 1, REF_BF16 = 2 };

typedef struct {
    int32_t dtype;              /* REF_F16 or REF_BF16 */
    int32_t layers, heads, head_dim;
    int32_t bits_k, bits_v;     /* 2, 3, 4, 8, or 16 (= stored unchanged) */
    int32_t group_k;            /* tokens per K group (one group per channel) */
    int32_t group_v;            /* channels per V group (one group per token) */
    int32_t codec;              /* 0 none, 1 huff8 */
    int32_t transform;          /* 0 none, 1 Walsh-Hadamard over head_dim (ref_hadamard_row),
                                   2 delta against an anchor token (ref_delta_row) */
    int32_t anchor_period;      /* transform 2: tokens per run, a power of two in 8..128; else 0 */
    /* optional per-head bit widths, index l*heads + h, values 2, 3, 4 or 8; when a table is
     * given the uniform width of that tensor (bits_k / bits_v) must be 0.  With codec 1 the chunks
     * are ordered by width and every width has its own code table (see kvc_ref.c). */
    const uint8_t *head_bits_k, *head_bits_v;
} ref_config;

/* Element index of x[l][h][t][0] (channel stride is 1):
 *   l*stride_layer + h*stride_head + tok(t)
 *   tok(t) = t*stride_token                                         if block_tokens == 0
 *          = table[t / block_tokens]*stride_block
 *            + (t % block_tokens)*stride_token                      otherwise            */
typedef struct {
    int64_t stride_layer, stride_head, stride_token, stride_block;
    int32_t block_tokens;
    const int32_t *block_table;
} ref_layout;

/* number formats */
float    ref_f16_to_f32(uint16_t h);
uint16_t ref_f32_to_f16(float f);
float    ref_bf16_to_f32(uint16_t h);
uint16_t ref_f32_to_bf16(float f);

/* transform T: one head_dim-long row of 16-bit values -> the same, see kvc_ref.c */
void     ref_hadamard_row(const uint16_t *in, uint16_t *out, int dim, int dtype, int inverse);
void     ref_delta_row(const uint16_t *x, const uint16_t *anchor, uint16_t *out, int dim, int dtype,
                       int inverse);

/* quantizer on one group held as floats */
void     ref_group_meta(const float *x, int n, int bits, uint16_t *scale_h, uint16_t *zero_h);
void     ref_group_quantize(const float *x, int n, int bits, uint16_t scale_h, uint16_t zero_h,
                            uint8_t *q);
uint16_t ref_dequantize(int q, uint16_t scale_h, uint16_t zero_h, int dtype);

/* bit packing of n codes of `bits` bits; n*bits must be a multiple of 8 */
void ref_pack(const uint8_t *q, int64_t n, int bits, uint8_t *out);
void ref_unpack(const uint8_t *in, int64_t n, int bits, uint8_t *q);

/* entropy coder pieces */
void    ref_huff_lengths(const uint32_t hist[256], uint8_t len[256]);
void    ref_huff_codes(const uint8_t len[256], uint16_t code[256]);
int64_t ref_huff_encode_chunk(const uint8_t *raw, int rows, int row_bytes, const uint8_t len[256],
                              uint8_t *body);
int     ref_huff_decode_chunk(const uint8_t *body, int64_t body_bytes, int rows, int row_bytes,
                              const uint8_t len[256], uint8_t *raw);

/* geometry */
int     ref_check_config(const ref_config *c);
int64_t ref_chunks_per_head(int64_t tokens);
int     ref_payload_size(const ref_config *c, int64_t tokens, uint64_t *bytes, int *is_exact);

/* one (layer, head) of one tensor (is_v = 0 for K, 1 for V):
 * codes: tokens * head_dim * bits / 8 packed bytes in [t][d] order
 * meta : K  [ceil(tokens/group_k)][head_dim] pairs, V [tokens][head_dim/group_v] pairs,
 *        each pair = scale (fp16 bits) then zero (fp16 bits)                             */
int ref_compress_head(const ref_config *c, int is_v, const void *src, const ref_layout *lay,
                      int64_t tokens, int l, int h, uint8_t *codes, uint16_t *meta);
/* anchors (delta transform only, else NULL): this head's anchor rows,
 * [ceil(tokens/anchor_period)][head_dim] */
int ref_decompress_head(const ref_config *c, int is_v, const uint8_t *codes, const uint16_t *meta,
                        const uint16_t *anchors, int64_t tokens, int l, int h, void *dst,
                        const ref_layout *lay);

/* code-length tables of the two sections (codec 1), from the deterministic sample */
int ref_huff_tables(const ref_config *c, const void *k, const void *v, const ref_layout *lay,
                    int64_t tokens, uint8_t len_k[256], uint8_t len_v[256]);
/* body of one chunk (index within its section), given that section's table */
int64_t ref_encode_chunk_at(const ref_config *c, int is_v, const void *src, const ref_layout *lay,
                            int64_t tokens, int64_t chunk, const uint8_t len[256], uint8_t *body);

/* whole request */
int ref_compress(const ref_config *c, const void *k, const void *v, const ref_layout *lay,
                 int64_t tokens, uint8_t *payload, uint64_t capacity, uint64_t *out_bytes);
int ref_decompress(const uint8_t *payload, uint64_t bytes, void *k, void *v,
                   const ref_layout *lay, const ref_config *expect);
int ref_inspect(const uint8_t *header, ref_config *c, int64_t *tokens, uint64_t *total_bytes,
                uint64_t sections[10]);

#ifdef __cplusplus
}
#endif
#endif
