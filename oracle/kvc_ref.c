/*
 * kvc_ref.c -- CPU oracle (test infrastructure only; see kvc_ref.h).
 *
 * Plain C, single-threaded, no blocking or fusion: each function takes the steps of
 * the method in the order the paper composes them (section 5.1: quantizer Q, then
 * codec C; the receiver inverts them).  Build with -O2 -ffp-contract=off so that
 * every fp32 operation written here is one rounded fp32 operation.
 */
#include "kvc_ref.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

#define CHUNK_ROWS 128      /* token rows of one head per coder chunk */
#define SUB_ROWS   2        /* token rows per sub-block                */
#define SUBS       64       /* sub-blocks per chunk                    */
#define MAX_LEN    12       /* longest code word                       */
#define HEADER     128

/* ------------------------------------------------------------------ formats */

static uint32_t f32_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }
static float bits_f32(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }

/* IEEE binary16 -> binary32, exact. */
float ref_f16_to_f32(uint16_t h)
{
    int sign = h >> 15, e = (h >> 10) & 31, m = h & 1023;
    double v;
    if (e == 31) v = m ? NAN : INFINITY;
    else if (e == 0) v = ldexp((double)m, -24);               /* subnormal: m * 2^-24 */
    else v = ldexp(1.0 + (double)m / 1024.0, e - 15);
    return (float)(sign ? -v : v);
}

/* binary32 -> binary16, round to nearest, ties to even; overflow gives infinity. */
uint16_t ref_f32_to_f16(float f)
{
    if (isnan(f)) return 0x7e00;
    uint16_t sign = signbit(f) ? 0x8000 : 0;
    double a = fabs((double)f);
    if (a >= 65520.0) return sign | 0x7c00;     /* 65520 is the tie between 65504 and 2^16 */
    if (a < ldexp(1.0, -14)) {
        /* subnormal range: multiples of 2^-24; a count of 1024 is the smallest normal */
        return sign | (uint16_t)nearbyint(a * 16777216.0);
    }
    int e;
    double fr = frexp(a, &e);                   /* a = fr * 2^e, fr in [0.5, 1) */
    double m = nearbyint((2.0 * fr - 1.0) * 1024.0);
    int E = e - 1 + 15;
    if (m == 1024.0) { m = 0.0; E += 1; }
    return sign | (uint16_t)(E << 10) | (uint16_t)m;
}

/* bfloat16 is the upper half of binary32. */
float ref_bf16_to_f32(uint16_t h) { return bits_f32((uint32_t)h << 16); }

uint16_t ref_f32_to_bf16(float f)
{
    if (isnan(f)) return 0x7fc0;
    uint32_t u = f32_bits(f), low = u & 0xffffu, up = u >> 16;
    if (low > 0x8000u || (low == 0x8000u && (up & 1u))) up += 1;   /* nearest, ties to even */
    return (uint16_t)up;
}

static float load_elem(const void *base, int dtype, int64_t idx)
{
    uint16_t w = ((const uint16_t *)base)[idx];
    return dtype == REF_F16 ? ref_f16_to_f32(w) : ref_bf16_to_f32(w);
}

/* ------------------------------------------------------------------ transform T
 *
 * KVServe section 5.1 lists a Hadamard rotation (QuaRot) among the transformer modules that may
 * precede the quantizer; the paper gives no formula.  Reading taken here: every head_dim-long row
 * x of K and of V becomes y = s * H x, H the Walsh-Hadamard matrix in natural (Sylvester) order,
 * H[i][j] = (-1)^popcount(i & j), and decompression applies s' * H to the reconstructed row.
 * H H = dim * I, so s * s' = 1 / dim makes the pair an identity; with dim = 2^m the factors are
 * the powers of two s = 2^-floor(m/2), s' = 2^-ceil(m/2) (1/8 and 1/16 for head_dim 128), which
 * scale without rounding.  H x is computed by the fast transform, whose operation order is part
 * of the definition because fp32 sums round: for h = 1, 2, 4, ..., dim/2, every pair (j, j + h)
 * with bit h of j clear becomes (a + b, a - b), one fp32 operation each.  The scaled result is
 * limited to the finite range of the tensor's type and rounded to it (nearest even).  A tensor
 * stored unchanged (16 bits) is not transformed, so that this setting stays lossless.
 */
void ref_hadamard_row(const uint16_t *in, uint16_t *out, int dim, int dtype, int inverse)
{
    float x[1024];
    int m = 0;
    while ((1 << m) < dim) ++m;
    for (int i = 0; i < dim; ++i) x[i] = dtype == REF_F16 ? ref_f16_to_f32(in[i]) : ref_bf16_to_f32(in[i]);
    for (int h = 1; h < dim; h <<= 1)
        for (int j = 0; j < dim; ++j)
            if (!(j & h)) {
                float a = x[j], b = x[j + h];
                x[j] = a + b;
                x[j + h] = a - b;
            }
    const float scale = 1.0f / (float)(1 << (inverse ? (m + 1) / 2 : m / 2));
    const float top = dtype == REF_F16 ? 65504.0f : 3.3895313892515355e38f;
    for (int i = 0; i < dim; ++i) {
        float y = x[i] * scale;
        if (y > top) y = top;
        if (y < -top) y = -top;
        out[i] = dtype == REF_F16 ? ref_f32_to_f16(y) : ref_f32_to_bf16(y);
    }
}

/*
 * The other transform of section 5.1 built here is the delta against an anchor token (the paper
 * names it and refers to CacheGen for it).  Reading: the tokens of a head are cut into runs of
 * `anchor_period` consecutive tokens; the first token of a run is its anchor and travels unchanged
 * (16 bits) beside the codes; every row is replaced by its difference from the anchor row of its
 * run before the quantizer (an anchor row by zeros), and decompression adds the anchor back to the
 * reconstructed difference (an anchor row is its stored copy).  A difference or sum is the exact
 * value rounded once to the tensor type, limited to the type's finite range.  fp32 arithmetic
 * followed by the rounding to 16 bits gives exactly that: the wider format has more than twice
 * the digits of the narrow one, so the first rounding cannot change the second.
 */
void ref_delta_row(const uint16_t *x, const uint16_t *anchor, uint16_t *out, int dim, int dtype,
                   int inverse)
{
    const float top = dtype == REF_F16 ? 65504.0f : 3.3895313892515355e38f;
    for (int d = 0; d < dim; ++d) {
        float a = dtype == REF_F16 ? ref_f16_to_f32(x[d]) : ref_bf16_to_f32(x[d]);
        float b = dtype == REF_F16 ? ref_f16_to_f32(anchor[d]) : ref_bf16_to_f32(anchor[d]);
        float y = inverse ? a + b : a - b;
        if (y > top) y = top;
        if (y < -top) y = -top;
        out[d] = dtype == REF_F16 ? ref_f32_to_f16(y) : ref_f32_to_bf16(y);
    }
}

static int64_t row_offset(const ref_layout *lay, int l, int h, int64_t t)
{
    int64_t o = (int64_t)l * lay->stride_layer + (int64_t)h * lay->stride_head;
    if (lay->block_tokens == 0) return o + t * lay->stride_token;
    return o + (int64_t)lay->block_table[t / lay->block_tokens] * lay->stride_block
             + (t % lay->block_tokens) * lay->stride_token;
}

/* ---------------------------------------------------------------- quantizer */

/*
 * Per-group metadata (reading; the paper states only "asymmetric" with per-group
 * metadata, section 7.1 and 7.3): affine min-max quantization.
 *   zero  = fp16(min)                       (clamped to the finite fp16 range first)
 *   scale = fp16((max - min) / (2^bits-1))  (fp32 subtract, fp32 divide, then fp16)
 * A zero of either sign counts as +0, so that the stored bits are unique.
 */
void ref_group_meta(const float *x, int n, int bits, uint16_t *scale_h, uint16_t *zero_h)
{
    float mn = x[0], mx = x[0];
    for (int i = 1; i < n; ++i) {
        if (x[i] < mn) mn = x[i];
        if (x[i] > mx) mx = x[i];
    }
    if (mn == 0.0f) mn = fabsf(mn);
    if (mx == 0.0f) mx = fabsf(mx);
    float lo = mn;
    if (lo < -65504.0f) lo = -65504.0f;
    if (lo > 65504.0f) lo = 65504.0f;
    *zero_h = ref_f32_to_f16(lo);
    float range = mx - mn;
    float qmax = (float)((1 << bits) - 1);
    float s = range / qmax;
    if (s > 65504.0f) s = 65504.0f;
    *scale_h = ref_f32_to_f16(s);
}

/*
 * Codes (reading): q = clamp(round_half_even((x - zero) * (1/scale)), 0, 2^bits-1) with the
 * stored (rounded) zero and scale, each arithmetic step one rounded fp32 operation; a zero
 * scale gives code 0 everywhere.  The paper fixes no precision for the integer decision; it is
 * taken in fp32, the precision of the two operations that produce its argument.
 */
void ref_group_quantize(const float *x, int n, int bits, uint16_t scale_h, uint16_t zero_h,
                        uint8_t *q)
{
    float z = ref_f16_to_f32(zero_h), s = ref_f16_to_f32(scale_h);
    float inv = (s == 0.0f) ? 0.0f : 1.0f / s;
    float qmax = (float)((1 << bits) - 1);
    for (int i = 0; i < n; ++i) {
        float d = x[i] - z;
        float t = d * inv;
        float r = nearbyintf(t);                /* default rounding mode: ties to even */
        if (r < 0.0f) r = 0.0f;
        if (r > qmax) r = qmax;
        q[i] = (uint8_t)r;
    }
}

/* Reconstruction: x^ = round_to_output(q * scale + zero), one fused fp32 multiply-add,
 * kept inside the finite range of the output type. */
uint16_t ref_dequantize(int q, uint16_t scale_h, uint16_t zero_h, int dtype)
{
    float y = fmaf((float)q, ref_f16_to_f32(scale_h), ref_f16_to_f32(zero_h));
    if (dtype == REF_F16) {
        if (y > 65504.0f) y = 65504.0f;
        if (y < -65504.0f) y = -65504.0f;
        return ref_f32_to_f16(y);
    }
    const float bmax = 3.3895313892515355e38f;  /* largest finite bfloat16 */
    if (y > bmax) y = bmax;
    if (y < -bmax) y = -bmax;
    return ref_f32_to_bf16(y);
}

/* ------------------------------------------------------------------ packing */

/* Element i occupies bits [i*bits, i*bits+bits) of the stream; stream bit k is bit k%8 of
 * byte k/8 (reading; the paper does not describe packing). */
void ref_pack(const uint8_t *q, int64_t n, int bits, uint8_t *out)
{
    memset(out, 0, (size_t)(n * bits / 8));
    for (int64_t i = 0; i < n; ++i)
        for (int b = 0; b < bits; ++b) {
            int64_t k = i * bits + b;
            if ((q[i] >> b) & 1) out[k >> 3] |= (uint8_t)(1u << (k & 7));
        }
}

void ref_unpack(const uint8_t *in, int64_t n, int bits, uint8_t *q)
{
    for (int64_t i = 0; i < n; ++i) {
        unsigned v = 0;
        for (int b = 0; b < bits; ++b) {
            int64_t k = i * bits + b;
            v |= (unsigned)((in[k >> 3] >> (k & 7)) & 1) << b;
        }
        q[i] = (uint8_t)v;
    }
}

/* ------------------------------------------------------------ entropy coder */

/*
 * Code lengths (reading; the paper names a codec stage, section 5.1, without defining
 * one): Huffman over byte values.  Weights = hist + 1.  Repeatedly join the two nodes
 * with the smallest (weight, id); a leaf's id is its byte value, the k-th joined node's
 * id is 256 + k.  If a code word would be longer than MAX_LEN, replace every weight w
 * by max(1, (w+1)/2) and build again.
 */
void ref_huff_lengths(const uint32_t hist[256], uint8_t len[256])
{
    uint64_t w0[256];
    for (int s = 0; s < 256; ++s) w0[s] = (uint64_t)hist[s] + 1;
    for (;;) {
        uint64_t w[511];
        int parent[511], alive[511];
        for (int i = 0; i < 511; ++i) { parent[i] = -1; alive[i] = 0; w[i] = 0; }
        for (int s = 0; s < 256; ++s) { w[s] = w0[s]; alive[s] = 1; }
        for (int k = 0; k < 255; ++k) {
            int pick[2];
            for (int j = 0; j < 2; ++j) {
                int best = -1;
                for (int i = 0; i < 256 + k; ++i)       /* ids ascend, so '<' keeps the lower id */
                    if (alive[i] && (best < 0 || w[i] < w[best])) best = i;
                alive[best] = 0;
                pick[j] = best;
            }
            int id = 256 + k;
            w[id] = w[pick[0]] + w[pick[1]];
            alive[id] = 1;
            parent[pick[0]] = parent[pick[1]] = id;
        }
        int longest = 0;
        for (int s = 0; s < 256; ++s) {
            int d = 0;
            for (int i = s; parent[i] >= 0; i = parent[i]) ++d;
            len[s] = (uint8_t)d;
            if (d > longest) longest = d;
        }
        if (longest <= MAX_LEN) return;
        for (int s = 0; s < 256; ++s) {
            w0[s] = (w0[s] + 1) >> 1;
            if (w0[s] < 1) w0[s] = 1;
        }
    }
}

/* Canonical code words: by increasing length, then increasing byte value. */
void ref_huff_codes(const uint8_t len[256], uint16_t code[256])
{
    unsigned next = 0;
    for (int L = 1; L <= MAX_LEN; ++L) {
        for (int s = 0; s < 256; ++s)
            if (len[s] == L) code[s] = (uint16_t)next++;
        next <<= 1;
    }
}

static void put_bit(uint8_t *words, int64_t pos, int bit)
{
    /* the stream is a sequence of 32-bit little-endian words filled from bit 31 down */
    int64_t w = pos >> 5;
    int k = 31 - (int)(pos & 31);
    if (bit) words[w * 4 + (k >> 3)] |= (uint8_t)(1u << (k & 7));
}

static int get_bit(const uint8_t *words, int64_t pos)
{
    int64_t w = pos >> 5;
    int k = 31 - (int)(pos & 31);
    return (words[w * 4 + (k >> 3)] >> (k & 7)) & 1;
}

static int64_t align16(int64_t n) { return (n + 15) & ~(int64_t)15; }

/*
 * One chunk = up to CHUNK_ROWS token rows (row_bytes packed bytes each) of one head.
 * Coded body: SUBS x u16 bit counts, one per sub-block of SUB_ROWS rows; then the code
 * words of all bytes, most significant bit first, sub-blocks back to back; zero-padded
 * to 16 bytes.  If that is not smaller than the raw bytes the chunk is stored raw.
 * Returns the body size.
 */
int64_t ref_huff_encode_chunk(const uint8_t *raw, int rows, int row_bytes, const uint8_t len[256],
                              uint8_t *body)
{
    uint16_t code[256];
    ref_huff_codes(len, code);
    int64_t raw_bytes = (int64_t)rows * row_bytes;
    int64_t sub_bytes = (int64_t)SUB_ROWS * row_bytes;
    int64_t bits_of[SUBS], total = 0;
    for (int j = 0; j < SUBS; ++j) {
        int64_t b0 = j * sub_bytes, b1 = b0 + sub_bytes;
        if (b1 > raw_bytes) b1 = raw_bytes;
        bits_of[j] = 0;
        for (int64_t i = b0; i < b1; ++i) bits_of[j] += len[raw[i]];
        total += bits_of[j];
    }
    int64_t coded = align16(2 * SUBS + 4 * ((total + 31) / 32));
    if (coded >= raw_bytes) {
        memcpy(body, raw, (size_t)raw_bytes);
        return raw_bytes;
    }
    memset(body, 0, (size_t)coded);
    for (int j = 0; j < SUBS; ++j) {
        body[2 * j] = (uint8_t)(bits_of[j] & 255);
        body[2 * j + 1] = (uint8_t)(bits_of[j] >> 8);
    }
    int64_t pos = 0;
    for (int64_t i = 0; i < raw_bytes; ++i) {
        int L = len[raw[i]];
        for (int b = L - 1; b >= 0; --b) put_bit(body + 2 * SUBS, pos++, (code[raw[i]] >> b) & 1);
    }
    return coded;
}

int ref_huff_decode_chunk(const uint8_t *body, int64_t body_bytes, int rows, int row_bytes,
                          const uint8_t len[256], uint8_t *raw)
{
    int64_t raw_bytes = (int64_t)rows * row_bytes;
    if (body_bytes == raw_bytes) { memcpy(raw, body, (size_t)raw_bytes); return REF_OK; }
    if (body_bytes > raw_bytes || body_bytes < 2 * SUBS) return REF_ERR_FORMAT;
    /* canonical decoding: the code words of length L are the count[L] consecutive integers
     * from first[L], in the order of sorted[] (by length, then byte value) */
    int count[MAX_LEN + 2], first[MAX_LEN + 2], start[MAX_LEN + 2], sorted[256], n = 0;
    unsigned next = 0;
    for (int L = 1; L <= MAX_LEN; ++L) {
        count[L] = 0; first[L] = (int)next; start[L] = n;
        for (int s = 0; s < 256; ++s)
            if (len[s] == L) { sorted[n++] = s; ++count[L]; ++next; }
        next <<= 1;
    }
    int64_t total = 0;
    for (int j = 0; j < SUBS; ++j) total += body[2 * j] | (body[2 * j + 1] << 8);
    if (align16(2 * SUBS + 4 * ((total + 31) / 32)) != body_bytes) return REF_ERR_FORMAT;
    int64_t pos = 0;
    for (int64_t i = 0; i < raw_bytes; ++i) {
        int acc = 0, L = 0, found = -1;
        while (found < 0) {
            if (L == MAX_LEN || pos >= total) return REF_ERR_FORMAT;
            acc = (acc << 1) | get_bit(body + 2 * SUBS, pos++);
            ++L;
            if (acc - first[L] >= 0 && acc - first[L] < count[L]) found = sorted[start[L] + acc - first[L]];
        }
        raw[i] = (uint8_t)found;
    }
    return pos == total ? REF_OK : REF_ERR_FORMAT;
}

/* ----------------------------------------------------------------- geometry */

static int bits_ok(int b) { return b == 2 || b == 3 || b == 4 || b == 8 || b == 16; }

/*
 * Mixed precision at head granularity (KVServe section 5.1: "mixed-precision at layer-wise and
 * head-wise granularity", and MixHQ: heads that matter keep a high precision, the others drop to
 * very few bits instead of being pruned).  The paper names the mechanism only; the reading here:
 * an optional table per tensor gives the width of every (layer, head); groups, metadata and
 * code order are those of the uniform case, the codes of the heads follow each other in
 * (layer, head) order, each with its own width, and the tables travel in the payload's
 * auxiliary section (K table, then V table, one byte per head).  Which head gets which width is
 * the caller's business (the paper takes it from trained head masks).
 *
 * Together with the lossless stage (section 5.1 composes any quantizer with any codec): the chunks of
 * a section are then ordered by width first (2, 3, 4, 8), inside a width by (layer, head, chunk), and
 * every width present in a tensor has its own code table, built from a sample of that width's chunks
 * (bytes that pack four 2-bit codes and bytes that hold one 8-bit code have nothing in common).  The
 * auxiliary section starts with eight tables of 256 length bytes, K widths 2, 3, 4, 8, then V widths
 * 2, 3, 4, 8 (all zero for a width the tensor does not use; a tensor without a table counts as one
 * width), then the directory in that chunk order, then the width tables.
 */
static const int WIDTHS[4] = {2, 3, 4, 8};

static int bits_at(const ref_config *c, int is_v, int64_t lh);

static int has_tables(const ref_config *c) { return c->head_bits_k || c->head_bits_v; }

/* bytes of code tables at the start of the auxiliary section (codec 1) */
static int64_t code_table_bytes(const ref_config *c) { return has_tables(c) ? 8 * 256 : 2 * 256; }

/* heads of tensor is_v whose width is `bits`, in (layer, head) order; returns their number */
static int64_t heads_of_width(const ref_config *c, int is_v, int bits, int64_t *list)
{
    int64_t n = 0;
    for (int64_t lh = 0; lh < (int64_t)c->layers * c->heads; ++lh)
        if (bits_at(c, is_v, lh) == bits) { if (list) list[n] = lh; ++n; }
    return n;
}
static int bits_at(const ref_config *c, int is_v, int64_t lh)
{
    const uint8_t *t = is_v ? c->head_bits_v : c->head_bits_k;
    return t ? t[lh] : (is_v ? c->bits_v : c->bits_k);
}

static int table_ok(const ref_config *c, int is_v)
{
    const uint8_t *t = is_v ? c->head_bits_v : c->head_bits_k;
    if (!t) return 1;
    if ((is_v ? c->bits_v : c->bits_k) != 0) return 0;
    for (int64_t i = 0; i < (int64_t)c->layers * c->heads; ++i)
        if (t[i] != 2 && t[i] != 3 && t[i] != 4 && t[i] != 8) return 0;
    return 1;
}

/* limits that keep every byte count of a payload far below 2^63 */
#define MAX_HEADS ((int64_t)1 << 20)
#define MAX_TOKENS ((int64_t)1 << 32)

int ref_check_config(const ref_config *c)
{
    if (!c) return REF_ERR_ARG;
    if (c->dtype != REF_F16 && c->dtype != REF_BF16) return REF_ERR_ARG;
    if (c->layers < 1 || c->heads < 1 || c->head_dim < 8 || c->head_dim % 8) return REF_ERR_ARG;
    if ((int64_t)c->layers * c->heads > MAX_HEADS || c->head_dim > 1024) return REF_ERR_ARG;
    if (!table_ok(c, 0) || !table_ok(c, 1)) return REF_ERR_ARG;
    if ((!c->head_bits_k && !bits_ok(c->bits_k)) || (!c->head_bits_v && !bits_ok(c->bits_v))) return REF_ERR_ARG;
    if (c->bits_k != 16 && (c->group_k < 1 || c->group_k > CHUNK_ROWS || CHUNK_ROWS % c->group_k))
        return REF_ERR_ARG;
    if (c->bits_v != 16 && (c->group_v < 1 || c->head_dim % c->group_v)) return REF_ERR_ARG;
    if (c->codec != 0 && c->codec != 1) return REF_ERR_ARG;
    if (c->codec == 1 && (c->bits_k == 16 || c->bits_v == 16)) return REF_ERR_UNSUPPORTED;
    if (c->transform < 0 || c->transform > 2) return REF_ERR_ARG;
    if (c->transform == 2) {
        int a = c->anchor_period;
        if (a < 8 || a > 128 || (a & (a - 1))) return REF_ERR_ARG;
    } else if (c->anchor_period != 0) return REF_ERR_ARG;
    if (c->transform == 1 && ((c->head_dim & (c->head_dim - 1)) || c->head_dim > 1024)) return REF_ERR_UNSUPPORTED;
    return REF_OK;
}

int64_t ref_chunks_per_head(int64_t tokens) { return (tokens + CHUNK_ROWS - 1) / CHUNK_ROWS; }

typedef struct {
    int64_t meta_k, meta_v, aux, codes_k, codes_v;       /* byte sizes (codes: raw size) */
    int64_t off_meta_k, off_meta_v, off_aux, off_codes_k, off_codes_v, total;
    int64_t chunks_k, chunks_v;
    int64_t anchors_k, anchors_v, off_anchors_k, off_anchors_v;   /* inside the auxiliary section */
} geometry;

/* anchor rows one head of a tensor carries (delta transform; a tensor stored unchanged has none) */
static int64_t anchor_rows(const ref_config *c, int is_v, int64_t T)
{
    if (c->transform != 2) return 0;
    if (!(is_v ? c->head_bits_v : c->head_bits_k) && (is_v ? c->bits_v : c->bits_k) == 16) return 0;
    return (T + c->anchor_period - 1) / c->anchor_period;
}

/*
 * Payload = header | K meta | V meta | auxiliary section | K codes | V codes, every part
 * starting on a 16-byte boundary.  The auxiliary section holds the coder's tables and directory
 * or the per-head width tables, then (delta transform, from the next 16-byte boundary) the anchor
 * rows of K and of V, [layer][head][run][channel], 16 bits each.  Metadata is two fp16 values per group
 * (the 32 bits per group behind the paper's 5.33x figure for 2 bits and groups of 32,
 * section 7.3); codes are bits/8 bytes per element.
 */
static void layout_of(const ref_config *c, int64_t T, geometry *g)
{
    int64_t LH = (int64_t)c->layers * c->heads, D = c->head_dim;
    g->meta_k = c->bits_k == 16 ? 0 : 4 * LH * ((T + c->group_k - 1) / c->group_k) * D;
    g->meta_v = c->bits_v == 16 ? 0 : 4 * LH * T * (D / c->group_v);
    g->codes_k = g->codes_v = 0;
    for (int64_t lh = 0; lh < LH; ++lh) {
        g->codes_k += T * D * bits_at(c, 0, lh) / 8;
        g->codes_v += T * D * bits_at(c, 1, lh) / 8;
    }
    g->chunks_k = g->chunks_v = LH * ref_chunks_per_head(T);
    g->aux = c->codec ? code_table_bytes(c) + 4 * (g->chunks_k + g->chunks_v + 1) : 0;
    g->aux += (c->head_bits_k ? LH : 0) + (c->head_bits_v ? LH : 0);
    g->anchors_k = 2 * LH * anchor_rows(c, 0, T) * D;
    g->anchors_v = 2 * LH * anchor_rows(c, 1, T) * D;
    if (c->transform == 2) g->aux = align16(g->aux) + g->anchors_k + g->anchors_v;
    g->off_meta_k = HEADER;
    g->off_meta_v = g->off_meta_k + align16(g->meta_k);
    g->off_aux = g->off_meta_v + align16(g->meta_v);
    g->off_codes_k = g->off_aux + align16(g->aux);
    g->off_anchors_k = g->off_codes_k - g->anchors_v - g->anchors_k;
    g->off_anchors_v = g->off_codes_k - g->anchors_v;
    g->off_codes_v = g->off_codes_k + align16(g->codes_k);
    g->total = g->off_codes_v + align16(g->codes_v);
}

/* Exact without the coder; with it, the bound reached when every chunk is stored raw. */
int ref_payload_size(const ref_config *c, int64_t tokens, uint64_t *bytes, int *is_exact)
{
    int rc = ref_check_config(c);
    if (rc) return rc;
    if (tokens < 0 || tokens > MAX_TOKENS || !bytes) return REF_ERR_ARG;
    geometry g;
    layout_of(c, tokens, &g);
    *bytes = (uint64_t)g.total;
    if (is_exact) *is_exact = c->codec == 0;
    return REF_OK;
}

/* ----------------------------------------------------------- one (l, h) head */

/*
 * K: one group per channel d and block of group_k consecutive tokens (the last block of a
 * sequence may be shorter).  V: one group per token and block of group_v consecutive
 * channels.  Codes keep the [t][d] order of the input for both.
 */
int ref_compress_head(const ref_config *c, int is_v, const void *src, const ref_layout *lay,
                      int64_t T, int l, int h, uint8_t *codes, uint16_t *meta)
{
    int D = c->head_dim, bits = bits_at(c, is_v, (int64_t)l * c->heads + h);
    if (bits == 16) {
        for (int64_t t = 0; t < T; ++t)
            memcpy(codes + t * D * 2, (const uint16_t *)src + row_offset(lay, l, h, t), (size_t)D * 2);
        return REF_OK;
    }
    if (c->transform) {
        /* T first: the quantizer then sees the transformed rows as its input tensor */
        uint16_t *xt = (uint16_t *)malloc((size_t)(T * D) * 2 + 2);
        if (!xt) return REF_ERR_ARG;
        for (int64_t t = 0; t < T; ++t) {
            const uint16_t *row = (const uint16_t *)src + row_offset(lay, l, h, t);
            if (c->transform == 1) ref_hadamard_row(row, xt + t * D, D, c->dtype, 0);
            else ref_delta_row(row, (const uint16_t *)src + row_offset(lay, l, h, t - t % c->anchor_period),
                               xt + t * D, D, c->dtype, 0);
        }
        ref_config plain = *c;
        plain.transform = plain.anchor_period = 0;
        plain.head_bits_k = plain.head_bits_v = NULL;
        plain.bits_k = plain.bits_v = bits;
        ref_layout rows = {0, 0, D, 0, 0, NULL};
        int rc = ref_compress_head(&plain, is_v, xt, &rows, T, 0, 0, codes, meta);
        free(xt);
        return rc;
    }
    uint8_t *q = (uint8_t *)malloc((size_t)(T * D) + 1);
    float *grp = (float *)malloc(sizeof(float) * (size_t)(c->group_k > D ? c->group_k : D));
    uint8_t *gq = (uint8_t *)malloc((size_t)(c->group_k > D ? c->group_k : D));
    if (!q || !grp || !gq) { free(q); free(grp); free(gq); return REF_ERR_ARG; }
    if (!is_v) {
        int g = c->group_k;
        for (int64_t tb = 0; tb * g < T; ++tb) {
            int n = (int)((T - tb * g) < g ? (T - tb * g) : g);
            for (int d = 0; d < D; ++d) {
                for (int i = 0; i < n; ++i)
                    grp[i] = load_elem(src, c->dtype, row_offset(lay, l, h, tb * g + i) + d);
                uint16_t s, z;
                ref_group_meta(grp, n, bits, &s, &z);
                ref_group_quantize(grp, n, bits, s, z, gq);
                meta[(tb * D + d) * 2] = s;
                meta[(tb * D + d) * 2 + 1] = z;
                for (int i = 0; i < n; ++i) q[(tb * g + i) * D + d] = gq[i];
            }
        }
    } else {
        int g = c->group_v, nb = D / g;
        for (int64_t t = 0; t < T; ++t)
            for (int cb = 0; cb < nb; ++cb) {
                for (int i = 0; i < g; ++i)
                    grp[i] = load_elem(src, c->dtype, row_offset(lay, l, h, t) + cb * g + i);
                uint16_t s, z;
                ref_group_meta(grp, g, bits, &s, &z);
                ref_group_quantize(grp, g, bits, s, z, gq);
                meta[(t * nb + cb) * 2] = s;
                meta[(t * nb + cb) * 2 + 1] = z;
                for (int i = 0; i < g; ++i) q[t * D + cb * g + i] = gq[i];
            }
    }
    ref_pack(q, T * D, bits, codes);
    free(q); free(grp); free(gq);
    return REF_OK;
}

int ref_decompress_head(const ref_config *c, int is_v, const uint8_t *codes, const uint16_t *meta,
                        const uint16_t *anchors, int64_t T, int l, int h, void *dst,
                        const ref_layout *lay)
{
    int D = c->head_dim, bits = bits_at(c, is_v, (int64_t)l * c->heads + h);
    uint16_t *out = (uint16_t *)dst;
    if (bits == 16) {
        for (int64_t t = 0; t < T; ++t)
            memcpy(out + row_offset(lay, l, h, t), codes + t * D * 2, (size_t)D * 2);
        return REF_OK;
    }
    if (c->transform) {
        /* reconstruct the transformed rows, then undo T row by row */
        uint16_t *xt = (uint16_t *)malloc((size_t)(T * D) * 2 + 2);
        if (!xt) return REF_ERR_ARG;
        if (c->transform == 2 && !anchors && T > 0) { free(xt); return REF_ERR_ARG; }
        ref_config plain = *c;
        plain.transform = plain.anchor_period = 0;
        plain.head_bits_k = plain.head_bits_v = NULL;
        plain.bits_k = plain.bits_v = bits;
        ref_layout rows = {0, 0, D, 0, 0, NULL};
        int rc = ref_decompress_head(&plain, is_v, codes, meta, NULL, T, 0, 0, xt, &rows);
        for (int64_t t = 0; t < T && rc == REF_OK; ++t) {
            uint16_t *row = out + row_offset(lay, l, h, t);
            if (c->transform == 1) ref_hadamard_row(xt + t * D, row, D, c->dtype, 1);
            else {
                const uint16_t *anchor = anchors + (t / c->anchor_period) * D;
                if (t % c->anchor_period == 0) memcpy(row, anchor, (size_t)D * 2);
                else ref_delta_row(xt + t * D, anchor, row, D, c->dtype, 1);
            }
        }
        free(xt);
        return rc;
    }
    uint8_t *q = (uint8_t *)malloc((size_t)(T * D) + 1);
    if (!q) return REF_ERR_ARG;
    ref_unpack(codes, T * D, bits, q);
    for (int64_t t = 0; t < T; ++t)
        for (int d = 0; d < D; ++d) {
            int64_t m = is_v ? (t * (D / c->group_v) + d / c->group_v)
                             : ((t / c->group_k) * D + d);
            out[row_offset(lay, l, h, t) + d] =
                ref_dequantize(q[t * D + d], meta[2 * m], meta[2 * m + 1], c->dtype);
        }
    free(q);
    return REF_OK;
}

/* ----------------------------------------------------------- coder plumbing */

static int64_t head_code_bytes(const ref_config *c, int is_v, int64_t T)
{
    return T * c->head_dim * (is_v ? c->bits_v : c->bits_k) / 8;
}

/* byte offset of head lh's codes inside its section, and their size */
static int64_t head_code_off(const ref_config *c, int is_v, int64_t T, int64_t lh, int64_t *bytes)
{
    int64_t off = 0;
    for (int64_t j = 0; j < lh; ++j) off += T * c->head_dim * bits_at(c, is_v, j) / 8;
    if (bytes) *bytes = T * c->head_dim * bits_at(c, is_v, lh) / 8;
    return off;
}

static int64_t head_meta_pairs(const ref_config *c, int is_v, int64_t T)
{
    if (!(is_v ? c->head_bits_v : c->head_bits_k) && (is_v ? c->bits_v : c->bits_k) == 16) return 0;
    return is_v ? T * (c->head_dim / c->group_v)
                : ((T + c->group_k - 1) / c->group_k) * c->head_dim;
}

/* raw packed bytes of chunk `chunk` of a section: rows [cb*128, ...) of head (l, h) */
static int chunk_raw(const ref_config *c, int is_v, const void *src, const ref_layout *lay,
                     int64_t T, int64_t chunk, uint8_t *raw, int *rows_out)
{
    int64_t cph = ref_chunks_per_head(T);
    int64_t lh = chunk / cph, cb = chunk % cph;
    int l = (int)(lh / c->heads), h = (int)(lh % c->heads);
    int row_bytes = c->head_dim * (is_v ? c->bits_v : c->bits_k) / 8;
    uint8_t *codes = (uint8_t *)malloc((size_t)head_code_bytes(c, is_v, T) + 1);
    uint16_t *meta = (uint16_t *)malloc((size_t)head_meta_pairs(c, is_v, T) * 4 + 4);
    if (!codes || !meta) { free(codes); free(meta); return REF_ERR_ARG; }
    int rc = ref_compress_head(c, is_v, src, lay, T, l, h, codes, meta);
    int64_t r0 = cb * CHUNK_ROWS, r1 = r0 + CHUNK_ROWS;
    if (r1 > T) r1 = T;
    memcpy(raw, codes + r0 * row_bytes, (size_t)((r1 - r0) * row_bytes));
    *rows_out = (int)(r1 - r0);
    free(codes); free(meta);
    return rc;
}

/* Table sample (reading): chunks floor(i*n/16), i = 0..15, each counted once. */
static int sample_hist(const ref_config *c, int is_v, const void *src, const ref_layout *lay,
                       int64_t T, uint32_t hist[256])
{
    int64_t n = (int64_t)c->layers * c->heads * ref_chunks_per_head(T), last = -1;
    int row_bytes = c->head_dim * (is_v ? c->bits_v : c->bits_k) / 8;
    uint8_t *raw = (uint8_t *)malloc((size_t)CHUNK_ROWS * row_bytes);
    if (!raw) return REF_ERR_ARG;
    memset(hist, 0, 256 * sizeof(uint32_t));
    for (int i = 0; i < 16 && n > 0; ++i) {
        int64_t ch = (int64_t)i * n / 16;
        if (ch == last) continue;
        last = ch;
        int rows;
        int rc = chunk_raw(c, is_v, src, lay, T, ch, raw, &rows);
        if (rc) { free(raw); return rc; }
        for (int64_t b = 0; b < (int64_t)rows * row_bytes; ++b) hist[raw[b]]++;
    }
    free(raw);
    return REF_OK;
}

int ref_huff_tables(const ref_config *c, const void *k, const void *v, const ref_layout *lay,
                    int64_t T, uint8_t len_k[256], uint8_t len_v[256])
{
    uint32_t hist[256];
    int rc = sample_hist(c, 0, k, lay, T, hist);
    if (rc) return rc;
    ref_huff_lengths(hist, len_k);
    rc = sample_hist(c, 1, v, lay, T, hist);
    if (rc) return rc;
    ref_huff_lengths(hist, len_v);
    return REF_OK;
}

int64_t ref_encode_chunk_at(const ref_config *c, int is_v, const void *src, const ref_layout *lay,
                            int64_t T, int64_t chunk, const uint8_t len[256], uint8_t *body)
{
    int row_bytes = c->head_dim * (is_v ? c->bits_v : c->bits_k) / 8;
    uint8_t *raw = (uint8_t *)malloc((size_t)CHUNK_ROWS * row_bytes);
    if (!raw) return REF_ERR_ARG;
    int rows;
    int rc = chunk_raw(c, is_v, src, lay, T, chunk, raw, &rows);
    int64_t n = rc ? rc : ref_huff_encode_chunk(raw, rows, row_bytes, len, body);
    free(raw);
    return n;
}

/* ----------------------------------------------------------- whole request */

static void put_u16(uint8_t *p, unsigned v) { p[0] = (uint8_t)v; p[1] = (uint8_t)(v >> 8); }
static void put_u32(uint8_t *p, uint32_t v) { for (int i = 0; i < 4; ++i) p[i] = (uint8_t)(v >> (8 * i)); }
static void put_u64(uint8_t *p, uint64_t v) { for (int i = 0; i < 8; ++i) p[i] = (uint8_t)(v >> (8 * i)); }
static unsigned get_u16(const uint8_t *p) { return p[0] | (p[1] << 8); }
static uint32_t get_u32(const uint8_t *p) { uint32_t v = 0; for (int i = 0; i < 4; ++i) v |= (uint32_t)p[i] << (8 * i); return v; }
static uint64_t get_u64(const uint8_t *p) { uint64_t v = 0; for (int i = 0; i < 8; ++i) v |= (uint64_t)p[i] << (8 * i); return v; }

/*
 * Header, 128 bytes, little endian:
 *   0 "KVC1" | 4 u16 version=1 | 6 u8 dtype | 7 u8 codec | 8 i32 layers | 12 i32 heads |
 *   16 i32 head_dim | 20 u8 bits_k | 21 u8 bits_v | 22 u16 group_k | 24 u16 group_v |
 *   26 u8 transform | 27 u8 width-table flags | 28 u16 anchor period | 30..31 zero |
 *   32 i64 tokens | 40 u64 total bytes |
 *   48.. five (offset u64, bytes u64) pairs: K meta, V meta, coder aux, K codes, V codes
 */
static void write_header(uint8_t *p, const ref_config *c, int64_t T, const geometry *g,
                         int64_t bytes_codes_k, int64_t bytes_codes_v, int64_t total)
{
    memset(p, 0, HEADER);
    memcpy(p, "KVC1", 4);
    put_u16(p + 4, 1);
    p[6] = (uint8_t)c->dtype;
    p[7] = (uint8_t)c->codec;
    put_u32(p + 8, (uint32_t)c->layers);
    put_u32(p + 12, (uint32_t)c->heads);
    put_u32(p + 16, (uint32_t)c->head_dim);
    p[20] = (uint8_t)c->bits_k;
    p[21] = (uint8_t)c->bits_v;
    put_u16(p + 22, (unsigned)c->group_k);
    put_u16(p + 24, (unsigned)c->group_v);
    p[26] = (uint8_t)c->transform;
    p[27] = (uint8_t)((c->head_bits_k ? 1 : 0) | (c->head_bits_v ? 2 : 0));
    put_u16(p + 28, (unsigned)c->anchor_period);
    put_u64(p + 32, (uint64_t)T);
    put_u64(p + 40, (uint64_t)total);
    put_u64(p + 48, (uint64_t)g->off_meta_k);  put_u64(p + 56, (uint64_t)g->meta_k);
    put_u64(p + 64, (uint64_t)g->off_meta_v);  put_u64(p + 72, (uint64_t)g->meta_v);
    put_u64(p + 80, (uint64_t)g->off_aux);     put_u64(p + 88, (uint64_t)g->aux);
    put_u64(p + 96, (uint64_t)g->off_codes_k); put_u64(p + 104, (uint64_t)bytes_codes_k);
    put_u64(p + 112, (uint64_t)(g->off_codes_k + align16(bytes_codes_k)));
    put_u64(p + 120, (uint64_t)bytes_codes_v);
}

int ref_inspect(const uint8_t *p, ref_config *c, int64_t *tokens, uint64_t *total_bytes,
                uint64_t sections[10])
{
    if (!p || !c) return REF_ERR_ARG;
    if (memcmp(p, "KVC1", 4) != 0 || get_u16(p + 4) != 1) return REF_ERR_FORMAT;
    memset(c, 0, sizeof *c);
    c->dtype = p[6];
    c->codec = p[7];
    c->layers = (int32_t)get_u32(p + 8);
    c->heads = (int32_t)get_u32(p + 12);
    c->head_dim = (int32_t)get_u32(p + 16);
    c->bits_k = p[20];
    c->bits_v = p[21];
    c->group_k = (int32_t)get_u16(p + 22);
    c->group_v = (int32_t)get_u16(p + 24);
    c->transform = p[26];
    c->anchor_period = (int32_t)get_u16(p + 28);
    if (p[30] | p[31]) return REF_ERR_FORMAT;
    /* per-head tables sit at the start of the auxiliary section: the pointers are only valid
     * when `p` is the whole payload, not just its header */
    {
        int64_t LH = (int64_t)c->layers * c->heads;
        const uint8_t *aux = p + get_u64(p + 80);
        if (p[27] & ~3) return REF_ERR_FORMAT;
        if (c->codec && p[27])       /* behind the eight code tables and the directory */
            aux += 8 * 256 + 4 * (2 * LH * ref_chunks_per_head((int64_t)get_u64(p + 32)) + 1);
        if (p[27] & 1) { c->head_bits_k = aux; aux += LH; }
        if (p[27] & 2) c->head_bits_v = aux;
    }
    if (tokens) *tokens = (int64_t)get_u64(p + 32);
    if (total_bytes) *total_bytes = get_u64(p + 40);
    if (sections) for (int i = 0; i < 10; ++i) sections[i] = get_u64(p + 48 + 8 * i);
    {
        /* the tables themselves are checked by ref_decompress, which knows the payload size */
        ref_config fields = *c;
        if (fields.head_bits_k) { fields.head_bits_k = NULL; fields.bits_k = fields.bits_k ? 0xff : 4; }
        if (fields.head_bits_v) { fields.head_bits_v = NULL; fields.bits_v = fields.bits_v ? 0xff : 4; }
        if (ref_check_config(&fields) != REF_OK || (int64_t)get_u64(p + 32) < 0 ||
            (int64_t)get_u64(p + 32) > MAX_TOKENS)
            return REF_ERR_FORMAT;
    }
    return REF_OK;
}

int ref_compress(const ref_config *c, const void *k, const void *v, const ref_layout *lay,
                 int64_t T, uint8_t *payload, uint64_t capacity, uint64_t *out_bytes)
{
    int rc = ref_check_config(c);
    if (rc) return rc;
    if (T < 0 || T > MAX_TOKENS || !payload || !lay || (T > 0 && (!k || !v))) return REF_ERR_ARG;
    geometry g;
    layout_of(c, T, &g);
    if (capacity < (uint64_t)g.total) return REF_ERR_CAPACITY;
    memset(payload, 0, (size_t)g.total);

    /* delta transform: the anchor rows travel as they are */
    for (int is_v = 0; is_v < 2; ++is_v) {
        int64_t n = anchor_rows(c, is_v, T);
        uint16_t *dst = (uint16_t *)(payload + (is_v ? g.off_anchors_v : g.off_anchors_k));
        for (int l = 0; l < c->layers; ++l)
            for (int h = 0; h < c->heads; ++h)
                for (int64_t r = 0; r < n; ++r, dst += c->head_dim)
                    memcpy(dst, (const uint16_t *)(is_v ? v : k) + row_offset(lay, l, h, r * c->anchor_period),
                           (size_t)c->head_dim * 2);
    }

    /* Q: quantize and pack both tensors, head by head */
    uint8_t *codes[2];
    for (int is_v = 0; is_v < 2; ++is_v) {
        int64_t hm = head_meta_pairs(c, is_v, T) * 4;
        uint8_t *cbase = c->codec ? (uint8_t *)malloc((size_t)(is_v ? g.codes_v : g.codes_k) + 1)
                                  : payload + (is_v ? g.off_codes_v : g.off_codes_k);
        if (!cbase) return REF_ERR_ARG;
        codes[is_v] = cbase;
        uint8_t *mbase = payload + (is_v ? g.off_meta_v : g.off_meta_k);
        for (int l = 0; l < c->layers; ++l)
            for (int h = 0; h < c->heads; ++h) {
                int64_t lh = (int64_t)l * c->heads + h;
                rc = ref_compress_head(c, is_v, is_v ? v : k, lay, T, l, h,
                                       cbase + head_code_off(c, is_v, T, lh, NULL),
                                       (uint16_t *)(mbase + lh * hm));
                if (rc) return rc;
            }
    }
    {
        /* the width tables follow the coder's tables and directory (if any) */
        int64_t LH = (int64_t)c->layers * c->heads;
        uint8_t *tab = payload + g.off_aux + (c->codec ? code_table_bytes(c) + 4 * (g.chunks_k + g.chunks_v + 1) : 0);
        if (c->head_bits_k) { memcpy(tab, c->head_bits_k, (size_t)LH); tab += LH; }
        if (c->head_bits_v) memcpy(tab, c->head_bits_v, (size_t)LH);
    }
    if (!c->codec) {
        write_header(payload, c, T, &g, g.codes_k, g.codes_v, g.total);
        if (out_bytes) *out_bytes = (uint64_t)g.total;
        return REF_OK;
    }

    /* C: per tensor and width, a table from the sample, then chunk after chunk; the directory holds
     * the running sum of body sizes in units of 16 bytes (entry i = where chunk i starts, K chunks
     * first, one more entry for the end).  Without width tables a tensor is one width and the
     * chunk order is (layer, head, chunk). */
    uint8_t *aux = payload + g.off_aux;
    const int64_t tab_bytes = code_table_bytes(c), LHall = (int64_t)c->layers * c->heads;
    int64_t cph = ref_chunks_per_head(T), dir = 0, idx = 0, bytes_codes[2];
    uint8_t *out = payload + g.off_codes_k;
    int64_t *list = (int64_t *)malloc(sizeof(int64_t) * (size_t)(LHall + 1));
    if (!list) return REF_ERR_ARG;
    for (int is_v = 0; is_v < 2; ++is_v) {
        int64_t start = dir;
        for (int wi = 0; wi < 5; ++wi) {
            int bits = wi < 4 ? WIDTHS[wi] : 16;                 /* (16 never occurs with the coder) */
            int64_t heads_w = heads_of_width(c, is_v, bits, list);
            if (heads_w == 0 || bits == 16) continue;
            int row_bytes = c->head_dim * bits / 8;
            int64_t n = heads_w * cph;
            uint32_t hist[256];
            int64_t last = -1;
            memset(hist, 0, sizeof hist);
            for (int i = 0; i < 16 && n > 0; ++i) {
                int64_t ch = (int64_t)i * n / 16;
                if (ch == last) continue;
                last = ch;
                int64_t lh = list[ch / cph], cb = ch % cph;
                int64_t r0 = cb * CHUNK_ROWS, r1 = r0 + CHUNK_ROWS > T ? T : r0 + CHUNK_ROWS;
                const uint8_t *raw = codes[is_v] + head_code_off(c, is_v, T, lh, NULL) + r0 * row_bytes;
                for (int64_t b = 0; b < (r1 - r0) * row_bytes; ++b) hist[raw[b]]++;
            }
            uint8_t *len = aux + 256 * (has_tables(c) ? 4 * is_v + wi : is_v);
            ref_huff_lengths(hist, len);
            for (int64_t ch = 0; ch < n; ++ch, ++idx) {
                int64_t lh = list[ch / cph], cb = ch % cph;
                int64_t r0 = cb * CHUNK_ROWS, r1 = r0 + CHUNK_ROWS > T ? T : r0 + CHUNK_ROWS;
                put_u32(aux + tab_bytes + 4 * idx, (uint32_t)(dir / 16));
                dir += ref_huff_encode_chunk(codes[is_v] + head_code_off(c, is_v, T, lh, NULL) + r0 * row_bytes,
                                             (int)(r1 - r0), row_bytes, len, out + dir);
            }
        }
        bytes_codes[is_v] = dir - start;
        free(codes[is_v]);
    }
    free(list);
    put_u32(aux + tab_bytes + 4 * idx, (uint32_t)(dir / 16));
    int64_t total = g.off_codes_k + dir;
    write_header(payload, c, T, &g, bytes_codes[0], bytes_codes[1], total);
    if (out_bytes) *out_bytes = (uint64_t)total;
    return REF_OK;
}

int ref_decompress(const uint8_t *payload, uint64_t bytes, void *k, void *v,
                   const ref_layout *lay, const ref_config *expect)
{
    if (!payload || bytes < HEADER || !lay) return REF_ERR_ARG;
    ref_config c;
    int64_t T;
    uint64_t total, sec[10];
    int rc = ref_inspect(payload, &c, &T, &total, sec);
    if (rc) return rc;
    if (total > bytes) return REF_ERR_FORMAT;
    {
        int64_t LH = (int64_t)c.layers * c.heads;
        uint64_t tables = (uint64_t)((c.head_bits_k ? LH : 0) + (c.head_bits_v ? LH : 0));
        if (tables && sec[4] + sec[5] > total) return REF_ERR_FORMAT;
        if (ref_check_config(&c) != REF_OK) return REF_ERR_FORMAT;
        if (expect) {
            ref_config a = *expect, b = c;
            a.head_bits_k = a.head_bits_v = b.head_bits_k = b.head_bits_v = NULL;
            if (memcmp(&a, &b, sizeof a) != 0) return REF_ERR_MISMATCH;
            if (!expect->head_bits_k != !c.head_bits_k || !expect->head_bits_v != !c.head_bits_v) return REF_ERR_MISMATCH;
            if (c.head_bits_k && memcmp(expect->head_bits_k, c.head_bits_k, (size_t)LH)) return REF_ERR_MISMATCH;
            if (c.head_bits_v && memcmp(expect->head_bits_v, c.head_bits_v, (size_t)LH)) return REF_ERR_MISMATCH;
        }
    }
    geometry g;
    layout_of(&c, T, &g);
    if (sec[0] != (uint64_t)g.off_meta_k || sec[1] != (uint64_t)g.meta_k ||
        sec[2] != (uint64_t)g.off_meta_v || sec[3] != (uint64_t)g.meta_v ||
        sec[4] != (uint64_t)g.off_aux || sec[5] != (uint64_t)g.aux ||
        sec[6] != (uint64_t)g.off_codes_k)
        return REF_ERR_FORMAT;
    if (!c.codec && (sec[7] != (uint64_t)g.codes_k || sec[8] != (uint64_t)g.off_codes_v ||
                     sec[9] != (uint64_t)g.codes_v || total != (uint64_t)g.total))
        return REF_ERR_FORMAT;

    const uint8_t *aux = payload + g.off_aux;
    const int64_t tab_bytes = code_table_bytes(&c), LHall = (int64_t)c.layers * c.heads;
    int64_t cph = ref_chunks_per_head(T);
    int64_t *place = (int64_t *)malloc(sizeof(int64_t) * (size_t)(LHall + 1));    /* head -> rank in the chunk order */
    int64_t *list = (int64_t *)malloc(sizeof(int64_t) * (size_t)(LHall + 1));
    if (!place || !list) { free(place); free(list); return REF_ERR_ARG; }
    for (int is_v = 0; is_v < 2; ++is_v) {
        int64_t hm = head_meta_pairs(&c, is_v, T) * 4, at = 0;
        for (int wi = 0; wi < 4; ++wi) {              /* chunk order: by width, then (layer, head) */
            int64_t n = heads_of_width(&c, is_v, WIDTHS[wi], list);
            for (int64_t i = 0; i < n; ++i) place[list[i]] = at++;
        }
        const uint8_t *mbase = payload + (is_v ? g.off_meta_v : g.off_meta_k);
        uint8_t *head = (uint8_t *)malloc((size_t)(T * c.head_dim) + 1);              /* room for 8-bit codes */
        if (!head) { free(place); free(list); return REF_ERR_ARG; }
        for (int l = 0; l < c.layers; ++l)
            for (int h = 0; h < c.heads; ++h) {
                int64_t lh = (int64_t)l * c.heads + h;
                const uint8_t *codes = payload + (is_v ? g.off_codes_v : g.off_codes_k) +
                                       head_code_off(&c, is_v, T, lh, NULL);
                if (c.codec) {
                    int bits = bits_at(&c, is_v, lh), wi = bits == 2 ? 0 : bits == 3 ? 1 : bits == 4 ? 2 : 3;
                    int row_bytes = c.head_dim * bits / 8;
                    const uint8_t *len = aux + 256 * (has_tables(&c) ? 4 * is_v + wi : is_v);
                    for (int64_t cb = 0; cb < cph; ++cb) {
                        int64_t idx = (is_v ? g.chunks_k : 0) + place[lh] * cph + cb;
                        uint64_t a = 16ull * get_u32(aux + tab_bytes + 4 * idx);
                        uint64_t b = 16ull * get_u32(aux + tab_bytes + 4 * (idx + 1));
                        int64_t r0 = cb * CHUNK_ROWS, r1 = r0 + CHUNK_ROWS > T ? T : r0 + CHUNK_ROWS;
                        if (b < a || (uint64_t)g.off_codes_k + b > total) { free(head); free(place); free(list); return REF_ERR_FORMAT; }
                        rc = ref_huff_decode_chunk(payload + g.off_codes_k + a, (int64_t)(b - a),
                                                   (int)(r1 - r0), row_bytes, len, head + r0 * row_bytes);
                        if (rc) { free(head); free(place); free(list); return rc; }
                    }
                    codes = head;
                }
                const uint16_t *anchors = (const uint16_t *)(payload + (is_v ? g.off_anchors_v : g.off_anchors_k)) +
                                          lh * anchor_rows(&c, is_v, T) * c.head_dim;
                rc = ref_decompress_head(&c, is_v, codes, (const uint16_t *)(mbase + lh * hm), anchors,
                                         T, l, h, is_v ? v : k, lay);
                if (rc) { free(head); free(place); free(list); return rc; }
            }
        free(head);
    }
    free(place);
    free(list);
    return REF_OK;
}
