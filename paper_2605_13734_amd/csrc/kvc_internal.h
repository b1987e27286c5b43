// Host-side declarations shared by the translation units of libkvc (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kvc_device.h"

namespace kvc {

// Arguments of the codec-free quantize / dequantize kernels for one tensor of one request.
struct QuantArgs {
    TensorView x;               // source (compress) or destination (decompress)
    uint8_t *codes;             // section base inside the payload
    uint8_t *meta;              // metadata section base
    long long tokens;
    int heads;
    int group;                  // runtime copy of the group size
    int dense;                  // rows of a head are contiguous: stride_token == head_dim, no block table
    int head_minor;             // the heads of a token lie next to each other (stride_head < stride_token, as in a
                                // paged pool): neighbouring work units then take the same tokens of neighbouring heads
    int rotate;                 // stage T: rows are Hadamard-transformed on the way in / back on the way out
    // stage T, delta transform: the tensor's anchor rows inside the payload,
    // [layer * heads + head][ceil(tokens / period)][128] (null = transform off), period = 1 << anchor_shift
    uint16_t *anchors;
    int anchor_shift;
    // per-head bit widths (null = one width for all heads): the heads this launch covers, and for
    // every head the sum of the widths of the heads before it (its codes start at that many times
    // tokens * 16 bytes into the section)
    const int *head_list;
    const long long *bits_before;
    long long units_per_head;   // work units (one wave each) per (layer, head)
    long long total_units;
    int *status;                // device status word of the request
};

// The same tensor (K or V) of several requests of a call in one launch, their workgroups one request
// after the other.
// All items take the same kernel (same plan; same layout class, see QuantArgs::dense).
constexpr int kQuantBatch = 12;     // (the argument block stays below 4 KB)
struct QuantBatch {
    QuantArgs item[kQuantBatch];
    unsigned start[kQuantBatch + 1];    // first workgroup of every item in the launch (set by the launcher)
    int n;
};

// The item a workgroup belongs to, and its number among the item's workgroups (the same in all lanes).
template <class Batch> __device__ __forceinline__ int batch_item(const Batch &b, unsigned &wg)
{
    int i = 0;
    while (i + 1 < b.n && blockIdx.x >= b.start[i + 1]) ++i;
    wg = blockIdx.x - b.start[i];
    return i;
}

// Geometry of one payload (all byte counts), shared by host code of compress / decompress.
struct Geometry {
    long long meta_k, meta_v, aux, codes_k, codes_v;
    long long aux_base;          // tables / directory part of the auxiliary section (before the anchors)
    long long code_tables;       // bytes of the coder's tables at the start of the auxiliary section (0, 512 or 2048)
    long long off_dir;           // the coder's directory
    long long off_widths, widths;    // the per-head width tables
    long long anchors_k, anchors_v, off_anchors_k, off_anchors_v;
    long long off_meta_k, off_meta_v, off_aux, off_codes_k, off_codes_v, total;
    long long chunks_k, chunks_v;
};

struct HeaderBytes { uint32_t w[32]; };

int launch_compress_tensor(int is_v, int bits, int group, int dtype, const QuantBatch &b, hipStream_t s);
int launch_decompress_tensor(int is_v, int bits, int group, int dtype, const QuantBatch &b, hipStream_t s);
// one translation unit per code width (kvc_quant.hip compiled with -DKVC_BITS=...)
#define KVC_DECLARE_QUANT(B)                                                                              \
    int launch_compress_bits##B(int is_v, int group, int dtype, const QuantBatch &b, hipStream_t s);     \
    int launch_decompress_bits##B(int is_v, int dtype, const QuantBatch &b, hipStream_t s);
KVC_DECLARE_QUANT(2) KVC_DECLARE_QUANT(3) KVC_DECLARE_QUANT(4) KVC_DECLARE_QUANT(8)
#undef KVC_DECLARE_QUANT
// Service work of one request before its tensors are compressed (see compress_prologue_kernel).
struct PrologueItem {
    uint32_t *payload;              // request payload base
    HeaderBytes header;
    long long pad_off[2], pad_words[2];     // zero padding: byte offset inside the payload, 32-bit words
    const uint32_t *aux_src;        // device image of the width tables, copied to payload + aux_off
    long long aux_off, aux_words;
    uint32_t *zero[2];              // coder scratch that starts from zero: histograms; ticket and scan state
    long long zero_words[2];
    unsigned long long *out_bytes;  // the request's size word
    unsigned long long total;
    int write_total;                // the size is known on the host (no coder, or an empty request)
    uint32_t *dir0;                 // empty request with the coder: the directory's only entry
    int *status;
};
constexpr int kPrologueBatch = 12;  // requests per launch (the argument block stays below 4 KB)
struct PrologueArgs {
    PrologueItem item[kPrologueBatch];
    int n;
};

// Header (and width table) check of one request before it is decompressed.
struct CheckItem {
    const uint32_t *payload;
    HeaderBytes expect;
    uint32_t mask;                  // bit i = compare header word i
    const uint8_t *tables, *plan_tables;    // width tables in the payload and their device image
    long long table_bytes;
    int *status;
};
constexpr int kCheckBatch = 20;
struct CheckArgs {
    CheckItem item[kCheckBatch];
    int n;
};

int launch_compress_prologue(const PrologueArgs &a, hipStream_t s);
int launch_decompress_prologue(const CheckArgs &a, hipStream_t s);
int launch_fill_u32(uint32_t *dst, uint32_t value, long long n, hipStream_t s);

// ---- lossless stage (codec 1) -----------------------------------------------------------

// Code tables of a request: one per tensor, or with per-head widths one per tensor and width
// (slot 4 * is_v + index of the width in 2, 3, 4, 8).
constexpr int kTableSlots = 8;

// Per-request scratch inside the caller's workspace (device memory).
struct CoderScratch {
    uint32_t *hist;             // [kTableSlots][256] sample histograms
    uint32_t *enc;              // [kTableSlots][256] code | length << 16
    uint16_t *lut;              // [kTableSlots][4096] decode table: symbol | length << 8
    unsigned long long *state;  // scan state, one word per encode workgroup (in launch order)
    uint32_t *ticket;           // work-order counter
};

// Chunks (= waves) per encoder workgroup.  One look-back per workgroup is the encoder's serial part,
// so the variants whose registers allow 512 threads (2- to 4-bit codes, groups of 32, the dense
// layout; not the V kernels with the transforms for bf16 rows or 3-bit codes) take eight chunks per workgroup; 8-bit
// chunks need twice the LDS and take two.  `transform`: the launch applies stage T.
constexpr int enc_waves(int bits, int group, int dtype, bool dense, bool is_v, bool transform)
{
    return bits == 8 ? 2 : (group == 32 && dense && !(is_v && transform && (dtype == DT_BF16 || bits == 3))) ? 8 : 4;
}

// One launch of the coder: a tensor, or with per-head widths the heads of one width of a tensor
// (q.head_list); the launches of a request follow each other in chunk order (K before V, widths
// ascending) and share the ticket counter and the scan state.
struct CoderArgs {
    QuantArgs q;                // tensor, meta, tokens, status ...
    uint8_t *payload;           // request payload base
    long long off_aux;          // the code tables (256 length bytes per slot)
    long long off_dir;          // the directory
    long long off_bodies;       // first chunk body (= K codes offset)
    long long capacity;         // payload bytes available
    long long chunks;           // chunks of this launch
    long long chunk_base;       // directory index of this launch's first chunk
    long long wg_base;          // scan-state index of this launch's first workgroup
    long long k_wgs;            // encode workgroups of all K launches
    long long total_wgs;        // encode workgroups of all launches of the request
    long long total_chunks;     // K and V together
    int is_v;
    int tab;                    // table slot of this launch
    int slots, slot_mask;       // table slots of the request's format (2 or 8) and the ones in use
    CoderScratch ws;
    unsigned long long *out_bytes;   // device: true payload size (written by the last workgroup)
};

// One launch of the coder for several requests of a call (the table kernels: blockIdx.y picks the
// request; encoder and decoder: the requests' workgroups one after the other).  All items are
// the same launch of their request (same tensor, width and kernel variant; see request_window).
constexpr int kCoderBatch = 8;      // (the argument block stays below 4 KB)
struct CoderBatch {
    CoderArgs item[kCoderBatch];
    unsigned start[kCoderBatch + 1];    // encoder and decoder: first workgroup of every item (set by the launcher)
    int n;
};
static_assert(sizeof(CoderBatch) <= 4000, "kernel arguments are limited to 4 KB");
static_assert(sizeof(QuantBatch) <= 4000, "kernel arguments are limited to 4 KB");

int launch_table_sample(int bits, int group, int dtype, const CoderBatch &b, hipStream_t s);
int launch_build_tables(const CoderBatch &b, hipStream_t s);
int launch_encode_section(int bits, int group, int dtype, const CoderBatch &b, hipStream_t s);
int launch_decode_prepare(const CoderBatch &b, hipStream_t s);
int launch_decode_section(int bits, int group, int dtype, const CoderBatch &b, hipStream_t s);
// one translation unit per code width (kvc_huff_enc.hip / kvc_huff_dec.hip compiled with -DKVC_BITS=...)
#define KVC_DECLARE_CODER(B)                                                                  \
    int launch_encode_bits##B(int group, int dtype, const CoderBatch &b, hipStream_t s);      \
    int launch_decode_bits##B(int dtype, const CoderBatch &b, hipStream_t s);
KVC_DECLARE_CODER(2) KVC_DECLARE_CODER(3) KVC_DECLARE_CODER(4) KVC_DECLARE_CODER(8)
#undef KVC_DECLARE_CODER

}  // namespace kvc
