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

// Geometry of one payload (all byte counts), shared by host code of compress / decompress.
struct Geometry {
    long long meta_k, meta_v, aux, codes_k, codes_v;
    long long aux_base;          // tables / directory part of the auxiliary section (before the anchors)
    long long anchors_k, anchors_v, off_anchors_k, off_anchors_v;
    long long off_meta_k, off_meta_v, off_aux, off_codes_k, off_codes_v, total;
    long long chunks_k, chunks_v;
};

struct HeaderBytes { uint32_t w[32]; };

int launch_compress_tensor(int is_v, int bits, int group, int dtype, const QuantArgs &a, hipStream_t s);
int launch_decompress_tensor(int is_v, int bits, int group, int dtype, const QuantArgs &a, hipStream_t s);
int launch_write_header(uint8_t *dst, const HeaderBytes &h, hipStream_t s);
// Compare a payload header with the one the plan implies; `mask` bit i = compare word i.
int launch_check_header(const uint8_t *hdr, const HeaderBytes &expect, uint32_t mask, int *status,
                        hipStream_t s);
int launch_fill_u32(uint32_t *dst, uint32_t value, long long n, hipStream_t s);
int launch_check_bytes(const uint8_t *a, const uint8_t *b, long long n, int *status, hipStream_t s);

// ---- lossless stage (codec 1) -----------------------------------------------------------

// Per-request scratch inside the caller's workspace (device memory).
struct CoderScratch {
    uint32_t *hist;             // [2][256] sample histograms (K, V)
    uint32_t *enc;              // [2][256] code | length << 16
    uint16_t *lut;              // [2][4096] decode table: symbol | length << 8
    unsigned long long *state;  // scan state, one word per encode workgroup (K then V)
    uint32_t *ticket;           // work-order counter
};

struct CoderArgs {
    QuantArgs q;                // tensor, meta, tokens, status ...
    uint8_t *payload;           // request payload base
    long long off_aux;          // tables (2 x 256 length bytes) then directory
    long long off_bodies;       // first chunk body (= K codes offset)
    long long capacity;         // payload bytes available
    long long chunks;           // chunks in this section
    long long chunk_base;       // directory index of this section's first chunk
    long long wg_base;          // scan-state index of this section's first workgroup
    long long total_wgs;        // encode workgroups of K and V together
    long long total_chunks;     // K and V together
    int is_v;
    CoderScratch ws;
    unsigned long long *out_bytes;   // device: true payload size (written by the last workgroup)
};

int launch_coder_tables(int bits_k, int bits_v, int group_k, int group_v, int dtype,
                        const CoderArgs &k, const CoderArgs &v, hipStream_t s);
int launch_encode_section(int bits, int group, int dtype, const CoderArgs &a, hipStream_t s);
int launch_decode_prepare(const CoderArgs &k, hipStream_t s);
int launch_decode_section(int bits, int group, int dtype, const CoderArgs &a, hipStream_t s);

}  // namespace kvc
