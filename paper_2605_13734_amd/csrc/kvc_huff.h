// Shared device code of the lossless stage (codec C of the pipeline, KVServe section 5.1) fused
// with the quantizer: canonical, length-limited Huffman coding of the packed code bytes.
//
// Format (per section K or V): chunks of 128 token rows of one head; a chunk body is
// 64 x u16 sub-block bit counts (a sub-block = 2 rows), then the code words, most
// significant bit first in 32-bit little-endian words, sub-blocks back to back, padded
// to 16 bytes -- or the raw packed bytes when that is not smaller.  Bodies are stored
// back to back; a directory of running offsets (16-byte units) locates them.
//
// One wave owns one chunk: it quantizes the chunk into LDS, every lane then codes one
// sub-block, and the body is copied to its final place, which comes from a single-pass
// prefix sum over workgroups (ticket order + look-back on a state word per workgroup).
// Decoding mirrors it: body -> LDS, every lane decodes one sub-block with a 4096-entry
// table, the packed rows are rebuilt in LDS and dequantized from there.
//
// The kernels live in three sources: kvc_huff_tables.hip (table sample, code construction,
// decode tables), kvc_huff_enc.hip and kvc_huff_dec.hip (compiled once per code width, KVC_BITS).
#pragma once

#include "kvc_internal.h"
#include "kvc_tile.h"
#include "../../include/kvc.h"

namespace kvc {

// Scan state of a workgroup: bits 63:62 = 2 once its inclusive prefix (bits 0..39) is known.
// Before that, every wave adds its chunk's size to bits 0..39 and its share of kAggComplete to
// the arrival count in bits 40..47; the sum of sizes is the workgroup's aggregate once the
// count is complete.  Sizes and prefixes are in 16-byte units.
constexpr unsigned long long kFlagPrefix = 2ull << 62, kValueMask = (1ull << 40) - 1;
constexpr int kAggShift = 40, kAggComplete = 8;
constexpr int kSpinLimit = 1 << 20;

template <int BITS> struct ChunkGeom {
    static constexpr int kRowBytes = 16 * BITS;            // packed bytes of one token row
    static constexpr int kSubBytes = 2 * kRowBytes;        // one sub-block
    static constexpr int kSubStride = kSubBytes + 16;      // LDS stride (bank spread, 16-byte aligned)
    static constexpr int kWords = kSubBytes / 4;           // words a lane holds for its sub-block
    static constexpr int kLds = kSubs * kSubStride;        // LDS bytes per wave
    static constexpr int kDecWaves = BITS == 8 ? 2 : 4;    // decoder: waves per workgroup (they share the 8 KB table)
};

// The decoder's LDS layout of a chunk.  4-bit codes: sub-blocks without padding, pieces rotated
// (fetch_codes, LAYOUT 2), 8 KB per wave, so that four workgroups of four waves and their 8 KB
// tables fill a compute unit's 160 KB exactly.  Other widths: the encoder's padded layout.
template <int BITS> struct DecGeom {
    static constexpr bool kRotated = BITS == 4;
    static constexpr int kLayout = kRotated ? 2 : 1;
    static constexpr int kStride = kRotated ? ChunkGeom<BITS>::kSubBytes : ChunkGeom<BITS>::kSubStride;
    static constexpr int kLds = kSubs * kStride;
    // address of 16-byte piece `piece` of sub-block `sub`
    static __device__ __forceinline__ uint8_t *piece_ptr(uint8_t *lds, uint32_t sub, uint32_t piece)
    {
        if (kRotated) return lds + sub * kStride + (((piece + sub) & 7u) << 4);
        return lds + sub * kStride + piece * 16;
    }
};

// ---- chunk <-> LDS -------------------------------------------------------------------------

template <int BITS> __device__ __forceinline__ uint8_t *lds_row(uint8_t *lds, int r)
{
    return code_row<BITS, true>(lds, r);
}

struct ChunkPos {
    long long lh, cb, head_off, row0;
    int rows;
};

__device__ __forceinline__ ChunkPos chunk_pos(const QuantArgs &a, long long chunk)
{
    ChunkPos c;
    const long long cph = (a.tokens + kChunkRows - 1) / kChunkRows;
    const long long slot = chunk / cph;                 // with per-head widths: the slot-th head of this launch's width
    c.lh = a.head_list ? a.head_list[slot] : slot;
    c.cb = chunk - slot * cph;
    const long long l = c.lh / a.heads, h = c.lh - l * a.heads;
    c.head_off = l * a.x.stride_layer + h * a.x.stride_head;
    c.row0 = c.cb * kChunkRows;
    const long long left = a.tokens - c.row0;
    c.rows = left < kChunkRows ? (int)left : kChunkRows;
    return c;
}

// Quantize and pack the chunk's rows into the wave's LDS region (sub-block layout) and,
// when `write_meta`, store the group metadata to the payload.  K group parameters are
// exchanged through the 16 padding bytes that follow each sub-block.
// XF = false leaves the code of stage T out (for launches that have no transform): in one kernel
// with the plain path it costs the plain path its registers, most of all for token blocks of 64
// and 128 rows.
template <int BITS, int G, int DT, bool IS_V> struct UnitGeom {
    static constexpr int kRows = IS_V ? kPassRows : G;             // rows of a unit: a pass, or a K token block
    static constexpr int kPasses = kRows / kPassRows, kUnits = kChunkRows / kRows;
};

// One unit of a chunk: the rows [u * kRows, ...) of the chunk are loaded, transformed, quantized and
// packed; their codes go to the rows lds_row0 ... of the LDS region.
template <int BITS, int G, int DT, bool IS_V, bool DENSE, bool XF = true>
__device__ __forceinline__ void quantize_unit(const QuantArgs &a, const ChunkPos &c, int u, uint8_t *lds, int lds_row0,
                                              bool write_meta, bool &bad, bool have_blocks = false, const int *blocks = nullptr)
{
    constexpr int RU = UnitGeom<BITS, G, DT, IS_V>::kRows, PU = UnitGeom<BITS, G, DT, IS_V>::kPasses;
    const long long row0 = c.row0 + u * RU;
    u32x4 raw[PU * 8];
#pragma unroll
    for (int p = 0; p < PU; ++p)
        load_pass<DENSE>(a.x, c.head_off, row0 + p * kPassRows, a.tokens, raw + p * 8, bad, have_blocks, have_blocks ? blocks[p] : 0);
    if (XF && a.rotate) rotate_rows<DT, PU * 8>(raw);
    if (XF && a.anchors)
        delta_rows<DT, DENSE, PU * 8>(a.x, c.head_off, row0, a.tokens, a.anchor_shift,
                                      head_anchors(a.anchors, c.lh, a.tokens, a.anchor_shift), write_meta, raw, bad);
    if (!IS_V) {
        const long long nb = (a.tokens + G - 1) / G;
        KParams kp;
        uint8_t *meta_block = write_meta ? a.meta + (c.lh * nb + row0 / G) * (kDim * 4) : nullptr;
        k_group_params<BITS, DT, PU * 8, ChunkGeom<BITS>::kSubStride>(raw, lds + ChunkGeom<BITS>::kSubBytes, meta_block, kp);
        forget_unpacked<DT, PU * 8>(raw);
        k_emit<BITS, DT, PU, true>(raw, kp, code_row<BITS, true>(lds, lds_row0), c.rows - u * RU);
    } else {
        constexpr int NG = kDim / G;
        VParams vp;
        v_pass_params<BITS, G, DT>(raw, vp);
        forget_unpacked<DT, PU * 8>(raw);
        uint32_t *meta = write_meta ? (uint32_t *)a.meta + (c.lh * a.tokens + row0) * NG : nullptr;
        v_emit<BITS, G, DT, true>(raw, vp, code_row<BITS, true>(lds, lds_row0), c.rows - u * RU, meta);
    }
}

template <int BITS, int G, int DT, bool IS_V, bool DENSE, bool XF = true>
__device__ __forceinline__ void quantize_chunk(const QuantArgs &a, const ChunkPos &c, uint8_t *lds, bool write_meta,
                                               bool &bad)
{
    constexpr int RU = UnitGeom<BITS, G, DT, IS_V>::kRows, NU = UnitGeom<BITS, G, DT, IS_V>::kUnits;
    constexpr int PU = UnitGeom<BITS, G, DT, IS_V>::kPasses;
    // paged source: the block-table entries of a unit's passes are requested one unit ahead
    const bool paged = !DENSE && a.x.block_table != nullptr && a.x.bt_wave;
    int blocks[PU], blocks_next[PU];
#pragma unroll
    for (int p = 0; p < PU; ++p) blocks[p] = blocks_next[p] = paged ? pass_blocks(a.x, c.row0 + p * kPassRows, a.tokens) : 0;
#pragma unroll 1
    for (int u = 0; u < NU; ++u) {
        if (u * RU >= c.rows) break;
        if (paged && (u + 1) * RU < c.rows) {
#pragma unroll
            for (int p = 0; p < PU; ++p) blocks_next[p] = pass_blocks(a.x, c.row0 + (u + 1) * RU + p * kPassRows, a.tokens);
        }
        quantize_unit<BITS, G, DT, IS_V, DENSE, XF>(a, c, u, lds, u * RU, write_meta, bad, paged, blocks);
#pragma unroll
        for (int p = 0; p < PU; ++p) blocks[p] = blocks_next[p];
    }
}

// The lane's sub-block (rows 2*lane, 2*lane+1) from LDS into registers.
template <int BITS> __device__ __forceinline__ void load_sub(const uint8_t *lds, uint32_t *sym)
{
    constexpr int W = ChunkGeom<BITS>::kWords;
    const u32x4 *p = (const u32x4 *)(lds + lane_id() * ChunkGeom<BITS>::kSubStride);
#pragma unroll
    for (int k = 0; k < W / 4; ++k) {
        u32x4 v = p[k];
        sym[4 * k] = v[0]; sym[4 * k + 1] = v[1]; sym[4 * k + 2] = v[2]; sym[4 * k + 3] = v[3];
    }
}

template <int BITS> __device__ __forceinline__ void store_sub(uint8_t *lds, const uint32_t *sym)
{
    constexpr int W = ChunkGeom<BITS>::kWords;
    u32x4 *p = (u32x4 *)(lds + lane_id() * ChunkGeom<BITS>::kSubStride);
#pragma unroll
    for (int k = 0; k < W / 4; ++k) {
        u32x4 v;
        v[0] = sym[4 * k]; v[1] = sym[4 * k + 1]; v[2] = sym[4 * k + 2]; v[3] = sym[4 * k + 3];
        p[k] = v;
    }
}

// inclusive prefix sum over the 64 lanes
__device__ __forceinline__ uint32_t wave_inclusive_sum(uint32_t v)
{
    const int lane = lane_id();
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint32_t o = (uint32_t)__builtin_amdgcn_ds_bpermute((lane - d) << 2, (int)v);
        if (lane >= d) v += o;
    }
    return v;
}

static inline int launched() { return hipGetLastError() == hipSuccess ? KVC_OK : KVC_ERR_DEVICE; }

}  // namespace kvc
