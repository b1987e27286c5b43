// Lossless stage, decoder: one wave per chunk; body -> LDS, every lane decodes one sub-block with a
// 4096-entry table, the packed rows are rebuilt in LDS and dequantized from there.  Compiled once per
// code width (-DKVC_BITS=2, 3, 4 or 8).  See kvc_huff.h.

#include "kvc_huff.h"

#ifndef KVC_BITS
#error "compile with -DKVC_BITS=2, 3, 4 or 8"
#endif

namespace kvc {

// ---- decoder ---------------------------------------------------------------------------------

struct BitReader {
    unsigned long long window;   // upcoming bits, left aligned
    int avail;
    const uint32_t *next;        // next word (LDS)
    const uint32_t *last;        // last readable word
};

__device__ __forceinline__ void refill(BitReader &br)
{
    if (br.avail <= 32) {
        br.window |= (unsigned long long)(*br.next) << (32 - br.avail);
        br.avail += 32;
        if (br.next < br.last) ++br.next;
    }
}

template <int W> __device__ __forceinline__ void decode_half(uint32_t *sym, const uint16_t *lut, int half, BitReader &br)
{
#pragma unroll
    for (int k = 0; k < W / 2; ++k) {
        uint32_t w = 0;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const uint32_t e = lut[(uint32_t)(br.window >> 52)];
            const uint32_t len = e >> 8;
            w = __builtin_amdgcn_alignbit(e, w, 8);      // symbol byte enters at the top; after 4 symbols the first is lowest
            br.window <<= len;
            br.avail -= (int)len;
            if (b & 1) refill(br);
        }
        sym[half * (W / 2) + k] = w;
    }
}

// metadata of the 32 rows starting at chunk row `r0`: K = the lane's 8 channels of that token
// block (two 16-byte loads), V = the lane's group in each of its 8 rows
__device__ __forceinline__ void load_meta_k(const QuantArgs &q, const ChunkPos &c, int r0, u32x4 &m0, u32x4 &m1)
{
    const int col = lane_id() & 15;
    const long long nb = (q.tokens + q.group - 1) / q.group;
    const u32x4 *m = (const u32x4 *)(q.meta + ((c.lh * nb + (c.row0 + r0) / q.group) * kDim + col * 8) * 4);
    m0 = m[0];
    m1 = m[1];
}

__device__ __forceinline__ void load_meta_v(const QuantArgs &q, const ChunkPos &c, int r0, uint32_t mv[8])
{
    const int lane = lane_id(), col = lane & 15, rsub = lane >> 4;
    const int ng = kDim / q.group, shift = q.group == 32 ? 2 : (q.group == 64 ? 3 : 4);
    const uint32_t *m = (const uint32_t *)q.meta + (c.lh * q.tokens + c.row0 + r0) * ng + (col >> shift);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int r = 4 * i + rsub;
        mv[i] = m[(r0 + r < c.rows ? r : 0) * ng];
    }
}

// Dequantize a decoded chunk from the wave's LDS region and store its rows; the metadata of a
// pass is in flight one pass ahead.  meta0 / meta1 (K) or metav (V): the first pass's metadata.
// first_anchor (delta transform): the first pass's anchor row.
template <int BITS, int DT, bool IS_V, bool DENSE, int TR>
__device__ __forceinline__ void dequant_chunk(const CoderArgs &a, const ChunkPos &c, uint8_t *lds, const u32x4 &meta0,
                                              const u32x4 &meta1, const uint32_t metav[8], const u32x4 &first_anchor,
                                              int first_blocks, bool &bad)
{
    using Dec = DecGeom<BITS>;
    const uint16_t *anchors = TR >= 2 ? head_anchors(a.q.anchors, c.lh, a.q.tokens, a.q.anchor_shift) : nullptr;
    constexpr bool one_anchor = TR == 2;
    u32x4 anchor = first_anchor, anchor_next = first_anchor;
    u32x4 mk0 = meta0, mk1 = meta1;
    uint32_t mv[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) mv[i] = metav[i];
    // paged destination: the block-table entries of a pass are in flight one pass ahead as well
    const bool paged = !DENSE && a.q.x.block_table != nullptr && a.q.x.bt_wave;
    int blocks = first_blocks, blocks_next = first_blocks;
#pragma unroll 1
    for (int p = 0; p < kChunkRows / kPassRows; ++p) {
        if (p * kPassRows >= c.rows) break;
        float scale[8], zero[8];
        const bool clamp = IS_V ? v_meta_floats<BITS, DT>(mv, scale, zero) : k_meta_floats<BITS, DT>(mk0, mk1, scale, zero);
        if ((p + 1) * kPassRows < c.rows) {
            if (!IS_V) load_meta_k(a.q, c, (p + 1) * kPassRows, mk0, mk1);
            else load_meta_v(a.q, c, (p + 1) * kPassRows, mv);
            if (one_anchor) anchor_next = load_anchor(anchors, a.q.anchor_shift, c.row0 + (p + 1) * kPassRows);
            if (paged) blocks_next = pass_blocks(a.q.x, c.row0 + (p + 1) * kPassRows, c.row0 + c.rows);
        }
        PassFetch f;
        pass_fetch<BITS, DENSE, Dec::kLayout>(f, lds, a.q.x, c.head_off, c.row0 + p * kPassRows, c.rows - p * kPassRows, p * kPassRows,
                                              paged, blocks);
        dequant_pass<BITS, DT, IS_V, DENSE, TR>(f, scale, zero, clamp, a.q.x, c.head_off, c.row0 + p * kPassRows,
                                                c.rows - p * kPassRows, bad, anchors, a.q.anchor_shift,
                                                one_anchor ? &anchor : nullptr);
        anchor = anchor_next;
        blocks = blocks_next;
    }
}

// TR: the inverse of stage T that the launch applies (see dequant_pass_rows).  One kernel per
// transform: in one kernel, every path pays for the registers of the most expensive one (the anchors
// of short runs, the rotation) with its fourth wave per SIMD.
template <int BITS, int DT, bool IS_V, bool DENSE, int TR>
__global__ __launch_bounds__(ChunkGeom<BITS>::kDecWaves * 64) void decode_kernel(CoderBatch batch)
{
    using Geo = ChunkGeom<BITS>;
    using Dec = DecGeom<BITS>;
    constexpr int W = Geo::kWords, NW = Geo::kDecWaves;
    unsigned wg;
    const CoderArgs &a = batch.item[batch_item(batch, wg)];
    __shared__ __attribute__((aligned(16))) uint8_t lds_all[NW * Dec::kLds];
    __shared__ uint16_t lut[4096];

    const int tid = threadIdx.x, wave = tid >> 6, lane = lane_id();      // (kept per lane: as a scalar it costs this kernel its fourth wave per SIMD)
    long long chunk = (long long)wg * NW + wave;
    const bool live = chunk < a.chunks;
    if (!DENSE && live && a.q.head_minor) {
        // destination with the heads of a token next to each other: neighbouring waves take the same
        // rows of neighbouring heads, so that what they store together is contiguous
        const long long cph = (a.q.tokens + kChunkRows - 1) / kChunkRows;
        const long long t = chunk / a.q.heads, h = chunk - t * a.q.heads;
        const long long l = t / cph, cb = t - l * cph;
        chunk = (l * a.q.heads + h) * cph + cb;
    }
    uint8_t *lds = lds_all + wave * Dec::kLds;
    // Register headroom.  On this GPU a 64-bit shift whose count sits in the last VGPR of the
    // wave's allocation shifts by the lane number instead, now and then, once three or four such
    // waves share a SIMD (LLVM knows and avoids the fault for gfx90a only).  A build of this
    // kernel that needed exactly 112 registers kept a code length in v111 for `window <<= len`
    // and decoded the last two symbols of a sub-block wrongly in one wave of seven at full size.
    // Naming a higher register keeps the allocation (128: still four waves per SIMD) above every
    // register the code touches; the build checks the assembly of all kernels for the pattern.
    if (BITS == 8) asm volatile("" ::: "v255");        // (the 8-bit kernel keeps more rows in registers: two waves per SIMD either way)
    else asm volatile("" ::: "v127");

    // Round trip 1: the chunk's two directory entries and the status word, with the decode
    // table right behind them.
    unsigned long long d0 = 0, d1 = 0;
    int st = 0;
    if (live) {
        const uint32_t *dir = (const uint32_t *)(a.payload + a.off_dir) + a.chunk_base + chunk;
        d0 = dir[0];
        d1 = dir[1];
        st = *a.q.status;
    }
    constexpr int LUTN = 512 / (NW * 64);
    u32x4 lutv[LUTN];
    {
        const u32x4 *src = (const u32x4 *)(a.ws.lut + 4096 * a.tab);
#pragma unroll
        for (int i = 0; i < LUTN; ++i) lutv[i] = src[tid + i * NW * 64];
    }
    ChunkPos c = chunk_pos(a.q, live ? chunk : 0);
    const uint32_t raw_bytes = (uint32_t)c.rows * Geo::kRowBytes;
    const unsigned long long size = (d1 - d0) * 16;
    bool ok = live && !(st & (KVC_DEV_BAD_HEADER | KVC_DEV_BAD_TABLE));
    if (ok && (d1 < d0 || size > raw_bytes || (long long)(a.off_bodies + d1 * 16) > a.capacity ||
               (size != raw_bytes && size < 2 * kSubs + 16))) {
        if (lane == 0) atomicOr(a.q.status, KVC_DEV_BAD_CHUNK);
        ok = false;
    }
    // Round trip 2: the body (into registers) and the metadata of the first pass.
    constexpr int NB = 2 * BITS;                       // 16-byte pieces per lane of a full raw chunk
    u32x4 bodyv[NB];
    u32x4 meta0 = {0, 0, 0, 0}, meta1 = {0, 0, 0, 0};
    uint32_t metav[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    u32x4 anchor0 = {0, 0, 0, 0};                      // delta transform: the first pass's anchor row
    int blocks0 = 0;                                   // paged destination: the first pass's block-table entries (pass_blocks)
    if (ok) {
        const uint8_t *body = a.payload + a.off_bodies + d0 * 16;
#pragma unroll
        for (int k = 0; k < NB; ++k) {
            const uint32_t o = (k * 64 + lane) * 16;
            if (o < size) bodyv[k] = __builtin_nontemporal_load((const u32x4 *)(body + o));
        }
        if (!IS_V) load_meta_k(a.q, c, 0, meta0, meta1);
        else load_meta_v(a.q, c, 0, metav);
        if (!DENSE && a.q.x.block_table != nullptr && a.q.x.bt_wave) blocks0 = pass_blocks(a.q.x, c.row0, c.row0 + c.rows);
        if (TR == 2)
            anchor0 = load_anchor(head_anchors(a.q.anchors, c.lh, a.q.tokens, a.q.anchor_shift), a.q.anchor_shift, c.row0);
    }
#pragma unroll
    for (int i = 0; i < LUTN; ++i) ((u32x4 *)lut)[tid + i * NW * 64] = lutv[i];
    __syncthreads();
    if (!ok) return;

    if (size == raw_bytes) {
        // stored raw: scatter the packed rows into the sub-block layout
#pragma unroll
        for (int k = 0; k < NB; ++k) {
            const uint32_t o = (k * 64 + lane) * 16;
            if (o < raw_bytes) {
                const uint32_t sub = o / Geo::kSubBytes, in = o - sub * Geo::kSubBytes;
                *(u32x4 *)Dec::piece_ptr(lds, sub, in / 16) = bodyv[k];
            }
        }
        wave_sync();
    } else {
#pragma unroll
        for (int k = 0; k < NB; ++k) {
            const uint32_t o = (k * 64 + lane) * 16;
            if (o < size) *(u32x4 *)(lds + o) = bodyv[k];
        }
        wave_sync();
        const uint32_t bits = ((const uint16_t *)lds)[lane];
        const uint32_t incl = wave_inclusive_sum(bits);
        const uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
        if (((2 * kSubs + 4 * ((total + 31) / 32) + 15) & ~15u) != size) {
            if (lane == 0) atomicOr(a.q.status, KVC_DEV_BAD_CHUNK);
            return;
        }
        const uint32_t start = incl - bits;
        const uint32_t *words = (const uint32_t *)(lds + 2 * kSubs);
        BitReader br;
        br.last = (const uint32_t *)(lds + size) - 1;
        const uint32_t *p = words + (start >> 5);
        p = p < br.last ? p : br.last;
        const uint32_t w0 = *p;
        p = p < br.last ? p + 1 : p;
        const uint32_t w1 = *p;
        p = p < br.last ? p + 1 : p;
        br.window = (((unsigned long long)w0 << 32) | w1) << (start & 31);
        br.avail = 64 - (int)(start & 31);
        br.next = p;
        uint32_t sym[W];
#pragma unroll
        for (int k = 0; k < W; ++k) sym[k] = 0;
        const int have = min(max(c.rows - 2 * lane, 0), 2);
        if (have > 0) decode_half<W>(sym, lut, 0, br);
        if (have > 1) decode_half<W>(sym, lut, 1, br);
        wave_sync();                                   // all lanes are done reading the coded words
        {
#pragma unroll
            for (int q = 0; q < W / 4; ++q) {
                u32x4 v;
                v[0] = sym[4 * q]; v[1] = sym[4 * q + 1]; v[2] = sym[4 * q + 2]; v[3] = sym[4 * q + 3];
                *(u32x4 *)Dec::piece_ptr(lds, lane, q) = v;
            }
        }
        wave_sync();
    }

    // dequantize the rows from LDS
    bool bad = false;
    dequant_chunk<BITS, DT, IS_V, DENSE, TR>(a, c, lds, meta0, meta1, metav, anchor0, blocks0, bad);
    if (bad) atomicOr(a.q.status, KVC_DEV_BAD_BLOCK);
}

// ---- launchers ----------------------------------------------------------------------------------

template <int BITS, int DT, bool IS_V> static int decode_launch(const CoderBatch &b, hipStream_t s)
{
    constexpr int NW = ChunkGeom<BITS>::kDecWaves;
    const CoderArgs &a = b.item[0];
    CoderBatch placed = b;
    unsigned need = 0;
    for (int i = 0; i < b.n; ++i) {
        placed.start[i] = need;
        need += (unsigned)((b.item[i].chunks + NW - 1) / NW);
    }
    placed.start[b.n] = need;
    if (need == 0) return KVC_OK;
    const dim3 grid(need), block(NW * 64);
    const int tr = a.q.rotate ? 1 : !a.q.anchors ? 0 : a.q.anchor_shift >= 5 ? 2 : 3;
#define KVC_DECODE(D, T) hipLaunchKernelGGL((decode_kernel<BITS, DT, IS_V, D, T>), grid, block, 0, s, placed)
    if (a.q.dense) {
        if (tr == 0) KVC_DECODE(true, 0); else if (tr == 1) KVC_DECODE(true, 1); else if (tr == 2) KVC_DECODE(true, 2); else KVC_DECODE(true, 3);
    } else {
        if (tr == 0) KVC_DECODE(false, 0); else if (tr == 1) KVC_DECODE(false, 1); else if (tr == 2) KVC_DECODE(false, 2); else KVC_DECODE(false, 3);
    }
#undef KVC_DECODE
    return launched();
}

#define KVC_PASTE2(a, b) a##b
#define KVC_PASTE(a, b) KVC_PASTE2(a, b)

int KVC_PASTE(launch_decode_bits, KVC_BITS)(int dtype, const CoderBatch &a, hipStream_t s)
{
    if (a.item[0].is_v) return dtype == DT_F16 ? decode_launch<KVC_BITS, DT_F16, true>(a, s) : decode_launch<KVC_BITS, DT_BF16, true>(a, s);
    return dtype == DT_F16 ? decode_launch<KVC_BITS, DT_F16, false>(a, s) : decode_launch<KVC_BITS, DT_BF16, false>(a, s);
}

}  // namespace kvc
