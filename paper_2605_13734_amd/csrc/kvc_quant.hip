// Codec-free kernels: quantize + pack (compress) and unpack + dequantize (decompress) one
// tensor of one request straight between the KV layout and the payload sections.
// One wave per work unit, four units per workgroup, no barriers.
//   K compress unit   = one token block of G rows x 128 channels (all 128 per-channel groups)
//   other units       = 32 token rows
// Stage Q of the pipeline (KVServe section 5.1); memory-bound, so no matrix cores.
// Compiled once per code width (-DKVC_BITS=2, 3, 4 or 8).

#include "kvc_quant.h"

#ifndef KVC_BITS
#error "compile with -DKVC_BITS=2, 3, 4 or 8"
#endif

namespace kvc {

// ---- K: groups along tokens, one per channel ------------------------------------------------

// XF = false leaves the code of stage T out (for launches without a transform): sharing a kernel
// with it doubles the registers of the plain path for token blocks of 64 and 128 rows.
template <int BITS, int G, int DT, bool DENSE, bool XF>
__global__ __launch_bounds__(256) void compress_k_kernel(QuantBatch b)
{
    unsigned wg;
    const QuantArgs &a = b.item[batch_item(b, wg)];
    __shared__ __attribute__((aligned(16))) float xch_all[4 * kXchFloats];
    UnitPos u;
    if (!unit_pos(a, wg, u)) return;
    constexpr int P = G / kPassRows;
    const long long row0 = u.blk * G;
    bool bad = false;
    u32x4 raw[P * 8];
#pragma unroll
    for (int p = 0; p < P; ++p) load_pass<DENSE>(a.x, u.head_off, row0 + p * kPassRows, a.tokens, raw + p * 8, bad);
    if (XF && a.rotate) rotate_rows<DT, P * 8>(raw);
    if (XF && a.anchors)
        delta_rows<DT, DENSE, P * 8>(a.x, u.head_off, row0, a.tokens, a.anchor_shift,
                                     head_anchors(a.anchors, u.lh, a.tokens, a.anchor_shift), true, raw, bad);
    KParams kp;
    uint8_t *meta_block = a.meta + (u.lh * a.units_per_head + u.blk) * (kDim * 4);
    k_group_params<BITS, DT, P * 8, 16>(raw, (uint8_t *)(xch_all + wave_id() * kXchFloats), meta_block, kp);
    forget_unpacked<DT, P * 8>(raw);
    uint8_t *codes = head_codes<BITS>(a, u.lh) + row0 * (16 * BITS);
    const long long left = a.tokens - row0;
    k_emit<BITS, DT, P, false>(raw, kp, codes, left < G ? (int)left : G);
    report(a.status, bad);
}

template <int BITS, int DT, bool DENSE>
__global__ __launch_bounds__(256) void decompress_k_kernel(QuantBatch b)
{
    unsigned wg;
    const QuantArgs &a = b.item[batch_item(b, wg)];
    UnitPos u;
    if (!unit_pos(a, wg, u)) return;
    if (*a.status & KVC_DEV_BAD_HEADER) return;
    const int col = lane_id() & 15;
    const long long row0 = u.blk * kPassRows;
    const long long tb = row0 / a.group, nb = (a.tokens + a.group - 1) / a.group;
    const u32x4 *m = (const u32x4 *)(a.meta + ((u.lh * nb + tb) * kDim + col * 8) * 4);
    const u32x4 m0 = m[0], m1 = m[1];
    uint8_t *codes = head_codes<BITS>(a, u.lh) + row0 * (16 * BITS);
    const long long left = a.tokens - row0;
    const int rows = left < kPassRows ? (int)left : kPassRows;
    PassFetch f;
    pass_fetch<BITS, DENSE, 0>(f, codes, a.x, u.head_off, row0, rows);
    float scale[8], zero[8];
    const bool clamp = k_meta_floats<BITS, DT>(m0, m1, scale, zero);
    bool bad = false;
    dequant_pass_any<BITS, DT, false, DENSE>(f, scale, zero, clamp, a.x, u.head_off, row0, rows, bad, a.rotate != 0,
                                             a.anchors ? head_anchors(a.anchors, u.lh, a.tokens, a.anchor_shift) : nullptr,
                                             a.anchor_shift);
    report(a.status, bad);
}

// ---- V: groups along channels, one set per token -----------------------------------------------

template <int BITS, int GV, int DT, bool DENSE>
__global__ __launch_bounds__(256) void compress_v_kernel(QuantBatch b)
{
    unsigned wg;
    const QuantArgs &a = b.item[batch_item(b, wg)];
    UnitPos u;
    if (!unit_pos(a, wg, u)) return;
    constexpr int NG = kDim / GV;
    const long long row0 = u.blk * kPassRows;
    bool bad = false;
    u32x4 raw[8];
    load_pass<DENSE>(a.x, u.head_off, row0, a.tokens, raw, bad);
    if (a.rotate) rotate_rows<DT, 8>(raw);
    if (a.anchors)
        delta_rows<DT, DENSE, 8>(a.x, u.head_off, row0, a.tokens, a.anchor_shift,
                                 head_anchors(a.anchors, u.lh, a.tokens, a.anchor_shift), true, raw, bad);
    VParams vp;
    v_pass_params<BITS, GV, DT>(raw, vp);
    forget_unpacked<DT, 8>(raw);
    uint8_t *codes = head_codes<BITS>(a, u.lh) + row0 * (16 * BITS);
    uint32_t *meta = (uint32_t *)a.meta + (u.lh * a.tokens + row0) * NG;
    const long long left = a.tokens - row0;
    v_emit<BITS, GV, DT, false>(raw, vp, codes, left < kPassRows ? (int)left : kPassRows, meta);
    report(a.status, bad);
}

template <int BITS, int DT, bool DENSE>
__global__ __launch_bounds__(256) void decompress_v_kernel(QuantBatch b)
{
    unsigned wg;
    const QuantArgs &a = b.item[batch_item(b, wg)];
    UnitPos u;
    if (!unit_pos(a, wg, u)) return;
    if (*a.status & KVC_DEV_BAD_HEADER) return;
    const int lane = lane_id(), col = lane & 15, rsub = lane >> 4;
    const long long row0 = u.blk * kPassRows;
    const int lanes_shift = a.group == 32 ? 2 : (a.group == 64 ? 3 : 4), ng = kDim / a.group;
    const uint32_t *meta = (const uint32_t *)a.meta + (u.lh * a.tokens + row0) * ng + (col >> lanes_shift);
    const long long left = a.tokens - row0;
    const int rows = left < kPassRows ? (int)left : kPassRows;
    uint32_t mw[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) mw[i] = meta[(4 * i + rsub < rows ? 4 * i + rsub : 0) * ng];
    uint8_t *codes = head_codes<BITS>(a, u.lh) + row0 * (16 * BITS);
    PassFetch f;
    pass_fetch<BITS, DENSE, 0>(f, codes, a.x, u.head_off, row0, rows);
    float scale[8], zero[8];
    const bool clamp = v_meta_floats<BITS, DT>(mw, scale, zero);
    bool bad = false;
    dequant_pass_any<BITS, DT, true, DENSE>(f, scale, zero, clamp, a.x, u.head_off, row0, rows, bad, a.rotate != 0,
                                            a.anchors ? head_anchors(a.anchors, u.lh, a.tokens, a.anchor_shift) : nullptr,
                                            a.anchor_shift);
    report(a.status, bad);
}

// ---- launchers ----------------------------------------------------------------------------------

template <int BITS, int DT, bool DENSE> static int compress_bits_dt(int is_v, int group, const QuantBatch &b, hipStream_t s)
{
    const QuantArgs &a = b.item[0];
    if (!is_v) {
        const bool xf = a.rotate || a.anchors;
        switch (group) {
        case 32: KVC_LAUNCH((compress_k_kernel<BITS, 32, DT, DENSE, true>), b, s);
        case 64:
            if (xf) KVC_LAUNCH((compress_k_kernel<BITS, 64, DT, DENSE, true>), b, s);
            KVC_LAUNCH((compress_k_kernel<BITS, 64, DT, DENSE, false>), b, s);
        case 128:
            if (xf) KVC_LAUNCH((compress_k_kernel<BITS, 128, DT, DENSE, true>), b, s);
            KVC_LAUNCH((compress_k_kernel<BITS, 128, DT, DENSE, false>), b, s);
        }
    } else {
        switch (group) {
        case 32: KVC_LAUNCH((compress_v_kernel<BITS, 32, DT, DENSE>), b, s);
        case 64: KVC_LAUNCH((compress_v_kernel<BITS, 64, DT, DENSE>), b, s);
        case 128: KVC_LAUNCH((compress_v_kernel<BITS, 128, DT, DENSE>), b, s);
        }
    }
    return KVC_ERR_UNSUPPORTED;
}

template <int BITS, bool DENSE> static int decompress_bits_dense(int is_v, int dtype, const QuantBatch &b, hipStream_t s)
{
    if (!is_v) {
        if (dtype == DT_F16) KVC_LAUNCH((decompress_k_kernel<BITS, DT_F16, DENSE>), b, s);
        KVC_LAUNCH((decompress_k_kernel<BITS, DT_BF16, DENSE>), b, s);
    }
    if (dtype == DT_F16) KVC_LAUNCH((decompress_v_kernel<BITS, DT_F16, DENSE>), b, s);
    KVC_LAUNCH((decompress_v_kernel<BITS, DT_BF16, DENSE>), b, s);
}

#define KVC_PASTE2(a, b) a##b
#define KVC_PASTE(a, b) KVC_PASTE2(a, b)

int KVC_PASTE(launch_compress_bits, KVC_BITS)(int is_v, int group, int dtype, const QuantBatch &b, hipStream_t s)
{
    if (b.item[0].dense)
        return dtype == DT_F16 ? compress_bits_dt<KVC_BITS, DT_F16, true>(is_v, group, b, s)
                               : compress_bits_dt<KVC_BITS, DT_BF16, true>(is_v, group, b, s);
    return dtype == DT_F16 ? compress_bits_dt<KVC_BITS, DT_F16, false>(is_v, group, b, s)
                           : compress_bits_dt<KVC_BITS, DT_BF16, false>(is_v, group, b, s);
}

int KVC_PASTE(launch_decompress_bits, KVC_BITS)(int is_v, int dtype, const QuantBatch &b, hipStream_t s)
{
    return b.item[0].dense ? decompress_bits_dense<KVC_BITS, true>(is_v, dtype, b, s) : decompress_bits_dense<KVC_BITS, false>(is_v, dtype, b, s);
}

}  // namespace kvc
