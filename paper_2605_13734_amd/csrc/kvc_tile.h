// Per-wave tile operations of the quantizer: load a pass of 32 token rows, group statistics
// along tokens (K) or along channels (V), quantize + pack one row, and the inverse.
// Used by the codec-free kernels and by the coder kernels alike.
#pragma once

#include "kvc_device.h"

namespace kvc {

// The lane's 8 rows of a pass: row = row0 + 4*i + rsub.  Rows past the end of the sequence
// re-read the last valid row, which leaves every group's min and max unchanged.
__device__ __forceinline__ void load_pass(const TensorView &v, long long head_off, long long row0,
                                          long long tokens, u32x4 raw[8], bool &bad)
{
    const int lane = lane_id(), col = lane & 15, rsub = lane >> 4;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        long long row = row0 + 4 * i + rsub;
        row = row < tokens ? row : tokens - 1;
        const uint16_t *p = v.base + row_offset(v, head_off, row, bad) + col * 8;
        raw[i] = *(const u32x4 *)p;
    }
}

__device__ __forceinline__ uint32_t xlane_u32(uint32_t v, int xor_mask)
{
    return (uint32_t)__builtin_amdgcn_ds_bpermute((lane_id() ^ xor_mask) << 2, (int)v);
}

// K statistics: min / max of each of the lane's 8 channels over N loaded rows and over the
// 4 lanes (rsub = 0..3) that hold the other rows of the same channels.
template <int DT, int N>
__device__ __forceinline__ void k_stats(const u32x4 *raw, float mn[8], float mx[8])
{
    if (DT == DT_F16) {
        half2_t a[4], b[4];
#pragma unroll
        for (int w = 0; w < 4; ++w) a[w] = b[w] = as_half2(raw[0][w]);
#pragma unroll
        for (int n = 1; n < N; ++n)
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                half2_t x = as_half2(raw[n][w]);
                a[w] = __builtin_elementwise_min(a[w], x);
                b[w] = __builtin_elementwise_max(b[w], x);
            }
#pragma unroll
        for (int m = 16; m <= 32; m <<= 1)
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                half2_t oa = as_half2(xlane_u32(as_u32(a[w]), m));
                half2_t ob = as_half2(xlane_u32(as_u32(b[w]), m));
                a[w] = __builtin_elementwise_min(a[w], oa);
                b[w] = __builtin_elementwise_max(b[w], ob);
            }
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            mn[2 * w] = (float)a[w][0]; mn[2 * w + 1] = (float)a[w][1];
            mx[2 * w] = (float)b[w][0]; mx[2 * w + 1] = (float)b[w][1];
        }
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) mn[e] = mx[e] = elem_f32<DT>(raw[0], e);
#pragma unroll
        for (int n = 1; n < N; ++n)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float x = elem_f32<DT>(raw[n], e);
                mn[e] = fminf(mn[e], x);
                mx[e] = fmaxf(mx[e], x);
            }
        // bfloat16 values are exact in the top half of a float: exchange two per word
#pragma unroll
        for (int m = 16; m <= 32; m <<= 1)
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                uint32_t pa = (__float_as_uint(mn[2 * w]) >> 16) | (__float_as_uint(mn[2 * w + 1]) & 0xffff0000u);
                uint32_t pb = (__float_as_uint(mx[2 * w]) >> 16) | (__float_as_uint(mx[2 * w + 1]) & 0xffff0000u);
                pa = xlane_u32(pa, m);
                pb = xlane_u32(pb, m);
                mn[2 * w] = fminf(mn[2 * w], __uint_as_float(pa << 16));
                mn[2 * w + 1] = fminf(mn[2 * w + 1], __uint_as_float(pa & 0xffff0000u));
                mx[2 * w] = fmaxf(mx[2 * w], __uint_as_float(pb << 16));
                mx[2 * w + 1] = fmaxf(mx[2 * w + 1], __uint_as_float(pb & 0xffff0000u));
            }
    }
}

// Quantize the lane's 8 channels of one row with per-channel parameters (K).
template <int BITS, int DT>
__device__ __forceinline__ u32x2 k_quant_row(const u32x4 &raw, const GroupParams gp[8])
{
    uint32_t q[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) q[e] = quantize<BITS>(elem_f32<DT>(raw, e), gp[e].zero, gp[e].inv);
    return pack8<BITS>(q);
}

// V: the lane's 8 channels belong to one group shared with GV/8 - 1 neighbouring lanes.
template <int BITS, int GV, int DT>
__device__ __forceinline__ u32x2 v_quant_row(const u32x4 &raw, uint32_t &meta_word)
{
    float x[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = elem_f32<DT>(raw, e);
    float mn, mx;
    if (DT == DT_F16) {
        half2_t h[4];
#pragma unroll
        for (int w = 0; w < 4; ++w) h[w] = as_half2(raw[w]);
        half2_t a = __builtin_elementwise_min(__builtin_elementwise_min(h[0], h[1]),
                                              __builtin_elementwise_min(h[2], h[3]));
        half2_t b = __builtin_elementwise_max(__builtin_elementwise_max(h[0], h[1]),
                                              __builtin_elementwise_max(h[2], h[3]));
        mn = fminf((float)a[0], (float)a[1]);
        mx = fmaxf((float)b[0], (float)b[1]);
    } else {
        mn = fminf(fminf(fminf(x[0], x[1]), fminf(x[2], x[3])), fminf(fminf(x[4], x[5]), fminf(x[6], x[7])));
        mx = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
    }
    group_minmax<GV / 8>(mn, mx);
    GroupParams gp = make_group<BITS>(mn, mx);
    meta_word = gp.meta;
    uint32_t q[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) q[e] = quantize<BITS>(x[e], gp.zero, gp.inv);
    return pack8<BITS>(q);
}

// Reconstruct the lane's 8 channels of one row: x^ = round(code * scale + zero).
// meta[e] = scale bits | zero bits << 16 of channel e's group.
template <int BITS, int DT>
__device__ __forceinline__ u32x4 dequant_row(u32x2 codes, const uint32_t meta[8])
{
    uint32_t q[8];
    unpack8<BITS>(codes, q);
    u32x4 out;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        float a = __builtin_fmaf((float)q[2 * w], f16_bits_to_f32(meta[2 * w] & 0xffffu),
                                 f16_bits_to_f32(meta[2 * w] >> 16));
        float b = __builtin_fmaf((float)q[2 * w + 1], f16_bits_to_f32(meta[2 * w + 1] & 0xffffu),
                                 f16_bits_to_f32(meta[2 * w + 1] >> 16));
        out[w] = pack_out<DT>(a, b);
    }
    return out;
}

template <int BITS, int DT>
__device__ __forceinline__ u32x4 dequant_row_uniform(u32x2 codes, uint32_t meta_word)
{
    uint32_t q[8];
    unpack8<BITS>(codes, q);
    const float s = f16_bits_to_f32(meta_word & 0xffffu), z = f16_bits_to_f32(meta_word >> 16);
    u32x4 out;
#pragma unroll
    for (int w = 0; w < 4; ++w)
        out[w] = pack_out<DT>(__builtin_fmaf((float)q[2 * w], s, z), __builtin_fmaf((float)q[2 * w + 1], s, z));
    return out;
}

}  // namespace kvc
