// Per-wave tile operations of the quantizer: load a pass of 32 token rows, group statistics
// along tokens (K) or along channels (V), group parameters, quantize + pack one row, and the
// inverse.  Used by the codec-free kernels and by the coder kernels alike.
#pragma once

#include "kvc_device.h"

namespace kvc {

constexpr int kXchFloats = 256;    // per-wave LDS scratch for exchanging K group parameters

__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// The lane's 8 rows of a pass: row = row0 + 4*i + rsub.  Rows past the end of the sequence
// re-read the last valid row, which leaves every group's min and max unchanged.
// DENSE: rows of one head are contiguous (stride_token == head_dim, no block table), so a
// full pass is eight loads at constant offsets from one address.
template <bool DENSE>
__device__ __forceinline__ void load_pass(const TensorView &v, long long head_off, long long row0,
                                          long long tokens, u32x4 raw[8], bool &bad, bool have_blocks = false, int blocks = 0)
{
    const int lane = lane_id(), col = lane & 15, rsub = lane >> 4;
    if (DENSE && row0 + kPassRows <= tokens) {
        const u32x4 *p = (const u32x4 *)(v.base + head_off + (row0 + rsub) * kDim + col * 8);
#pragma unroll
        for (int i = 0; i < 8; ++i) raw[i] = __builtin_nontemporal_load(p + i * 64);
        return;
    }
    long long off[8];
    if (DENSE) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            long long row = row0 + 4 * i + rsub;
            row = row < tokens ? row : tokens - 1;
            off[i] = head_off + row * kDim;
        }
    } else {
        pass_offsets(v, head_off, row0, tokens, off, bad, have_blocks, blocks);      // (blocks: entries the caller had in flight)
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) raw[i] = __builtin_nontemporal_load((const u32x4 *)(v.base + off[i] + col * 8));
}

__device__ __forceinline__ uint32_t xlane_u32(uint32_t v, int xor_mask)
{
    return (uint32_t)__builtin_amdgcn_ds_bpermute((lane_id() ^ xor_mask) << 2, (int)v);
}

// packed fp16 min / max without the compiler's NaN-quieting copies (inputs are finite)
__device__ __forceinline__ uint32_t pk_min_f16(uint32_t a, uint32_t b)
{
    uint32_t d;
    asm("v_pk_min_f16 %0, %1, %2" : "=v"(d) : "v"(a), "v"(b));
    return d;
}
__device__ __forceinline__ uint32_t pk_max_f16(uint32_t a, uint32_t b)
{
    uint32_t d;
    asm("v_pk_max_f16 %0, %1, %2" : "=v"(d) : "v"(a), "v"(b));
    return d;
}

// min(-a, -b) per half: maxima are carried negated so that one packed minimum reduces a
// (min, -max) pair
__device__ __forceinline__ uint32_t pk_min_neg_f16(uint32_t a, uint32_t b)
{
    uint32_t d;
    asm("v_pk_min_f16 %0, %1, %2 neg_lo:[1,1] neg_hi:[1,1]" : "=v"(d) : "v"(a), "v"(b));
    return d;
}
// both halves = min(a.lo, a.hi)
__device__ __forceinline__ uint32_t pk_min_halves_f16(uint32_t a)
{
    uint32_t d;
    asm("v_pk_min_f16 %0, %1, %1 op_sel:[0,1] op_sel_hi:[1,0]" : "=v"(d) : "v"(a));
    return d;
}

template <typename T> __device__ __forceinline__ T pick4(int k, T v0, T v1, T v2, T v3)
{
    return (k & 2) ? ((k & 1) ? v3 : v2) : ((k & 1) ? v1 : v0);
}

// K statistics: min / max of the lane's channels over N loaded rows and over the 4 lanes
// (rsub = 0..3) that hold the other rows of the same channels.  The lane keeps the result for
// channels 2*rsub and 2*rsub+1 only (mn2 / mx2).
template <int DT, int N>
__device__ __forceinline__ void k_stats_own(const u32x4 *raw, float mn2[2], float mx2[2])
{
    const int rsub = lane_id() >> 4;
    if (DT == DT_F16) {
        uint32_t a[4], b[4];
#pragma unroll
        for (int w = 0; w < 4; ++w) a[w] = b[w] = raw[0][w];
#pragma unroll
        for (int n = 1; n < N; ++n)
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                a[w] = pk_min_f16(a[w], raw[n][w]);
                b[w] = pk_max_f16(b[w], raw[n][w]);
            }
#pragma unroll
        for (int m = 16; m <= 32; m <<= 1)
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                a[w] = pk_min_f16(a[w], xlane_u32(a[w], m));
                b[w] = pk_max_f16(b[w], xlane_u32(b[w], m));
            }
        const uint32_t pa = pick4(rsub, a[0], a[1], a[2], a[3]), pb = pick4(rsub, b[0], b[1], b[2], b[3]);
        mn2[0] = lo_f32<DT_F16>(pa); mn2[1] = hi_f32<DT_F16>(pa);
        mx2[0] = lo_f32<DT_F16>(pb); mx2[1] = hi_f32<DT_F16>(pb);
    } else {
        float mn[8], mx[8];
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
        uint32_t pa[4], pb[4];
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            pa[w] = (__float_as_uint(mn[2 * w]) >> 16) | (__float_as_uint(mn[2 * w + 1]) & 0xffff0000u);
            pb[w] = (__float_as_uint(mx[2 * w]) >> 16) | (__float_as_uint(mx[2 * w + 1]) & 0xffff0000u);
        }
#pragma unroll
        for (int m = 16; m <= 32; m <<= 1)
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const uint32_t oa = xlane_u32(pa[w], m), ob = xlane_u32(pb[w], m);
                const float l0 = fminf(__uint_as_float(pa[w] << 16), __uint_as_float(oa << 16));
                const float l1 = fminf(__uint_as_float(pa[w] & 0xffff0000u), __uint_as_float(oa & 0xffff0000u));
                const float h0 = fmaxf(__uint_as_float(pb[w] << 16), __uint_as_float(ob << 16));
                const float h1 = fmaxf(__uint_as_float(pb[w] & 0xffff0000u), __uint_as_float(ob & 0xffff0000u));
                pa[w] = (__float_as_uint(l0) >> 16) | (__float_as_uint(l1) & 0xffff0000u);
                pb[w] = (__float_as_uint(h0) >> 16) | (__float_as_uint(h1) & 0xffff0000u);
            }
        const uint32_t sa = pick4(rsub, pa[0], pa[1], pa[2], pa[3]), sb = pick4(rsub, pb[0], pb[1], pb[2], pb[3]);
        mn2[0] = __uint_as_float(sa << 16); mn2[1] = __uint_as_float(sa & 0xffff0000u);
        mx2[0] = __uint_as_float(sb << 16); mx2[1] = __uint_as_float(sb & 0xffff0000u);
    }
}

struct KParams {
    float zero[8], inv[8];   // of the lane's 8 channels
    bool clamp;              // wave-uniform: some group of this token block needs clamping
};

// Parameters of the 128 per-channel groups of one token block.  Each of the four lanes that
// share a channel octet computes two channels, stores their metadata (scale, zero as fp16)
// and publishes (zero, 1/scale) through 64 LDS slots of 16 bytes, XSTRIDE bytes apart, at `xch`.
// meta_block: the 512 bytes of this token block's metadata, or null to skip the store.
template <int BITS, int DT, int N, int XSTRIDE>
__device__ __forceinline__ void k_group_params(const u32x4 *raw, uint8_t *xch, uint8_t *meta_block, KParams &kp)
{
    const int lane = lane_id(), col = lane & 15, rsub = lane >> 4;
    float mn2[2], mx2[2];
    k_stats_own<DT, N>(raw, mn2, mx2);
    const GroupParams g0 = make_group<BITS, DT>(mn2[0], mx2[0]);
    const GroupParams g1 = make_group<BITS, DT>(mn2[1], mx2[1]);
    if (meta_block) {
        u32x2 m;
        m[0] = g0.meta;
        m[1] = g1.meta;
        *(u32x2 *)(meta_block + (col * 8 + rsub * 2) * 4) = m;
    }
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    f32x4 mine = {g0.zero, g0.inv, g1.zero, g1.inv};
    wave_sync();                                  // earlier readers of xch are done
    *(f32x4 *)(xch + lane * XSTRIDE) = mine;
    wave_sync();
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const f32x4 o = *(const f32x4 *)(xch + (k * 16 + col) * XSTRIDE);
        kp.zero[2 * k] = o[0]; kp.inv[2 * k] = o[1];
        kp.zero[2 * k + 1] = o[2]; kp.inv[2 * k + 1] = o[3];
    }
    kp.clamp = __builtin_amdgcn_ballot_w64(g0.clamp || g1.clamp) != 0;
}

// Quantize the lane's 8 channels of one row with per-channel parameters (K).
template <int BITS, int DT, bool CLAMP>
__device__ __forceinline__ u32x2 k_quant_row(const u32x4 &raw, const KParams &kp, float one)
{
    float t[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) t[e] = elem_minus<DT>(raw, e, kp.zero[e], one) * kp.inv[e];
    return codes8<BITS, CLAMP>(t);
}

// V: the lane's 8 channels of a row belong to one group shared with GV/8 - 1 neighbouring lanes.
template <int GV, int DT>
__device__ __forceinline__ void v_row_minmax(const u32x4 &raw, float &mn, float &mx)
{
    if (DT == DT_F16) {
        // everything stays packed: (min, -max) of the lane's 8 values in one register, reduced
        // over the group's lanes by packed minima, converted once at the end
        const uint32_t a = pk_min_halves_f16(pk_min_f16(pk_min_f16(raw[0], raw[1]), pk_min_f16(raw[2], raw[3])));
        const uint32_t b = pk_min_halves_f16(pk_min_f16(pk_min_neg_f16(raw[0], raw[1]), pk_min_neg_f16(raw[2], raw[3])));
        uint32_t p = (a & 0xffffu) | (b & 0xffff0000u);
        constexpr int LANES = GV / 8;
        p = pk_min_f16(p, dpp_u32<DPP_QUAD_XOR1>(p));
        p = pk_min_f16(p, dpp_u32<DPP_QUAD_XOR2>(p));
        if (LANES >= 8) p = pk_min_f16(p, dpp_u32<DPP_HALF_MIRROR>(p));
        if (LANES >= 16) p = pk_min_f16(p, dpp_u32<DPP_MIRROR>(p));
        mn = lo_f32<DT_F16>(p);
        mx = -hi_f32<DT_F16>(p);
        return;
    } else {
        float x[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = elem_f32<DT>(raw, e);
        mn = fminf(fminf(fminf(x[0], x[1]), fminf(x[2], x[3])), fminf(fminf(x[4], x[5]), fminf(x[6], x[7])));
        mx = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
    }
    group_minmax<GV / 8>(mn, mx);
}

struct VParams {
    float zero[8], inv[8];   // of the lane's group in each of its 8 rows
    uint32_t meta[8];        // meta[i] is meaningful on the lane that owns row i
    uint32_t owner_mask;     // bit i: this lane computed (and stores the metadata of) row i
    bool clamp;              // wave-uniform
};

// Parameters of the lane's group in each of its 8 rows.  The GV/8 lanes of a group hold the
// same (min, max) after the reduction; each of them finishes one or two of the 8 rows and the
// results travel back through ds_bpermute.  vp.meta[i] is valid on the lane that owns row i
// (vp.owner_mask bit i).
template <int BITS, int GV, int DT>
__device__ __forceinline__ void v_pass_params(const u32x4 raw[8], VParams &vp)
{
    constexpr int LANES = GV / 8;
    const int lane = lane_id(), k = lane & (LANES - 1), base = lane & ~(LANES - 1);
    float mn[8], mx[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v_row_minmax<GV, DT>(raw[i], mn[i], mx[i]);
    bool c = false;
    if (LANES == 4) {
        // lane k of the quad finishes rows k and k + 4
        const GroupParams g0 = make_group<BITS, DT>(pick4(k, mn[0], mn[1], mn[2], mn[3]), pick4(k, mx[0], mx[1], mx[2], mx[3]));
        const GroupParams g1 = make_group<BITS, DT>(pick4(k, mn[4], mn[5], mn[6], mn[7]), pick4(k, mx[4], mx[5], mx[6], mx[7]));
        c = g0.clamp || g1.clamp;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const GroupParams &g = i < 4 ? g0 : g1;
            const int src = (base + (i & 3)) << 2;
            vp.zero[i] = __uint_as_float((uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)__float_as_uint(g.zero)));
            vp.inv[i] = __uint_as_float((uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)__float_as_uint(g.inv)));
            vp.meta[i] = g.meta;
        }
        vp.owner_mask = (0x11u << k);
    } else {
        // lanes 0..7 of the group finish row k
        const int r = k & 7;
        const float a = (r & 4) ? pick4(r, mn[4], mn[5], mn[6], mn[7]) : pick4(r, mn[0], mn[1], mn[2], mn[3]);
        const float b = (r & 4) ? pick4(r, mx[4], mx[5], mx[6], mx[7]) : pick4(r, mx[0], mx[1], mx[2], mx[3]);
        const GroupParams g = make_group<BITS, DT>(a, b);
        c = g.clamp;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int src = (base + i) << 2;
            vp.zero[i] = __uint_as_float((uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)__float_as_uint(g.zero)));
            vp.inv[i] = __uint_as_float((uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)__float_as_uint(g.inv)));
            vp.meta[i] = g.meta;
        }
        vp.owner_mask = k < 8 ? (1u << k) : 0u;
    }
    vp.clamp = __builtin_amdgcn_ballot_w64(c) != 0;
}

template <int BITS, int DT, bool CLAMP>
__device__ __forceinline__ u32x2 v_quant_row(const u32x4 &raw, float zero, float inv, float one)
{
    float t[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) t[e] = elem_minus<DT>(raw, e, zero, one) * inv;
    return codes8<BITS, CLAMP>(t);
}

// Where the packed codes of tile row r go: row-major (payload section) or, when SUB, the LDS
// chunk layout of the coder (sub-blocks of two rows, each padded by 16 bytes).
template <int BITS, bool SUB> __device__ __forceinline__ uint8_t *code_row(uint8_t *base, int r)
{
    if (SUB) return base + (r >> 1) * (32 * BITS + 16) + (r & 1) * (16 * BITS);
    return base + r * (16 * BITS);
}

template <int BITS> __device__ __forceinline__ void store_codes(uint8_t *row, u32x2 w)
{
    // for 3 bits, w[0] already went through quad_words_from_24
    const int col = lane_id() & 15;
    if (BITS == 3) {
        if ((col & 3) != 3) *(uint32_t *)(row + (col >> 2) * 12 + (col & 3) * 4) = w[0];
    } else {
        store_row_codes<BITS>(row, w);
    }
}

template <int BITS, int DT, int P, bool SUB, bool CLAMP, bool FULL>
__device__ __forceinline__ void k_emit_rows(const u32x4 *raw, const KParams &kp, uint8_t *base, int rows)
{
    const int rsub = lane_id() >> 4;
    const float one = opaque_one();
#pragma unroll
    for (int p = 0; p < P; ++p)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int r = p * kPassRows + 4 * i + rsub;
            u32x2 w = k_quant_row<BITS, DT, CLAMP>(raw[p * 8 + i], kp, one);
            if (BITS == 3) w[0] = quad_words_from_24(w[0]);
            if (FULL || r < rows) store_codes<BITS>(code_row<BITS, SUB>(base, r), w);
            // a token block of 64 or 128 rows: keep the scheduler from interleaving all rows, which
            // would hold the floats of every row at once (255 registers and more)
            if (P >= 2) __builtin_amdgcn_sched_barrier(0);
        }
}

// Quantize, pack and store the P*32 rows of a K token block (`rows` of them exist).
template <int BITS, int DT, int P, bool SUB>
__device__ __forceinline__ void k_emit(const u32x4 *raw, const KParams &kp, uint8_t *base, int rows)
{
    const bool full = rows >= P * kPassRows;
    if (kp.clamp) {
        if (full) k_emit_rows<BITS, DT, P, SUB, true, true>(raw, kp, base, rows);
        else k_emit_rows<BITS, DT, P, SUB, true, false>(raw, kp, base, rows);
    } else {
        if (full) k_emit_rows<BITS, DT, P, SUB, false, true>(raw, kp, base, rows);
        else k_emit_rows<BITS, DT, P, SUB, false, false>(raw, kp, base, rows);
    }
}

template <int BITS, int GV, int DT, bool SUB, bool CLAMP, bool FULL>
__device__ __forceinline__ void v_emit_rows(const u32x4 raw[8], const VParams &vp, uint8_t *base, int rows,
                                            uint32_t *meta)
{
    constexpr int LANES = GV / 8, NG = kDim / GV;
    const int lane = lane_id(), col = lane & 15, rsub = lane >> 4;
    const float one = opaque_one();
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int r = 4 * i + rsub;
        u32x2 w = v_quant_row<BITS, DT, CLAMP>(raw[i], vp.zero[i], vp.inv[i], one);
        if (BITS == 3) w[0] = quad_words_from_24(w[0]);
        if (FULL || r < rows) {
            store_codes<BITS>(code_row<BITS, SUB>(base, r), w);
            if (meta && ((vp.owner_mask >> i) & 1u)) meta[r * NG + col / LANES] = vp.meta[i];
        }
    }
}

// One pass (32 rows, `rows` of them exist) of V; base / meta point at the pass's first row.
template <int BITS, int GV, int DT, bool SUB>
__device__ __forceinline__ void v_emit(const u32x4 raw[8], const VParams &vp, uint8_t *base, int rows, uint32_t *meta)
{
    const bool full = rows >= kPassRows;
    if (vp.clamp) {
        if (full) v_emit_rows<BITS, GV, DT, SUB, true, true>(raw, vp, base, rows, meta);
        else v_emit_rows<BITS, GV, DT, SUB, true, false>(raw, vp, base, rows, meta);
    } else {
        if (full) v_emit_rows<BITS, GV, DT, SUB, false, true>(raw, vp, base, rows, meta);
        else v_emit_rows<BITS, GV, DT, SUB, false, false>(raw, vp, base, rows, meta);
    }
}

// Reconstruct the lane's 8 channels of one row: x^ = round(code * scale + zero), one fused fp32
// multiply-add, then the output rounding.  CLAMP: see pack_out.
template <int BITS, int DT, bool CLAMP>
__device__ __forceinline__ u32x4 dequant_row(u32x2 codes, const float scale[8], const float zero[8])
{
    float q[8];
    unpack8<BITS>(codes, q);
    u32x4 out;
#pragma unroll
    for (int w = 0; w < 4; ++w)
        out[w] = pack_out<DT, CLAMP>(__builtin_fmaf(q[2 * w], scale[2 * w], zero[2 * w]),
                                     __builtin_fmaf(q[2 * w + 1], scale[2 * w + 1], zero[2 * w + 1]));
    return out;
}

template <int BITS, int DT, bool CLAMP>
__device__ __forceinline__ u32x4 dequant_row_uniform(u32x2 codes, float s, float z)
{
    float q[8];
    unpack8<BITS>(codes, q);
    u32x4 out;
#pragma unroll
    for (int w = 0; w < 4; ++w)
        out[w] = pack_out<DT, CLAMP>(__builtin_fmaf(q[2 * w], s, z), __builtin_fmaf(q[2 * w + 1], s, z));
    return out;
}

// Scale and zero of the lane's 8 channels from two 16-byte metadata loads (K), and whether any
// reconstruction of this token block can exceed the fp16 range (largest code * scale + zero).
template <int BITS, int DT>
__device__ __forceinline__ bool k_meta_floats(const u32x4 &m0, const u32x4 &m1, float scale[8], float zero[8])
{
    constexpr float qmax = (float)((1 << BITS) - 1);
    float top = -65504.0f;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const uint32_t w0 = m0[e], w1 = m1[e];
        scale[e] = f16_bits_to_f32(w0 & 0xffffu); zero[e] = f16_bits_to_f32(w0 >> 16);
        scale[4 + e] = f16_bits_to_f32(w1 & 0xffffu); zero[4 + e] = f16_bits_to_f32(w1 >> 16);
    }
    if (DT != DT_F16) return false;
#pragma unroll
    for (int e = 0; e < 8; ++e) top = fmaxf(top, __builtin_fmaf(qmax, scale[e], zero[e]));
    return __builtin_amdgcn_ballot_w64(top > 65504.0f) != 0;
}

// Same for the lane's group in each of its 8 rows (V), from one metadata word per row.
template <int BITS, int DT>
__device__ __forceinline__ bool v_meta_floats(const uint32_t mw[8], float scale[8], float zero[8])
{
    constexpr float qmax = (float)((1 << BITS) - 1);
    float top = -65504.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        scale[i] = f16_bits_to_f32(mw[i] & 0xffffu);
        zero[i] = f16_bits_to_f32(mw[i] >> 16);
    }
    if (DT != DT_F16) return false;
#pragma unroll
    for (int i = 0; i < 8; ++i) top = fmaxf(top, __builtin_fmaf(qmax, scale[i], zero[i]));
    return __builtin_amdgcn_ballot_w64(top > 65504.0f) != 0;
}

// The lane's packed codes of row r.  LAYOUT 0: rows back to back (payload section); 1: the
// coder's LDS layout, sub-blocks of two rows, each padded by 16 bytes; 2: the decoder's LDS
// layout for 4-bit codes, sub-blocks of two rows without padding whose eight 16-byte pieces are
// rotated by the sub-block's number (piece p of sub-block s sits at position (p + s) mod 8), so
// that both the row-wise and the sub-block-wise accesses spread over the banks.
template <int BITS, int LAYOUT> __device__ __forceinline__ u32x2 fetch_codes(uint8_t *codes, int r)
{
    if (LAYOUT == 2) {
        static_assert(LAYOUT != 2 || BITS == 4, "rotated layout is for 4-bit codes");
        const int col = lane_id() & 15, sub = r >> 1, piece = ((r & 1) << 2) + (col >> 2);
        u32x2 w;
        w[0] = *(const uint32_t *)(codes + sub * 128 + (((piece + sub) & 7) << 4) + ((col & 3) << 2));
        w[1] = 0;
        return w;
    }
    return load_row_codes<BITS>(code_row<BITS, LAYOUT == 1>(codes, r));
}

// ---- stage T, delta transform (KVServe section 5.1 names the difference from an anchor token
//      among the transformer modules): the tokens of a head form runs of 2^shift tokens, the first
//      token of a run is its anchor and travels unchanged; every row is quantized as its
//      difference from the anchor row of its run ------------------------------------------------

// a - b (ADD: a + b) element by element on two packed rows: the exact value rounded once to the
// tensor type and limited to its finite range.  fp16: the packed half-precision add is that
// rounding, and the packed minimum / maximum against +-65504 turn an overflow into the limit
// (inputs are finite, so no NaN can arise).  bf16: one fp32 operation and the conversion give the
// same, because fp32 carries more than twice the digits of the 16-bit type.
template <int DT, bool ADD> __device__ __forceinline__ u32x4 delta_row(const u32x4 &a, const u32x4 &b)
{
    u32x4 out;
    if (DT == DT_F16) {
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const f16x2_t x = __builtin_bit_cast(f16x2_t, (uint32_t)a[w]), y = __builtin_bit_cast(f16x2_t, (uint32_t)b[w]);
            const f16x2_t r = ADD ? x + y : x - y;
            out[w] = pk_max_f16(pk_min_f16(__builtin_bit_cast(uint32_t, r), 0x7bff7bffu), 0xfbfffbffu);
        }
        return out;
    }
    constexpr float top = 3.3895313892515355e38f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const float a0 = elem_f32<DT>(a, 2 * w), a1 = elem_f32<DT>(a, 2 * w + 1);
        const float b0 = elem_f32<DT>(b, 2 * w), b1 = elem_f32<DT>(b, 2 * w + 1);
        const float y0 = ADD ? a0 + b0 : a0 - b0, y1 = ADD ? a1 + b1 : a1 - b1;
        f32x2_t v = {__builtin_amdgcn_fmed3f(y0, -top, top), __builtin_amdgcn_fmed3f(y1, -top, top)};
        out[w] = __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
    }
    return out;
}

// One pass of rows just loaded (see load_pass: rows past the end repeat the last row) becomes
// differences from their anchors, which are read from the tensor again (they were loaded moments ago
// by this or a neighbouring wave).  NA anchors per pass: 1 for runs of 32 tokens or more, 2 for runs
// of 16, 4 for runs of 8 (the rows 4*i .. 4*i+3 that one load covers share a run).  A group of rows
// past the end takes the anchor of the last row, whose copies they are.  With `keep`, the lanes that
// hold an anchor row also store it to `anchors`, the head's anchor rows in the payload.
template <int DT, bool DENSE, int NA>
__device__ __forceinline__ void delta_pass(const TensorView &v, long long head_off, long long first, long long tokens,
                                           int shift, uint16_t *anchors, bool keep, u32x4 *raw, bool &bad)
{
    const int lane = lane_id(), col = lane & 15, rsub = lane >> 4;
    const long long mask = (1ll << shift) - 1;
    u32x4 anchor[NA];
#pragma unroll
    for (int k = 0; k < NA; ++k) {
        const long long r = first + k * (kPassRows / NA);
        const bool exists = r < tokens;
        const long long arow = (exists ? r : tokens - 1) & ~mask;
        const long long off = DENSE ? head_off + arow * kDim : row_offset(v, head_off, arow, bad);
        anchor[k] = *(const u32x4 *)(v.base + off + col * 8);
        if (keep && exists && r == arow && rsub == 0) *(u32x4 *)(anchors + (arow >> shift) * kDim + col * 8) = anchor[k];
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) raw[i] = delta_row<DT, false>(raw[i], anchor[(4 * i) / (kPassRows / NA)]);
}

// N/8 passes, runs of 2^shift tokens (8 or more)
template <int DT, bool DENSE, int N>
__device__ __forceinline__ void delta_rows(const TensorView &v, long long head_off, long long row0, long long tokens,
                                           int shift, uint16_t *anchors, bool keep, u32x4 *raw, bool &bad)
{
#pragma unroll
    for (int p = 0; p < N / 8; ++p) {
        const long long first = row0 + p * kPassRows;
        if (shift >= 5) delta_pass<DT, DENSE, 1>(v, head_off, first, tokens, shift, anchors, keep, raw + p * 8, bad);
        else if (shift == 4) delta_pass<DT, DENSE, 2>(v, head_off, first, tokens, shift, anchors, keep, raw + p * 8, bad);
        else delta_pass<DT, DENSE, 4>(v, head_off, first, tokens, shift, anchors, keep, raw + p * 8, bad);
    }
}

// the head's first anchor row inside the tensor's anchor section
__device__ __forceinline__ uint16_t *head_anchors(uint16_t *anchors, long long lh, long long tokens, int shift)
{
    return anchors + lh * ((tokens + (1ll << shift) - 1) >> shift) * kDim;
}

// a reconstructed difference row back to the token row: plus the anchor of its run; an anchor
// row is its stored copy
template <int DT>
__device__ __forceinline__ u32x4 add_anchor(const u32x4 &out, const u32x4 &anchor, int shift, long long row)
{
    return (row & ((1ll << shift) - 1)) == 0 ? anchor : delta_row<DT, true>(out, anchor);
}

__device__ __forceinline__ u32x4 load_anchor(const uint16_t *anchors, int shift, long long row)
{
    return *(const u32x4 *)(anchors + (row >> shift) * kDim + (lane_id() & 15) * 8);
}

// What a pass reads before it can store: the packed codes of the lane's 8 rows and, unless the rows
// are whole and dense, where each row goes.  Fetched ahead of everything that has to wait for the
// group parameters (the choice of the clamping variant does), so that codes, block-table entries and
// parameters travel together instead of one round trip after the other.
struct PassFetch {
    u32x2 w[8];
    long long off[8];
    bool bad;           // a block-table entry out of range: nothing of the pass is stored
};

template <int BITS, bool DENSE, int LAYOUT>
__device__ __forceinline__ void pass_fetch(PassFetch &f, uint8_t *codes, const TensorView &x, long long head_off,
                                           long long row0, int rows, int row_base = 0, bool have_blocks = false, int blocks = 0)
{
    const int rsub = lane_id() >> 4;
    f.bad = false;
    if (DENSE && rows >= kPassRows) {
#pragma unroll
        for (int i = 0; i < 8; ++i) f.w[i] = fetch_codes<BITS, LAYOUT>(codes, row_base + 4 * i + rsub);
        return;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int r = 4 * i + rsub;
        const bool ok = r < rows;                       // uniform over each quad of lanes
        f.w[i] = fetch_codes<BITS, LAYOUT>(codes, row_base + (ok ? r : 0));
        if (DENSE) f.off[i] = head_off + (row0 + (ok ? r : 0)) * kDim;
    }
    if (!DENSE) pass_offsets(x, head_off, row0, row0 + rows, f.off, f.bad, have_blocks, blocks);
}

// TR: the inverse of stage T applied to every row (0 none, 1 Hadamard, 2 plus the anchor of the row's
// run, runs of 32 tokens or more, 3 the same for runs of 8 or 16 tokens)
template <int BITS, int DT, bool IS_V, bool DENSE, bool CLAMP, int TR>
__device__ __forceinline__ void dequant_pass_rows(const PassFetch &f, const float scale[8], const float zero[8],
                                                  const TensorView &x, long long head_off, long long row0, int rows,
                                                  const uint16_t *anchors, int anchor_shift, const u32x4 *loaded_anchor)
{
    const int lane = lane_id(), col = lane & 15, rsub = lane >> 4;
    // delta transform: a run of 32 tokens or more covers the whole pass (row0 is a multiple of 32), and
    // the caller may have that one anchor in flight already; runs of 16 or 8 tokens take two or four
    // anchors per pass, one per 16 or 8 rows (an anchor past the end of the sequence is replaced by
    // the last one, and no row uses it)
    constexpr int NA = TR == 3 ? 4 : 1;
    u32x4 pass_anchor[NA];
    pass_anchor[0] = u32x4{0, 0, 0, 0};
    if (TR == 2) pass_anchor[0] = loaded_anchor ? *loaded_anchor : load_anchor(anchors, anchor_shift, row0);
    if (TR == 3) {
        const long long last = row0 + (rows < kPassRows ? rows : kPassRows) - 1;
#pragma unroll
        for (int k = 0; k < NA; ++k) {
            const long long r = row0 + ((long long)k << anchor_shift);
            pass_anchor[k] = pass_anchor[0];
            if ((k << anchor_shift) < kPassRows) pass_anchor[k] = load_anchor(anchors, anchor_shift, r < last ? r : last);
        }
    }
    // the anchor of the rows 4*i .. 4*i+3
    auto anchor_of = [&](int i) -> const u32x4 & {
        return TR != 3 ? pass_anchor[0] : anchor_shift == 4 ? pass_anchor[(i >> 2) % NA] : pass_anchor[(i >> 1) % NA];
    };
    // (every load of the pass was issued before the first store: the compiler cannot move a load across
    // a store it cannot tell apart from it, and a pass that alternates them pays one memory round
    // trip per row)
    if (DENSE && rows >= kPassRows) {
        u32x4 *dst = (u32x4 *)(x.base + head_off + (row0 + rsub) * kDim + col * 8);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            u32x4 out = IS_V ? dequant_row_uniform<BITS, DT, CLAMP>(f.w[i], scale[i], zero[i])
                             : dequant_row<BITS, DT, CLAMP>(f.w[i], scale, zero);
            if (TR == 1) out = hadamard_row<DT>(out, true);
            if (TR >= 2) out = add_anchor<DT>(out, anchor_of(i), anchor_shift, row0 + 4 * i + rsub);
            __builtin_nontemporal_store(out, dst + i * 64);
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int r = 4 * i + rsub;
        u32x4 out = IS_V ? dequant_row_uniform<BITS, DT, CLAMP>(f.w[i], scale[i], zero[i])
                         : dequant_row<BITS, DT, CLAMP>(f.w[i], scale, zero);
        if (TR == 1) out = hadamard_row<DT>(out, true);     // (all 16 lanes of a row take part)
        if (TR >= 2) out = add_anchor<DT>(out, anchor_of(i), anchor_shift, row0 + (r < rows ? r : 0));
        if (r < rows && !f.bad) __builtin_nontemporal_store(out, (u32x4 *)(x.base + f.off[i] + col * 8));
    }
}

// Dequantize the fetched pass and store its `rows` existing rows at token rows row0... of head
// `head_off`, after the inverse of stage T (TR 1: Hadamard; 2: the head's anchor rows of the delta
// transform).  K: scale / zero per channel of the lane; V: per row of the lane.
template <int BITS, int DT, bool IS_V, bool DENSE, int TR = 0>
__device__ __forceinline__ void dequant_pass(const PassFetch &f, const float scale[8], const float zero[8], bool clamp,
                                             const TensorView &x, long long head_off, long long row0, int rows, bool &bad,
                                             const uint16_t *anchors = nullptr, int anchor_shift = 0,
                                             const u32x4 *loaded_anchor = nullptr)
{
    bad |= f.bad;
    if (clamp) dequant_pass_rows<BITS, DT, IS_V, DENSE, true, TR>(f, scale, zero, x, head_off, row0, rows, anchors, anchor_shift, loaded_anchor);
    else dequant_pass_rows<BITS, DT, IS_V, DENSE, false, TR>(f, scale, zero, x, head_off, row0, rows, anchors, anchor_shift, loaded_anchor);
}

// the same with the transform chosen at run time (one copy of the pass per transform; a launch
// only ever runs one of them)
template <int BITS, int DT, bool IS_V, bool DENSE>
__device__ __forceinline__ void dequant_pass_any(const PassFetch &f, const float scale[8], const float zero[8], bool clamp,
                                                 const TensorView &x, long long head_off, long long row0, int rows, bool &bad,
                                                 bool rotate, const uint16_t *anchors, int anchor_shift)
{
    if (rotate) dequant_pass<BITS, DT, IS_V, DENSE, 1>(f, scale, zero, clamp, x, head_off, row0, rows, bad);
    else if (anchors && anchor_shift >= 5) dequant_pass<BITS, DT, IS_V, DENSE, 2>(f, scale, zero, clamp, x, head_off, row0, rows, bad, anchors, anchor_shift);
    else if (anchors) dequant_pass<BITS, DT, IS_V, DENSE, 3>(f, scale, zero, clamp, x, head_off, row0, rows, bad, anchors, anchor_shift);
    else dequant_pass<BITS, DT, IS_V, DENSE, 0>(f, scale, zero, clamp, x, head_off, row0, rows, bad);
}

// bf16 rows are widened to fp32 once for the statistics and once for the quantizer.  Left alone, the
// compiler keeps the widened copy of the whole unit alive from one to the other (64 registers per
// pass, against 32 for the rows themselves); after this statement it no longer knows that the rows
// are the ones it widened, and widens again (one shift or mask per element).
template <int DT, int N> __device__ __forceinline__ void forget_unpacked(u32x4 *raw)
{
    if (DT != DT_BF16) return;
#pragma unroll
    for (int i = 0; i < N; ++i) asm volatile("" : "+v"(raw[i][0]), "+v"(raw[i][1]), "+v"(raw[i][2]), "+v"(raw[i][3]));
}

// Stage T on the rows just loaded (see hadamard_row).
template <int DT, int N> __device__ __forceinline__ void rotate_rows(u32x4 *raw)
{
#pragma unroll
    for (int i = 0; i < N; ++i) raw[i] = hadamard_row<DT>(raw[i], false);
}

}  // namespace kvc
