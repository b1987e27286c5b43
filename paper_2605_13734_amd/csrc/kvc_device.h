// Device-side building blocks shared by the gfx950 kernels: lane geometry, row addressing,
// 16-bit float conversion, group statistics, the quantizer and the bit packers.
//
// Lane geometry of every kernel: a wave of 64 lanes covers 4 token rows of one head at a
// time; lane = 16*rsub + col, col owns channels [8*col, 8*col+8) (one 128-bit load),
// rsub picks the row.  A "pass" is 32 rows: row = row0 + 4*i + rsub, i = 0..7.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kvc {

constexpr int kDim = 128;          // head_dim the kernels are written for
constexpr int kPassRows = 32;      // token rows per wave pass
constexpr int kChunkRows = 128;    // token rows per coder chunk
constexpr int kSubs = 64;          // sub-blocks per chunk (2 rows each)
constexpr int kMaxLen = 12;        // longest code word
constexpr int kHeader = 128;

enum { DT_F16 = 1, DT_BF16 = 2 };

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// One tensor (K or V) of one request.
struct TensorView {
    uint16_t *base;
    long long stride_layer, stride_head, stride_token, stride_block;   // elements
    const int *block_table;     // null = contiguous
    int bt_shift;               // log2(block_tokens)
    int num_phys_blocks;
    int bt_wave;                // blocks of 4 tokens or more whose rows lie within 2^31 elements at a stride
                                // below 2^24: a pass needs one table entry per 4 rows, read once per wave
};

// Bit casts go through by-value scalars: applying __builtin_bit_cast directly to an element
// of an ext_vector (v[i]) reads element 0 with this compiler.
__device__ __forceinline__ half2_t as_half2(uint32_t u) { return __builtin_bit_cast(half2_t, u); }
__device__ __forceinline__ uint32_t as_u32(half2_t h) { return __builtin_bit_cast(uint32_t, h); }

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }
// The wave's index inside its workgroup, as a value the compiler knows to be the same in all lanes:
// everything derived from it (unit and chunk numbers, head offsets, block-table entries) is then
// computed once per wave by the scalar unit instead of once per lane.
__device__ __forceinline__ int wave_id() { return __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)); }

// Element offset of row t of head (l, h).  A block-table entry out of range is reported
// through `bad` and replaced by block 0, so the address is always inside the pool.
__device__ __forceinline__ long long row_offset(const TensorView &v, long long head_off, long long t,
                                                bool &bad)
{
    if (v.block_table == nullptr) return head_off + t * v.stride_token;
    int blk = v.block_table[t >> v.bt_shift];
    if ((unsigned)blk >= (unsigned)v.num_phys_blocks) { bad = true; blk = 0; }
    return head_off + (long long)blk * v.stride_block +
           (t & ((1ll << v.bt_shift) - 1)) * v.stride_token;
}

// Element offsets of the lane's 8 rows of the pass that starts at row0 (a multiple of 32; row0 and
// head_off the same in all lanes): row = row0 + 4*i + rsub, rows past the end of the sequence
// replaced by the last one.  With a block table whose blocks hold 4 tokens or more, the four rows
// 4*i .. 4*i+3 share a block: its entry is read and turned into a base once per wave, and a lane
// adds its row's place inside the block with a 24-bit multiply.
// The block-table entries of the rows row0 + 4*i, i = 0..7, of a pass (rows past `tokens` repeat the
// last one), one load: lane l brings entry l & 7.  row0 and tokens are the same in all lanes.
__device__ __forceinline__ int pass_blocks(const TensorView &v, long long row0, long long tokens)
{
    long long first = row0 + 4 * (lane_id() & 7);
    first = first < tokens ? first : tokens - 1;
    return v.block_table[first >> v.bt_shift];
}

// `ahead` (with have_ahead): the pass's entries from pass_blocks, when the caller had them in flight already.
__device__ __forceinline__ void pass_offsets(const TensorView &v, long long head_off, long long row0, long long tokens,
                                             long long off[8], bool &bad, bool have_ahead = false, int ahead = 0)
{
    const int rsub = lane_id() >> 4;
    if (v.block_table == nullptr || !v.bt_wave) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            long long row = row0 + 4 * i + rsub;
            row = row < tokens ? row : tokens - 1;
            off[i] = row_offset(v, head_off, row, bad);
        }
        return;
    }
    const int mask = (1 << v.bt_shift) - 1;
    const int entries = have_ahead ? ahead : pass_blocks(v, row0, tokens);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        int blk = __builtin_amdgcn_readlane(entries, i);
        if ((unsigned)blk >= (unsigned)v.num_phys_blocks) { bad = true; blk = 0; }
        const long long base = head_off + (long long)blk * v.stride_block;
        long long row = row0 + 4 * i + rsub;
        row = row < tokens ? row : tokens - 1;
        off[i] = base + (long long)__umul24((unsigned)((int)row & mask), (unsigned)v.stride_token);
    }
}

// ---- 16-bit floats ----------------------------------------------------------------------

template <int DT> __device__ __forceinline__ float lo_f32(uint32_t w)
{
    if (DT == DT_F16) return (float)__builtin_bit_cast(_Float16, (uint16_t)(w & 0xffffu));
    return __uint_as_float(w << 16);
}
template <int DT> __device__ __forceinline__ float hi_f32(uint32_t w)
{
    if (DT == DT_F16) return (float)__builtin_bit_cast(_Float16, (uint16_t)(w >> 16));
    return __uint_as_float(w & 0xffff0000u);
}
template <int DT> __device__ __forceinline__ float elem_f32(const u32x4 &r, int e)
{
    return (e & 1) ? hi_f32<DT>(r[e >> 1]) : lo_f32<DT>(r[e >> 1]);
}

// 1.0f in a register the optimizer cannot see through
__device__ __forceinline__ float opaque_one()
{
    float v;
    asm("v_mov_b32 %0, 1.0" : "=v"(v));
    return v;
}

// element e minus `zero`, rounded once to fp32.  For fp16 this is written as fma(x, 1, -zero),
// which the mixed-precision FMA computes straight from the 16-bit half of the register (the
// product with one is exact, so the result equals the rounded difference).
template <int DT> __device__ __forceinline__ float elem_minus(const u32x4 &r, int e, float zero, float one)
{
    if (DT == DT_F16) return __builtin_fmaf(elem_f32<DT>(r, e), one, -zero);
    return elem_f32<DT>(r, e) - zero;
}

__device__ __forceinline__ float f16_bits_to_f32(uint32_t h)
{
    return (float)__builtin_bit_cast(_Float16, (uint16_t)h);
}
__device__ __forceinline__ uint32_t f32_to_f16_bits(float f)
{
    return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)f);     // round to nearest even
}
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;                  // nearest even, finite input
}

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

// Keeps the compiler from merging an fp32 operation with a following conversion to fp16 into
// one mixed-precision instruction, which would round once instead of twice.
__device__ __forceinline__ float rounded_f32(float x)
{
    asm volatile("" : "+v"(x));
    return x;
}

// Two reconstructed values (results of code * scale + zero with fp16 scale and zero, code >= 0)
// -> one packed word of the output type, round to nearest even.  Such a value is never below
// zero >= -65504, so only the upper end of the fp16 range can be exceeded (CLAMP); it cannot
// leave the bfloat16 range at all.
template <int DT, bool CLAMP> __device__ __forceinline__ uint32_t pack_out(float a, float b)
{
    if (DT == DT_F16) {
        if (CLAMP) {
            a = fminf(a, 65504.0f);
            b = fminf(b, 65504.0f);
        } else {
            a = rounded_f32(a);
            b = rounded_f32(b);
        }
        return f32_to_f16_bits(a) | (f32_to_f16_bits(b) << 16);
    }
    f32x2_t v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));      // v_cvt_pk_bf16_f32
}

// ---- cross-lane helpers -----------------------------------------------------------------

template <int CTRL> __device__ __forceinline__ float dpp_f32(float v)
{
    return __uint_as_float((uint32_t)__builtin_amdgcn_update_dpp(0, (int)__float_as_uint(v), CTRL, 0xf, 0xf, true));
}
template <int CTRL> __device__ __forceinline__ uint32_t dpp_u32(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, true);
}
constexpr int DPP_QUAD_XOR1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int DPP_QUAD_XOR2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int DPP_HALF_MIRROR = 0x141;     // reverse within 8 lanes
constexpr int DPP_MIRROR = 0x140;          // reverse within 16 lanes
constexpr int DPP_QUAD_NEXT = 0xF9;        // quad_perm [1,2,3,3]: lane k reads lane k+1
constexpr int DPP_QUAD_PREV = 0x90;        // quad_perm [0,0,1,2]: lane k reads lane k-1

__device__ __forceinline__ float xlane_f32(float v, int xor_mask)
{
    return __uint_as_float((uint32_t)__builtin_amdgcn_ds_bpermute(((lane_id() ^ xor_mask) << 2),
                                                                  (int)__float_as_uint(v)));
}

// min and max over the `LANES` (4, 8 or 16) adjacent lanes that share a V group
template <int LANES> __device__ __forceinline__ void group_minmax(float &mn, float &mx)
{
    mn = fminf(mn, dpp_f32<DPP_QUAD_XOR1>(mn));
    mx = fmaxf(mx, dpp_f32<DPP_QUAD_XOR1>(mx));
    mn = fminf(mn, dpp_f32<DPP_QUAD_XOR2>(mn));
    mx = fmaxf(mx, dpp_f32<DPP_QUAD_XOR2>(mx));
    if (LANES >= 8) {
        mn = fminf(mn, dpp_f32<DPP_HALF_MIRROR>(mn));
        mx = fmaxf(mx, dpp_f32<DPP_HALF_MIRROR>(mx));
    }
    if (LANES >= 16) {
        mn = fminf(mn, dpp_f32<DPP_MIRROR>(mn));
        mx = fmaxf(mx, dpp_f32<DPP_MIRROR>(mx));
    }
}

// ---- transform (KVServe section 5.1, stage T: the Hadamard rotation among the transformer
//      modules) ---------------------------------------------------------------------------------

// The value of lane (lane ^ MASK), MASK = 1, 2, 4 or 8: within the 16 lanes that hold one row.
template <int MASK> __device__ __forceinline__ float xor_lane_f32(float v)
{
    if (MASK == 1) return dpp_f32<DPP_QUAD_XOR1>(v);
    if (MASK == 2) return dpp_f32<DPP_QUAD_XOR2>(v);
    // ds_swizzle, bit-mask mode: and 0x1f, or 0, xor MASK (no LDS memory is touched)
    return __uint_as_float((uint32_t)__builtin_amdgcn_ds_swizzle((int)__float_as_uint(v), (MASK << 10) | 0x1f));
}

typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));

// One row of 128 values, 8 per lane over 16 lanes (lane & 15 = col holds channels 8*col ...):
// y = H x * scale, H the Walsh-Hadamard matrix in natural order, as the fast transform with the
// strides 1, 2, 4 (inside the lane), 8, 16, 32, 64 (across lanes) in this order, every sum and
// difference one fp32 operation; scale = 1/8 on the way in, 1/16 on the way back (both exact);
// the result is limited to the finite range of the type and rounded to it.  All 16 lanes of a
// row must be active.
//
// How the same bits are reached with fewer instructions: the scale, a power of two, is applied
// in the first stage, which for fp16 input is computed straight from the packed halves by the
// mixed-precision FMA (scaling by a power of two commutes with every later rounding).  In a
// stage across lanes every lane computes own + c * other with c = +-1 on the operand that comes
// from the other lane, so that the lane exchange can ride on the multiply-add; the lane that
// should hold a - b then holds b - a, and a lane's values are negated once for every set bit
// of col.  That sign is folded into the first stage's factor, which flips the roles of c.
template <int DT> __device__ __forceinline__ u32x4 hadamard_row(const u32x4 &in, bool inverse)
{
    const int col = lane_id() & 15;
    const float factor = (__builtin_popcount(col) & 1 ? -1.0f : 1.0f) * (inverse ? 0.0625f : 0.125f);
    float x[8];
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const float lo = elem_f32<DT>(in, 2 * w), hi = elem_f32<DT>(in, 2 * w + 1) * factor;
        x[2 * w] = __builtin_fmaf(lo, factor, hi);
        x[2 * w + 1] = __builtin_fmaf(lo, factor, -hi);
    }
#pragma unroll
    for (int h = 2; h < 8; h <<= 1)
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (!(j & h)) {
                const float a = x[j], b = x[j + h];
                x[j] = a + b;
                x[j + h] = a - b;
            }
    // x[e] += c * (x[e] of lane ^ m): for m = 1, 2 and 8 the lane exchange is a DPP pattern (two quad
    // permutations, a rotation of the row of 16 by 8) that the multiply-add itself can carry
    // (v_fmac_f32 with a DPP source: one instruction, the same single rounding); the compiler does not
    // form it and keeps a separate move, so the eight of a stage are written out.  A DPP source must
    // not have been written by the two instructions before it (five, if that was a vector write of
    // EXEC): inside a block the writer of x[e] is eight instructions back, and the block opens with five
    // wait states.
#define KVC_FMAC_DPP8(CTRL)                                                                                          \
    asm("s_nop 4\n\t"                                                                                                \
        "v_fmac_f32_dpp %0, %0, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                                          \
        "v_fmac_f32_dpp %1, %1, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                                          \
        "v_fmac_f32_dpp %2, %2, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                                          \
        "v_fmac_f32_dpp %3, %3, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                                          \
        "v_fmac_f32_dpp %4, %4, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                                          \
        "v_fmac_f32_dpp %5, %5, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                                          \
        "v_fmac_f32_dpp %6, %6, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                                          \
        "v_fmac_f32_dpp %7, %7, %8 " CTRL " row_mask:0xf bank_mask:0xf"                                               \
        : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]), "+v"(x[4]), "+v"(x[5]), "+v"(x[6]), "+v"(x[7])             \
        : "v"(c))
#pragma unroll
    for (int m = 1; m < 16; m <<= 1) {
        const float c = (col & m) ? 1.0f : -1.0f;
        if (m == 1) KVC_FMAC_DPP8("quad_perm:[1,0,3,2]");
        else if (m == 2) KVC_FMAC_DPP8("quad_perm:[2,3,0,1]");
        else if (m == 8) KVC_FMAC_DPP8("row_ror:8");
        else {
#pragma unroll
            for (int e = 0; e < 8; ++e)
                x[e] = __builtin_fmaf(xor_lane_f32<4>(x[e]), c, x[e]);         // exact product, one rounded sum
        }
    }
#undef KVC_FMAC_DPP8
    constexpr float top = DT == DT_F16 ? 65504.0f : 3.3895313892515355e38f;
    u32x4 out;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        f32x2_t v = {__builtin_amdgcn_fmed3f(x[2 * w], -top, top), __builtin_amdgcn_fmed3f(x[2 * w + 1], -top, top)};
        if (DT == DT_F16) out[w] = __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2_t));
        else out[w] = __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
    }
    return out;
}

// ---- quantizer (KVServe section 5.1, stage Q: asymmetric, grouped; section 7.3: two
//      16-bit metadata values per group) ------------------------------------------------

struct GroupParams {
    float zero;       // fp16-rounded minimum, as float
    float inv;        // 1 / fp16-rounded scale (0 when the scale is 0)
    uint32_t meta;    // scale bits | zero bits << 16
    bool clamp;       // codes of this group can leave [0, 2^bits-1] before clamping
};

// range / (2^BITS - 1), correctly rounded: product with the rounded reciprocal, one exact
// residual, one correction.  Equal to IEEE division for every float in [0, 2^17] (checked
// exhaustively on the device by kvc_selftest).
template <int BITS> __device__ __forceinline__ float div_levels(float r)
{
    constexpr float qmax = (float)((1 << BITS) - 1);
    constexpr float c = 1.0f / qmax;
    const float q0 = r * c;
    const float e = __builtin_fmaf(-q0, qmax, r);
    return __builtin_fmaf(e, c, q0);
}

// 1 / s for a positive fp16-representable s: hardware estimate plus one Newton step, equal to
// IEEE division for all such s (checked exhaustively by kvc_selftest).
__device__ __forceinline__ float rcp_f16_exact(float s)
{
    const float y = __builtin_amdgcn_rcpf(s);
    const float e = __builtin_fmaf(-s, y, 1.0f);
    return __builtin_fmaf(y, e, y);
}

// zero = fp16(min), scale = fp16((max - min) / (2^bits - 1)); a zero of either sign is +0.
// With fp16 input the minimum is its own fp16 rounding and the scale cannot overflow.
template <int BITS, int DT> __device__ __forceinline__ GroupParams make_group(float mn, float mx)
{
    mn += 0.0f;
    mx += 0.0f;
    float lo = mn;
    if (DT != DT_F16) lo = __builtin_amdgcn_fmed3f(mn, -65504.0f, 65504.0f);
    const uint32_t zb = f32_to_f16_bits(lo);
    float s = rounded_f32(div_levels<BITS>(mx - mn));
    if (DT != DT_F16) s = fminf(s, 65504.0f);
    const uint32_t sb = f32_to_f16_bits(s);
    const float sh = f16_bits_to_f32(sb);
    GroupParams g;
    g.zero = (DT == DT_F16) ? lo : f16_bits_to_f32(zb);
    g.inv = (sh == 0.0f) ? 0.0f : rcp_f16_exact(sh);
    g.meta = sb | (zb << 16);
    // with a normal fp16 scale that was not limited and zero == min, (x - zero) * inv rounds into
    // [0, 2^bits - 1]; a bfloat16 group can have its zero point or its scale limited to the fp16 range
    g.clamp = sh < 6.103515625e-05f || (DT != DT_F16 && (g.zero != mn || sh >= 65504.0f));
    return g;
}

// code = clamp(round_half_even((x - zero) * inv), 0, 2^bits - 1); two rounded fp32 operations
// (the centered value x - zero is the first, its product with inv the second).
//
// codes8 turns the 8 products of one lane into BITS bytes, element i at bits
// [i*BITS, i*BITS+BITS), low bits first.  CLAMP = false is for groups whose codes cannot leave
// the range (GroupParams::clamp).  For 2, 4 and 8 bits the rounding is done by the
// float-to-byte conversion that inserts its result into a chosen byte of a word (round to
// nearest even on [0, 255], checked by kvc_selftest); the bytes are laid out so that one or
// two shifted ORs finish the word.  3-bit codes are rounded as floats, summed with their place
// values in fp32 (exact below 2^24) and converted once.
template <int BITS, bool CLAMP> __device__ __forceinline__ u32x2 codes8(float t[8])
{
    constexpr float qmax = (float)((1 << BITS) - 1);
    if (CLAMP) {
#pragma unroll
        for (int e = 0; e < 8; ++e) t[e] = __builtin_amdgcn_fmed3f(t[e], 0.0f, qmax);
    }
    u32x2 r;
    r[1] = 0;
    if (BITS == 8) {
        uint32_t a = 0, b = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            a = __builtin_amdgcn_cvt_pk_u8_f32(t[e], e, a);
            b = __builtin_amdgcn_cvt_pk_u8_f32(t[4 + e], e, b);
        }
        r[0] = a;
        r[1] = b;
    } else if (BITS == 4) {
        uint32_t even = 0, odd = 0;                 // bytes: codes 0 2 4 6 and 1 3 5 7
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            even = __builtin_amdgcn_cvt_pk_u8_f32(t[2 * e], e, even);
            odd = __builtin_amdgcn_cvt_pk_u8_f32(t[2 * e + 1], e, odd);
        }
        r[0] = (odd << 4) | even;
    } else if (BITS == 2) {
        uint32_t even = 0, odd = 0;                 // bytes: codes 0 4 2 6 and 1 5 3 7
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int byte = ((e & 1) << 1) | (e >> 1);       // 0 2 1 3
            even = __builtin_amdgcn_cvt_pk_u8_f32(t[2 * e], byte, even);
            odd = __builtin_amdgcn_cvt_pk_u8_f32(t[2 * e + 1], byte, odd);
        }
        const uint32_t pairs = (odd << 2) | even;   // bytes: codes 01, 45, 23, 67
        r[0] = (pairs | (pairs >> 12)) & 0xffffu;
    } else {
        float acc = __builtin_rintf(t[0]);
#pragma unroll
        for (int e = 1; e < 8; ++e) acc = __builtin_fmaf(__builtin_rintf(t[e]), (float)(1 << (BITS * e)), acc);
        r[0] = (uint32_t)acc;
    }
    return r;
}

// The lane's 8 codes as floats.  4- and 8-bit codes go through the byte-to-float conversions.
template <int BITS> __device__ __forceinline__ void unpack8(u32x2 w, float q[8])
{
    if (BITS == 8) {
#pragma unroll
        for (int e = 0; e < 8; ++e) q[e] = (float)((w[e >> 2] >> ((e & 3) * 8)) & 0xffu);
    } else if (BITS == 4) {
        const uint32_t lo = w[0] & 0x0f0f0f0fu, hi = (w[0] >> 4) & 0x0f0f0f0fu;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            q[2 * k] = (float)((lo >> (8 * k)) & 0xffu);
            q[2 * k + 1] = (float)((hi >> (8 * k)) & 0xffu);
        }
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) q[e] = (float)((w[0] >> (e * BITS)) & ((1u << BITS) - 1u));
    }
}

// 3-bit rows: the 4 lanes of a quad hold 4 x 24 bits = three aligned words.  Lane k < 3 of
// the quad ends up owning word k.
__device__ __forceinline__ uint32_t quad_words_from_24(uint32_t c24)
{
    int k = lane_id() & 3;
    uint32_t next = dpp_u32<DPP_QUAD_NEXT>(c24);
    return (k == 0) ? (c24 | (next << 24)) : ((c24 >> (8 * k)) | (next << (24 - 8 * k)));
}
// Inverse: lane k < 3 holds word k (lane 3 holds word 2 again); every lane gets its 24 bits.
__device__ __forceinline__ uint32_t quad_24_from_words(uint32_t word)
{
    int k = lane_id() & 3;
    uint32_t prev = dpp_u32<DPP_QUAD_PREV>(word);       // lane 0 reads itself
    uint32_t lo = (k == 0) ? word : (prev >> ((32 - 8 * k) & 31));
    uint32_t hi = (k == 0) ? 0u : (word << (8 * k));
    return (lo | hi) & 0xffffffu;
}

// Byte offset of a lane's packed codes inside a row of 16*BITS bytes, and the store itself.
// 2 bits: u16 per lane; 3 bits: word per lane for 3 lanes of 4; 4 bits: word; 8 bits: 2 words.
template <int BITS> __device__ __forceinline__ void store_row_codes(uint8_t *row, u32x2 w)
{
    int col = lane_id() & 15;
    if (BITS == 2) {
        *(uint16_t *)(row + col * 2) = (uint16_t)w[0];
    } else if (BITS == 3) {
        uint32_t word = quad_words_from_24(w[0]);
        if ((col & 3) != 3) *(uint32_t *)(row + (col >> 2) * 12 + (col & 3) * 4) = word;
    } else if (BITS == 4) {
        *(uint32_t *)(row + col * 4) = w[0];
    } else {
        *(u32x2 *)(row + col * 8) = w;
    }
}

template <int BITS> __device__ __forceinline__ u32x2 load_row_codes(const uint8_t *row)
{
    int col = lane_id() & 15;
    u32x2 w;
    w[1] = 0;
    if (BITS == 2) {
        w[0] = *(const uint16_t *)(row + col * 2);
    } else if (BITS == 3) {
        int k = col & 3;
        uint32_t word = *(const uint32_t *)(row + (col >> 2) * 12 + (k == 3 ? 2 : k) * 4);
        w[0] = quad_24_from_words(word);
    } else if (BITS == 4) {
        w[0] = *(const uint32_t *)(row + col * 4);
    } else {
        w = *(const u32x2 *)(row + col * 8);
    }
    return w;
}

}  // namespace kvc
