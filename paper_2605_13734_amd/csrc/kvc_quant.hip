// Codec-free kernels: quantize + pack (compress) and unpack + dequantize (decompress) one
// tensor of one request straight between the KV layout and the payload sections.
// One wave per work unit, four units per workgroup, no LDS, no barriers.
//   K compress unit   = one token block of G rows x 128 channels (all 128 per-channel groups)
//   other units       = 32 token rows
// Stage Q of the pipeline (KVServe section 5.1); memory-bound, so no matrix cores.

#include "kvc_internal.h"
#include "kvc_tile.h"
#include "../../include/kvc.h"

namespace kvc {

struct UnitPos {
    long long lh;        // layer * heads + head
    long long blk;       // unit index inside the head
    long long head_off;  // element offset of x[l][h][0][0]
};

__device__ __forceinline__ bool unit_pos(const QuantArgs &a, UnitPos &u)
{
    long long unit = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (unit >= a.total_units) return false;
    const long long slot = unit / a.units_per_head;
    u.lh = a.head_list ? a.head_list[slot] : slot;
    u.blk = unit - slot * a.units_per_head;
    long long l = u.lh / a.heads, h = u.lh - l * a.heads;
    u.head_off = l * a.x.stride_layer + h * a.x.stride_head;
    return true;
}

// first code byte of head lh (width BITS) in its section
template <int BITS> __device__ __forceinline__ uint8_t *head_codes(const QuantArgs &a, long long lh)
{
    const long long widths = a.bits_before ? a.bits_before[lh] : lh * BITS;
    return a.codes + widths * a.tokens * 16;
}

__device__ __forceinline__ void report(int *status, bool bad)
{
    if (bad) atomicOr(status, KVC_DEV_BAD_BLOCK);
}

// ---- K: groups along tokens, one per channel ------------------------------------------------

// XF = false leaves the code of stage T out (for launches without a transform): sharing a kernel
// with it doubles the registers of the plain path for token blocks of 64 and 128 rows.
template <int BITS, int G, int DT, bool DENSE, bool XF>
__global__ __launch_bounds__(256) void compress_k_kernel(QuantArgs a)
{
    __shared__ __attribute__((aligned(16))) float xch_all[4 * kXchFloats];
    UnitPos u;
    if (!unit_pos(a, u)) return;
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
    k_group_params<BITS, DT, P * 8, 16>(raw, (uint8_t *)(xch_all + (threadIdx.x >> 6) * kXchFloats), meta_block, kp);
    uint8_t *codes = head_codes<BITS>(a, u.lh) + row0 * (16 * BITS);
    const long long left = a.tokens - row0;
    k_emit<BITS, DT, P, false>(raw, kp, codes, left < G ? (int)left : G);
    report(a.status, bad);
}

template <int BITS, int DT, bool DENSE>
__global__ __launch_bounds__(256) void decompress_k_kernel(QuantArgs a)
{
    UnitPos u;
    if (!unit_pos(a, u)) return;
    if (*a.status & KVC_DEV_BAD_HEADER) return;
    const int col = lane_id() & 15;
    const long long row0 = u.blk * kPassRows;
    const long long tb = row0 / a.group, nb = (a.tokens + a.group - 1) / a.group;
    const u32x4 *m = (const u32x4 *)(a.meta + ((u.lh * nb + tb) * kDim + col * 8) * 4);
    const u32x4 m0 = m[0], m1 = m[1];
    float scale[8], zero[8];
    const bool clamp = k_meta_floats<BITS, DT>(m0, m1, scale, zero);
    uint8_t *codes = head_codes<BITS>(a, u.lh) + row0 * (16 * BITS);
    const long long left = a.tokens - row0;
    bool bad = false;
    dequant_pass_any<BITS, DT, false, DENSE, 0>(codes, scale, zero, clamp, a.x, u.head_off, row0,
                                                left < kPassRows ? (int)left : kPassRows, bad, a.rotate != 0,
                                                a.anchors ? head_anchors(a.anchors, u.lh, a.tokens, a.anchor_shift) : nullptr,
                                                a.anchor_shift);
    report(a.status, bad);
}

// ---- V: groups along channels, one set per token -----------------------------------------------

template <int BITS, int GV, int DT, bool DENSE>
__global__ __launch_bounds__(256) void compress_v_kernel(QuantArgs a)
{
    UnitPos u;
    if (!unit_pos(a, u)) return;
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
    uint8_t *codes = head_codes<BITS>(a, u.lh) + row0 * (16 * BITS);
    uint32_t *meta = (uint32_t *)a.meta + (u.lh * a.tokens + row0) * NG;
    const long long left = a.tokens - row0;
    v_emit<BITS, GV, DT, false>(raw, vp, codes, left < kPassRows ? (int)left : kPassRows, meta);
    report(a.status, bad);
}

template <int BITS, int DT, bool DENSE>
__global__ __launch_bounds__(256) void decompress_v_kernel(QuantArgs a)
{
    UnitPos u;
    if (!unit_pos(a, u)) return;
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
    float scale[8], zero[8];
    const bool clamp = v_meta_floats<BITS, DT>(mw, scale, zero);
    uint8_t *codes = head_codes<BITS>(a, u.lh) + row0 * (16 * BITS);
    bool bad = false;
    dequant_pass_any<BITS, DT, true, DENSE, 0>(codes, scale, zero, clamp, a.x, u.head_off, row0, rows, bad, a.rotate != 0,
                                               a.anchors ? head_anchors(a.anchors, u.lh, a.tokens, a.anchor_shift) : nullptr,
                                               a.anchor_shift);
    report(a.status, bad);
}

// ---- 16 bits: the tensor travels unchanged ----------------------------------------------------

template <bool TO_PAYLOAD>
__global__ __launch_bounds__(256) void copy_rows_kernel(QuantArgs a)
{
    UnitPos u;
    if (!unit_pos(a, u)) return;
    if (!TO_PAYLOAD && (*a.status & KVC_DEV_BAD_HEADER)) return;
    const int lane = lane_id(), col = lane & 15, rsub = lane >> 4;
    const long long row0 = u.blk * kPassRows;
    bool bad = false;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const long long row = row0 + 4 * i + rsub;
        if (row < a.tokens) {
            bool b = false;
            uint16_t *x = a.x.base + row_offset(a.x, u.head_off, row, b) + col * 8;
            u32x4 *p = (u32x4 *)(a.codes + ((u.lh * a.tokens + row) * kDim + col * 8) * 2);
            if (TO_PAYLOAD) *p = *(const u32x4 *)x;
            else if (!b) *(u32x4 *)x = *p;
            bad |= b;
        }
    }
    report(a.status, bad);
}

// ---- small service kernels --------------------------------------------------------------------

__global__ void write_header_kernel(uint32_t *dst, HeaderBytes h)
{
    if (threadIdx.x < 32) dst[threadIdx.x] = h.w[threadIdx.x];
}

__global__ void check_header_kernel(const uint32_t *hdr, HeaderBytes expect, uint32_t mask, int *status)
{
    const int i = threadIdx.x;
    bool diff = i < 32 && ((mask >> i) & 1u) && hdr[i] != expect.w[i];
    if (diff) atomicOr(status, KVC_DEV_BAD_HEADER);
}

// two byte strings of the same length must be equal (the width tables of payload and plan)
__global__ void check_bytes_kernel(const uint8_t *a, const uint8_t *b, long long n, int *status)
{
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n && a[i] != b[i]) atomicOr(status, KVC_DEV_BAD_HEADER);
}

__global__ void fill_u32_kernel(uint32_t *dst, uint32_t value, long long n)
{
    long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = value;
}

// ---- launchers ----------------------------------------------------------------------------------

static inline dim3 grid_for(long long units) { return dim3((unsigned)((units + 3) / 4)); }

#define KVC_LAUNCH(kernel, a, s)                                                        \
    do {                                                                                \
        if ((a).total_units > 0)                                                        \
            hipLaunchKernelGGL(kernel, grid_for((a).total_units), dim3(256), 0, s, a);  \
        return hipGetLastError() == hipSuccess ? KVC_OK : KVC_ERR_DEVICE;               \
    } while (0)

template <int BITS, int DT, bool DENSE> static int compress_bits_dt(int is_v, int group, const QuantArgs &a, hipStream_t s)
{
    if (!is_v) {
        const bool xf = a.rotate || a.anchors;
        switch (group) {
        case 32: KVC_LAUNCH((compress_k_kernel<BITS, 32, DT, DENSE, true>), a, s);
        case 64:
            if (xf) KVC_LAUNCH((compress_k_kernel<BITS, 64, DT, DENSE, true>), a, s);
            KVC_LAUNCH((compress_k_kernel<BITS, 64, DT, DENSE, false>), a, s);
        case 128:
            if (xf) KVC_LAUNCH((compress_k_kernel<BITS, 128, DT, DENSE, true>), a, s);
            KVC_LAUNCH((compress_k_kernel<BITS, 128, DT, DENSE, false>), a, s);
        }
    } else {
        switch (group) {
        case 32: KVC_LAUNCH((compress_v_kernel<BITS, 32, DT, DENSE>), a, s);
        case 64: KVC_LAUNCH((compress_v_kernel<BITS, 64, DT, DENSE>), a, s);
        case 128: KVC_LAUNCH((compress_v_kernel<BITS, 128, DT, DENSE>), a, s);
        }
    }
    return KVC_ERR_UNSUPPORTED;
}

template <int BITS> static int compress_bits(int is_v, int group, int dtype, const QuantArgs &a, hipStream_t s)
{
    if (a.dense)
        return dtype == DT_F16 ? compress_bits_dt<BITS, DT_F16, true>(is_v, group, a, s)
                               : compress_bits_dt<BITS, DT_BF16, true>(is_v, group, a, s);
    return dtype == DT_F16 ? compress_bits_dt<BITS, DT_F16, false>(is_v, group, a, s)
                           : compress_bits_dt<BITS, DT_BF16, false>(is_v, group, a, s);
}

int launch_compress_tensor(int is_v, int bits, int group, int dtype, const QuantArgs &a, hipStream_t s)
{
    switch (bits) {
    case 2: return compress_bits<2>(is_v, group, dtype, a, s);
    case 3: return compress_bits<3>(is_v, group, dtype, a, s);
    case 4: return compress_bits<4>(is_v, group, dtype, a, s);
    case 8: return compress_bits<8>(is_v, group, dtype, a, s);
    case 16: KVC_LAUNCH(copy_rows_kernel<true>, a, s);
    }
    return KVC_ERR_UNSUPPORTED;
}

template <int BITS, bool DENSE> static int decompress_bits_dense(int is_v, int dtype, const QuantArgs &a, hipStream_t s)
{
    if (!is_v) {
        if (dtype == DT_F16) KVC_LAUNCH((decompress_k_kernel<BITS, DT_F16, DENSE>), a, s);
        KVC_LAUNCH((decompress_k_kernel<BITS, DT_BF16, DENSE>), a, s);
    }
    if (dtype == DT_F16) KVC_LAUNCH((decompress_v_kernel<BITS, DT_F16, DENSE>), a, s);
    KVC_LAUNCH((decompress_v_kernel<BITS, DT_BF16, DENSE>), a, s);
}

template <int BITS> static int decompress_bits(int is_v, int dtype, const QuantArgs &a, hipStream_t s)
{
    return a.dense ? decompress_bits_dense<BITS, true>(is_v, dtype, a, s) : decompress_bits_dense<BITS, false>(is_v, dtype, a, s);
}

int launch_decompress_tensor(int is_v, int bits, int group, int dtype, const QuantArgs &a, hipStream_t s)
{
    (void)group;
    switch (bits) {
    case 2: return decompress_bits<2>(is_v, dtype, a, s);
    case 3: return decompress_bits<3>(is_v, dtype, a, s);
    case 4: return decompress_bits<4>(is_v, dtype, a, s);
    case 8: return decompress_bits<8>(is_v, dtype, a, s);
    case 16: KVC_LAUNCH(copy_rows_kernel<false>, a, s);
    }
    return KVC_ERR_UNSUPPORTED;
}

int launch_write_header(uint8_t *dst, const HeaderBytes &h, hipStream_t s)
{
    hipLaunchKernelGGL(write_header_kernel, dim3(1), dim3(64), 0, s, (uint32_t *)dst, h);
    return hipGetLastError() == hipSuccess ? KVC_OK : KVC_ERR_DEVICE;
}

int launch_check_header(const uint8_t *hdr, const HeaderBytes &expect, uint32_t mask, int *status, hipStream_t s)
{
    hipLaunchKernelGGL(check_header_kernel, dim3(1), dim3(64), 0, s, (const uint32_t *)hdr, expect, mask, status);
    return hipGetLastError() == hipSuccess ? KVC_OK : KVC_ERR_DEVICE;
}

int launch_check_bytes(const uint8_t *a, const uint8_t *b, long long n, int *status, hipStream_t s)
{
    if (n <= 0) return KVC_OK;
    hipLaunchKernelGGL(check_bytes_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, a, b, n, status);
    return hipGetLastError() == hipSuccess ? KVC_OK : KVC_ERR_DEVICE;
}

int launch_fill_u32(uint32_t *dst, uint32_t value, long long n, hipStream_t s)
{
    if (n <= 0) return KVC_OK;
    hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, dst, value, n);
    return hipGetLastError() == hipSuccess ? KVC_OK : KVC_ERR_DEVICE;
}

}  // namespace kvc
