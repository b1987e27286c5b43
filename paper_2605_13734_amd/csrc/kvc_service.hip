// Service kernels of the library (header write / check, fills, the 16-bit pass-through copy) and
// the dispatch of the codec-free launches over the code widths.

#include "kvc_quant.h"

namespace kvc {

// ---- 16 bits: the tensor travels unchanged ----------------------------------------------------

template <bool TO_PAYLOAD>
__global__ __launch_bounds__(256) void copy_rows_kernel(QuantBatch batch)
{
    unsigned wg;
    const QuantArgs &a = batch.item[batch_item(batch, wg)];
    UnitPos u;
    if (!unit_pos(a, wg, u)) return;
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

// ---- service kernels: everything of a call that is not a tensor pass, for all requests at once ----

// Before compression: the request's status word and header, the zero padding between the parts
// of the payload, the width tables (copied from their device image), the coder's histograms,
// work-order counter and scan state, and whatever the host already knows of the result (the
// payload size without the coder; the closed directory of an empty request).
// grid = (slices, requests); the zero fills are spread over the slices.
__global__ __launch_bounds__(256) void compress_prologue_kernel(PrologueArgs a)
{
    const PrologueItem &it = a.item[blockIdx.y];
    const long long first = (long long)blockIdx.x * 256 + threadIdx.x, step = (long long)gridDim.x * 256;
    if (blockIdx.x == 0) {
        const int t = threadIdx.x;
        if (t < 32) it.payload[t] = it.header.w[t];
        if (t == 32) *it.status = 0;
        if (t == 33 && it.write_total) *it.out_bytes = it.total;
        if (t == 34 && it.dir0) *it.dir0 = 0;
    }
    for (int k = 0; k < 2; ++k)
        for (long long i = first; i < it.pad_words[k]; i += step) it.payload[it.pad_off[k] / 4 + i] = 0;
    for (long long i = first; i < it.aux_words; i += step) it.payload[it.aux_off / 4 + i] = it.aux_src[i];
    for (int k = 0; k < 2; ++k)
        for (long long i = first; i < it.zero_words[k]; i += step) it.zero[k][i] = 0;
}

// Before decompression: the status word of every request, set to KVC_DEV_BAD_HEADER when the
// payload's header (the words selected by `mask`) or its width tables differ from the plan's.
// grid = requests, one workgroup each.
__global__ __launch_bounds__(256) void decompress_prologue_kernel(CheckArgs a)
{
    const CheckItem &it = a.item[blockIdx.x];
    const int t = threadIdx.x;
    int diff = t < 32 && ((it.mask >> t) & 1u) && it.payload[t] != it.expect.w[t];
    for (long long i = t; i < it.table_bytes; i += 256) diff |= it.tables[i] != it.plan_tables[i];
    diff = __syncthreads_or(diff);
    if (t == 0) *it.status = diff ? KVC_DEV_BAD_HEADER : 0;
}

__global__ void fill_u32_kernel(uint32_t *dst, uint32_t value, long long n)
{
    long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = value;
}

// ---- launchers ----------------------------------------------------------------------------------

int launch_compress_tensor(int is_v, int bits, int group, int dtype, const QuantBatch &b, hipStream_t s)
{
    switch (bits) {
    case 2: return launch_compress_bits2(is_v, group, dtype, b, s);
    case 3: return launch_compress_bits3(is_v, group, dtype, b, s);
    case 4: return launch_compress_bits4(is_v, group, dtype, b, s);
    case 8: return launch_compress_bits8(is_v, group, dtype, b, s);
    case 16: KVC_LAUNCH(copy_rows_kernel<true>, b, s);
    }
    return KVC_ERR_UNSUPPORTED;
}

int launch_decompress_tensor(int is_v, int bits, int group, int dtype, const QuantBatch &b, hipStream_t s)
{
    (void)group;
    switch (bits) {
    case 2: return launch_decompress_bits2(is_v, dtype, b, s);
    case 3: return launch_decompress_bits3(is_v, dtype, b, s);
    case 4: return launch_decompress_bits4(is_v, dtype, b, s);
    case 8: return launch_decompress_bits8(is_v, dtype, b, s);
    case 16: KVC_LAUNCH(copy_rows_kernel<false>, b, s);
    }
    return KVC_ERR_UNSUPPORTED;
}

int launch_compress_prologue(const PrologueArgs &a, hipStream_t s)
{
    long long most = 1;
    for (int i = 0; i < a.n; ++i)
        for (int k = 0; k < 2; ++k) most = a.item[i].zero_words[k] > most ? a.item[i].zero_words[k] : most;
    long long slices = (most + 4095) / 4096;           // 16 words per thread
    slices = slices < 1 ? 1 : (slices > 256 ? 256 : slices);
    hipLaunchKernelGGL(compress_prologue_kernel, dim3((unsigned)slices, (unsigned)a.n), dim3(256), 0, s, a);
    return hipGetLastError() == hipSuccess ? KVC_OK : KVC_ERR_DEVICE;
}

int launch_decompress_prologue(const CheckArgs &a, hipStream_t s)
{
    hipLaunchKernelGGL(decompress_prologue_kernel, dim3((unsigned)a.n), dim3(256), 0, s, a);
    return hipGetLastError() == hipSuccess ? KVC_OK : KVC_ERR_DEVICE;
}

int launch_fill_u32(uint32_t *dst, uint32_t value, long long n, hipStream_t s)
{
    if (n <= 0) return KVC_OK;
    hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, dst, value, n);
    return hipGetLastError() == hipSuccess ? KVC_OK : KVC_ERR_DEVICE;
}

}  // namespace kvc
