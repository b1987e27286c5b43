// Measurement aid (kvc_stream_probe): kernels that move the bytes of a tensor pass in the same
// shape as the quantizer / coder kernels do -- one wave per 128 token rows, 16 bytes per lane and
// access, four serial passes of 32 rows on the 16-bit side, the payload side in 16-byte pieces --
// and do no arithmetic beyond folding the loaded words into the stored ones.  What they reach is
// the practical ceiling of the memory system for this access pattern, which the benchmark prints
// beside the published HBM peak.

#include "kvc_internal.h"
#include "../../include/kvc.h"

namespace kvc {

// MODE 0: read 128 rows x 256 B, write `out_row` bytes per row (the compress direction).
// MODE 1: read `out_row` bytes per row, write 128 rows x 256 B (the decompress direction).
template <int MODE>
__global__ __launch_bounds__(256) void stream_probe_kernel(const uint8_t *src, uint8_t *dst, long long chunks, int out_row)
{
    const long long chunk = (long long)blockIdx.x * 4 + wave_id();
    if (chunk >= chunks) return;
    const int lane = lane_id();
    const long long wide = (long long)kChunkRows * kDim * 2, narrow = (long long)kChunkRows * out_row;
    if (MODE == 0) {
        const u32x4 *p = (const u32x4 *)(src + chunk * wide) + lane;
        u32x4 acc = {0, 0, 0, 0};
#pragma unroll 1
        for (int pass = 0; pass < 4; ++pass) {
            u32x4 v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = __builtin_nontemporal_load(p + (pass * 8 + i) * 64);
#pragma unroll
            for (int i = 0; i < 8; ++i) acc ^= v[i];
        }
        u32x4 *q = (u32x4 *)(dst + chunk * narrow);
        for (int k = lane; k * 16 < narrow; k += 64) q[k] = acc;
    } else {
        const u32x4 *p = (const u32x4 *)(src + chunk * narrow);
        u32x4 acc = {0, 0, 0, 0};
        for (int k = lane; k * 16 < narrow; k += 64) acc ^= __builtin_nontemporal_load(p + k);
        u32x4 *q = (u32x4 *)(dst + chunk * wide) + lane;
#pragma unroll 1
        for (int pass = 0; pass < 4; ++pass) {
#pragma unroll
            for (int i = 0; i < 8; ++i) __builtin_nontemporal_store(acc, q + (pass * 8 + i) * 64);
        }
    }
}

}  // namespace kvc

extern "C" int kvc_stream_probe(int mode, const void *src, void *dst, int64_t rows, int32_t payload_row_bytes,
                                void *hip_stream)
{
    using namespace kvc;
    if (!src || !dst || ((uintptr_t)src & 15) || ((uintptr_t)dst & 15)) return KVC_ERR_ARG;
    if ((mode != 0 && mode != 1) || rows < 0 || (rows % kChunkRows) != 0) return KVC_ERR_ARG;
    if (payload_row_bytes < 16 || payload_row_bytes > 256 || (payload_row_bytes & 15)) return KVC_ERR_ARG;
    const long long chunks = rows / kChunkRows;
    if (chunks == 0) return KVC_OK;
    if (chunks > (1ll << 32)) return KVC_ERR_CAPACITY;
    hipStream_t s = (hipStream_t)hip_stream;
    const dim3 grid((unsigned)((chunks + 3) / 4));
    if (mode == 0) hipLaunchKernelGGL(stream_probe_kernel<0>, grid, dim3(256), 0, s, (const uint8_t *)src, (uint8_t *)dst, chunks, payload_row_bytes);
    else hipLaunchKernelGGL(stream_probe_kernel<1>, grid, dim3(256), 0, s, (const uint8_t *)src, (uint8_t *)dst, chunks, payload_row_bytes);
    return hipGetLastError() == hipSuccess ? KVC_OK : KVC_ERR_DEVICE;
}
