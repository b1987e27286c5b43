// Exhaustive device-side checks of the arithmetic shortcuts the quantizer kernels rely on.
// Each check counts, over the whole domain on which the kernels use a shortcut, the inputs for
// which it differs from the plain IEEE operation it stands for; all counts must be zero.
#include "kvc_device.h"
#include "kvc_internal.h"
#include "../../include/kvc.h"

namespace kvc {

__device__ __forceinline__ void count(unsigned long long *slot, unsigned long long bad)
{
    // one atomic per wave
    const unsigned long long m = __builtin_amdgcn_ballot_w64(bad != 0);
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const uint32_t lo = (uint32_t)__builtin_amdgcn_ds_bpermute(((threadIdx.x & 63) ^ d) << 2, (int)(uint32_t)bad);
        bad += lo;
    }
    if (m != 0 && (threadIdx.x & 63) == 0) atomicAdd(slot, bad);
}

// range / (2^BITS - 1), limited to 65504 as the metadata stores it, for every non-negative float
// range including +infinity (max - min of two finite bfloat16 values can overflow).  fp16 input
// only reaches ranges up to 2 * 65504, where the limit never applies and the quotient itself is
// compared.
template <int BITS> __global__ __launch_bounds__(256) void selftest_div_kernel(unsigned long long *slot)
{
    constexpr float qmax = (float)((1 << BITS) - 1);
    const uint32_t last = 0x7f800000u;                     // +infinity
    unsigned long long bad = 0;
    for (unsigned long long u = blockIdx.x * 256ull + threadIdx.x; u <= last; u += gridDim.x * 256ull) {
        const float r = __uint_as_float((uint32_t)u);
        const float want = fminf(r / qmax, 65504.0f);      // correctly rounded division
        bad += __float_as_uint(fminf(rounded_f32(div_levels<BITS>(r)), 65504.0f)) != __float_as_uint(want);
    }
    count(slot, bad);
}

// 1 / s for every positive finite fp16 s
__global__ __launch_bounds__(256) void selftest_rcp_kernel(unsigned long long *slot)
{
    unsigned long long bad = 0;
    for (uint32_t h = blockIdx.x * 256u + threadIdx.x; h < 0x7c00u; h += gridDim.x * 256u) {
        if (h == 0) continue;
        const float s = f16_bits_to_f32(h);
        bad += __float_as_uint(rcp_f16_exact(s)) != __float_as_uint(1.0f / s);
    }
    count(slot, bad);
}

// x - zero for every pair of finite fp16 values (both halves of the packed register)
__global__ __launch_bounds__(256) void selftest_minus_kernel(unsigned long long *slot)
{
    unsigned long long bad = 0;
    const float one = opaque_one();
    const uint32_t zb = blockIdx.x;                        // one zero point per workgroup
    if ((zb & 0x7c00u) != 0x7c00u) {
        const float zero = f16_bits_to_f32(zb);
        for (uint32_t xb = threadIdx.x; xb < 0x10000u; xb += 256u) {
            if ((xb & 0x7c00u) == 0x7c00u) continue;
            const u32x4 r = {xb | (xb << 16), 0u, 0u, xb << 16};
            const float want = rounded_f32(f16_bits_to_f32(xb)) - zero;
            bad += __float_as_uint(elem_minus<DT_F16>(r, 0, zero, one)) != __float_as_uint(want);
            bad += __float_as_uint(elem_minus<DT_F16>(r, 1, zero, one)) != __float_as_uint(want);
            bad += __float_as_uint(elem_minus<DT_F16>(r, 7, zero, one)) != __float_as_uint(want);
        }
    }
    count(slot, bad);
}

// float -> byte conversion with insertion, for every float in [0, 255]: round to nearest even,
// placed in the selected byte, the other bytes kept
__global__ __launch_bounds__(256) void selftest_byte_kernel(unsigned long long *slot)
{
    const uint32_t last = 0x437f0000u;                     // 255.0f
    unsigned long long bad = 0;
    for (unsigned long long u = blockIdx.x * 256ull + threadIdx.x; u <= last; u += gridDim.x * 256ull) {
        const float t = __uint_as_float((uint32_t)u);
        const uint32_t want = (uint32_t)__builtin_rintf(t);
        const uint32_t keep = 0xa5c3961eu;
        bad += __builtin_amdgcn_cvt_pk_u8_f32(t, 0, keep) != ((keep & 0xffffff00u) | want);
        bad += __builtin_amdgcn_cvt_pk_u8_f32(t, 1, keep) != ((keep & 0xffff00ffu) | (want << 8));
        bad += __builtin_amdgcn_cvt_pk_u8_f32(t, 2, keep) != ((keep & 0xff00ffffu) | (want << 16));
        bad += __builtin_amdgcn_cvt_pk_u8_f32(t, 3, keep) != ((keep & 0x00ffffffu) | (want << 24));
    }
    count(slot, bad);
}

} // namespace kvc

extern "C" int kvc_selftest(uint64_t *counts, void *stream)
{
    using namespace kvc;
    if (counts == nullptr) return KVC_ERR_ARG;
    hipStream_t s = (hipStream_t)stream;
    unsigned long long *c = (unsigned long long *)counts;
    launch_fill_u32((uint32_t *)counts, 0u, 2 * KVC_SELFTEST_COUNTS, s);
    selftest_div_kernel<2><<<4096, 256, 0, s>>>(c + 0);
    selftest_div_kernel<3><<<4096, 256, 0, s>>>(c + 1);
    selftest_div_kernel<4><<<4096, 256, 0, s>>>(c + 2);
    selftest_div_kernel<8><<<4096, 256, 0, s>>>(c + 3);
    selftest_rcp_kernel<<<124, 256, 0, s>>>(c + 4);
    selftest_minus_kernel<<<65536, 256, 0, s>>>(c + 5);
    selftest_byte_kernel<<<4096, 256, 0, s>>>(c + 6);
    return hipGetLastError() == hipSuccess ? KVC_OK : KVC_ERR_DEVICE;
}
