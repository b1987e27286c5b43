// Shared pieces of the codec-free kernels: work-unit addressing and the launch helper.
// One wave per work unit, four units per workgroup.
#pragma once

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
    long long unit = (long long)blockIdx.x * 4 + wave_id();
    if (unit >= a.total_units) return false;
    if (a.head_minor) {
        // unit = (layer * units_per_head + block) * heads + head: the four waves of a workgroup read or
        // write the same token rows of four neighbouring heads, which are contiguous in memory
        const long long t = unit / a.heads;
        const long long l = t / a.units_per_head;
        u.blk = t - l * a.units_per_head;
        u.lh = l * a.heads + (unit - t * a.heads);
    } else {
        const long long slot = unit / a.units_per_head;
        u.lh = a.head_list ? a.head_list[slot] : slot;
        u.blk = unit - slot * a.units_per_head;
    }
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

// grid: x = workgroups of four units for the largest item, y = items
static inline dim3 grid_for(const QuantBatch &b)
{
    long long most = 0;
    for (int i = 0; i < b.n; ++i) most = b.item[i].total_units > most ? b.item[i].total_units : most;
    return dim3((unsigned)((most + 3) / 4), (unsigned)b.n);
}

#define KVC_LAUNCH(kernel, b, s)                                                        \
    do {                                                                                \
        const dim3 grid_ = grid_for(b);                                                 \
        if (grid_.x > 0 && grid_.y > 0)                                                 \
            hipLaunchKernelGGL(kernel, grid_, dim3(256), 0, s, b);                      \
        return hipGetLastError() == hipSuccess ? KVC_OK : KVC_ERR_DEVICE;               \
    } while (0)

}  // namespace kvc
