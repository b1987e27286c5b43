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

__device__ __forceinline__ bool unit_pos(const QuantArgs &a, unsigned wg, UnitPos &u)
{
    long long unit = (long long)wg * 4 + wave_id();
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

// workgroups of four units, item after item
static inline unsigned place_items(QuantBatch &b)
{
    unsigned at = 0;
    for (int i = 0; i < b.n; ++i) {
        b.start[i] = at;
        at += (unsigned)((b.item[i].total_units + 3) / 4);
    }
    b.start[b.n] = at;
    return at;
}

#define KVC_LAUNCH(kernel, batch, s)                                                    \
    do {                                                                                \
        QuantBatch placed_ = batch;                                                     \
        const unsigned wgs_ = place_items(placed_);                                     \
        if (wgs_ > 0) hipLaunchKernelGGL(kernel, dim3(wgs_), dim3(256), 0, s, placed_); \
        return hipGetLastError() == hipSuccess ? KVC_OK : KVC_ERR_DEVICE;               \
    } while (0)

}  // namespace kvc
