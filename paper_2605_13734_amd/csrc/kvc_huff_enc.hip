// Lossless stage, encoder: quantize + pack + Huffman-code one chunk per wave and place the body
// through a single-pass prefix sum over workgroups.  Compiled once per code width (-DKVC_BITS=2, 3,
// 4 or 8).  See kvc_huff.h for the format and the division of work.

#include "kvc_huff.h"

#ifndef KVC_BITS
#error "compile with -DKVC_BITS=2, 3, 4 or 8"
#endif

namespace kvc {

// ---- encoder ---------------------------------------------------------------------------------

// Encoder tables in LDS: code lengths as bytes, and code | length << 12 as 16-bit entries
// (narrow entries keep the hot byte values of a section in distinct banks).
struct EncTables {
    uint8_t len[256];
    uint16_t code[256];
};

// bit count of HALF (0 or 1) of the lane's sub-block
template <int W> __device__ __forceinline__ uint32_t half_bits(const uint32_t *sym, const EncTables &t, int half)
{
    uint32_t bits = 0;
#pragma unroll
    for (int k = 0; k < W / 2; ++k) {
        const uint32_t w = sym[half * (W / 2) + k];
#pragma unroll
        for (int b = 0; b < 4; ++b) bits += t.len[(w >> (8 * b)) & 255u];
    }
    return bits;
}

struct BitWriter {
    unsigned long long acc;
    uint32_t nbits;
    uint32_t *out;       // next word (LDS)
};

__device__ __forceinline__ void writer_start(BitWriter &bw, uint32_t *words, uint32_t bit)
{
    bw.acc = 0;
    bw.nbits = bit & 31;          // the leading bits of the first word belong to the previous stream
    bw.out = words + (bit >> 5);
}

__device__ __forceinline__ void put(BitWriter &bw, uint32_t e)
{
    const uint32_t len = e >> 12;
    bw.acc = (bw.acc << len) | (e & 0xfffu);
    bw.nbits += len;
}

__device__ __forceinline__ void flush(BitWriter &bw)
{
    if (bw.nbits >= 32) {
        atomicOr(bw.out, (uint32_t)(bw.acc >> (bw.nbits - 32)));
        ++bw.out;
        bw.nbits -= 32;
    }
}

__device__ __forceinline__ void writer_finish(BitWriter &bw)
{
    if (bw.nbits > 0) atomicOr(bw.out, (uint32_t)(bw.acc << (32 - bw.nbits)));
}

// Code the words [first, first + n) of the lane's sub-block.  Words of streams that share a
// boundary word are merged with LDS atomic OR (the region is zeroed beforehand).
template <int N> __device__ __forceinline__ void encode_words(const uint32_t *sym, const EncTables &t, BitWriter &bw)
{
#pragma unroll
    for (int k = 0; k < N; ++k) {
        const uint32_t w = sym[k];
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            put(bw, t.code[(w >> (8 * b)) & 255u]);
            if (b & 1) flush(bw);          // at most 24 new bits between checks
        }
    }
}

// Both halves of the sub-block as two independent streams (instruction-level parallelism).
template <int W> __device__ __forceinline__ void encode_two(const uint32_t *sym, const EncTables &t, BitWriter &b0, BitWriter &b1)
{
#pragma unroll
    for (int k = 0; k < W / 2; ++k) {
        const uint32_t w0 = sym[k], w1 = sym[W / 2 + k];
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            put(b0, t.code[(w0 >> (8 * b)) & 255u]);
            put(b1, t.code[(w1 >> (8 * b)) & 255u]);
            if (b & 1) { flush(b0); flush(b1); }
        }
    }
}

// One workgroup = kWaves chunks.  A chunk's body offset is the sum of all earlier bodies of the
// request (K chunks first, then V): a single-pass scan over one state word per workgroup.
// Workgroups take a ticket from a counter; wave 0 publishes the workgroup's total size, looks
// back over earlier tickets until it meets one that knows its inclusive prefix, and publishes
// its own.  Ticket order guarantees that every predecessor is already running, so the wait
// always ends; it is bounded by kSpinLimit all the same.
// Waves per SIMD the register allocation must leave room for: four where the workgroup has 512
// threads (see enc_waves); the other variants would spill, so they keep what they need.
template <int BITS, int G, int DT, bool IS_V, bool DENSE, bool XF> constexpr int enc_min_waves()
{
    return enc_waves(BITS, G, DT, DENSE, IS_V, XF) == 8 ? 4 : 1;
}

template <int BITS, int G, int DT, bool IS_V, bool DENSE, bool XF>
__global__ __launch_bounds__(enc_waves(BITS, G, DT, DENSE, IS_V, XF) * 64)
__attribute__((amdgpu_waves_per_eu(enc_min_waves<BITS, G, DT, IS_V, DENSE, XF>())))
void encode_kernel(CoderBatch batch)
{
    using Geo = ChunkGeom<BITS>;
    constexpr int W = Geo::kWords, NW = enc_waves(BITS, G, DT, DENSE, IS_V, XF);
    unsigned wg;
    const CoderArgs &a = batch.item[batch_item(batch, wg)];      // (which of them it is among the item's workgroups does not matter: the chunk comes from the ticket)
    (void)wg;
    __shared__ __attribute__((aligned(16))) uint8_t lds_all[NW * Geo::kLds];
    __shared__ EncTables enc;
    __shared__ uint32_t s_units[NW];
    __shared__ unsigned long long s_excl;
    __shared__ uint32_t s_ticket;

    const int tid = threadIdx.x, wave = wave_id(), lane = lane_id();
    if (tid == 0) s_ticket = atomicAdd(a.ws.ticket, 1u);
    for (int k = tid; k < 256; k += NW * 64) {
        const uint32_t e = a.ws.enc[256 * a.tab + k];             // code | length << 16
        enc.len[k] = (uint8_t)(e >> 16);
        enc.code[k] = (uint16_t)((e & 0xfffu) | ((e >> 16) << 12));
    }
    __syncthreads();
    const long long ticket = (unsigned)__builtin_amdgcn_readfirstlane((int)s_ticket);     // global order over K and V workgroups (the same in all lanes)
    const long long chunk = (ticket - a.wg_base) * NW + wave;
    const bool live = chunk < a.chunks;
    uint8_t *lds = lds_all + wave * Geo::kLds;

    uint32_t body_units = 0;      // body size in 16-byte units
    bool coded = false;
    int rows = 0;
    uint32_t sym[W];
    if (live) {
        ChunkPos c = chunk_pos(a.q, chunk);
        rows = c.rows;
        bool bad = false;
        quantize_chunk<BITS, G, DT, IS_V, DENSE, XF>(a.q, c, lds, true, bad);
        if (bad) atomicOr(a.q.status, KVC_DEV_BAD_BLOCK);
        wave_sync();
        load_sub<BITS>(lds, sym);
        const int have = min(max(rows - 2 * lane, 0), 2);        // valid rows of this sub-block
        uint32_t bits0 = 0, bits = 0;
        if (have > 0) bits0 = half_bits<W>(sym, enc, 0);
        bits = bits0;
        if (have > 1) bits += half_bits<W>(sym, enc, 1);
        const uint32_t incl = wave_inclusive_sum(bits);
        const uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
        const uint32_t raw_bytes = (uint32_t)rows * Geo::kRowBytes;
        const uint32_t coded_bytes = (2 * kSubs + 4 * ((total + 31) / 32) + 15) & ~15u;
        coded = coded_bytes < raw_bytes;
        body_units = (coded ? coded_bytes : raw_bytes) / 16;
        // the size goes out before the code words are written, so that successors see this
        // workgroup's aggregate as early as possible
        if (lane == 0)
            __hip_atomic_fetch_add(&a.ws.state[ticket], ((unsigned long long)(kAggComplete / NW) << kAggShift) | body_units,
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (coded) {
            wave_sync();                                          // every lane holds its symbols
            u32x4 zero = {0, 0, 0, 0};
            for (uint32_t o = lane * 16; o < coded_bytes; o += 64 * 16) *(u32x4 *)(lds + o) = zero;
            wave_sync();
            ((uint16_t *)lds)[lane] = (uint16_t)bits;
            const uint32_t start = incl - bits;
            uint32_t *words = (uint32_t *)(lds + 2 * kSubs);
            if (have > 1) {
                BitWriter b0, b1;
                writer_start(b0, words, start);
                writer_start(b1, words, start + bits0);
                encode_two<W>(sym, enc, b0, b1);
                writer_finish(b0);
                writer_finish(b1);
            } else if (have > 0) {
                BitWriter b0;
                writer_start(b0, words, start);
                encode_words<W / 2>(sym, enc, b0);
                writer_finish(b0);
            }
            wave_sync();
        }
    }
    if (!live && lane == 0)
        __hip_atomic_fetch_add(&a.ws.state[ticket], (unsigned long long)(kAggComplete / NW) << kAggShift, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
    if (lane == 0) s_units[wave] = body_units;
    __syncthreads();

    // ---- single-pass prefix sum over workgroups, in ticket order ------------------------------
    if (wave == 0) {
        unsigned long long agg = 0;
        for (int w = 0; w < NW; ++w) agg += s_units[w];
        unsigned long long excl = 0;
        bool timeout = false;
        if (ticket > 0) {
            long long idx = ticket - 1;
            int spins = 0;
            for (;;) {
                const long long j = idx - lane;
                unsigned long long v = kFlagPrefix;
                if (j >= 0) v = __hip_atomic_load(&a.ws.state[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                // 2: inclusive prefix, 1: complete aggregate, 0: not all waves have reported yet
                const unsigned flag = (v >> 62) == 2 ? 2u : ((unsigned)(v >> kAggShift) & 0xffu) == (unsigned)kAggComplete ? 1u : 0u;
                if (__builtin_amdgcn_ballot_w64(flag == 0) != 0) {
                    if (++spins > kSpinLimit) { timeout = true; break; }
                    __builtin_amdgcn_s_sleep(8);
                    continue;
                }
                const unsigned long long pm = __builtin_amdgcn_ballot_w64(flag == 2);
                const int stop = pm ? __builtin_ctzll(pm) : 63;      // nearest predecessor with a full prefix
                unsigned long long part = (lane <= stop) ? (v & kValueMask) : 0;
#pragma unroll
                for (int d = 32; d >= 1; d >>= 1) {
                    const uint32_t lo = (uint32_t)__builtin_amdgcn_ds_bpermute((lane ^ d) << 2, (int)(uint32_t)part);
                    const uint32_t hi = (uint32_t)__builtin_amdgcn_ds_bpermute((lane ^ d) << 2, (int)(uint32_t)(part >> 32));
                    part += ((unsigned long long)hi << 32) | lo;
                }
                excl += part;
                if (pm) break;
                idx -= 64;
            }
        }
        if (timeout) {
            excl = 0;
            if (lane == 0) atomicOr(a.q.status, KVC_DEV_SCAN_TIMEOUT);
        }
        if (lane == 0) {
            __hip_atomic_store(&a.ws.state[ticket], kFlagPrefix | ((excl + agg) & kValueMask), __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
            s_excl = timeout ? ~0ull : excl;
            if (ticket == a.total_wgs - 1 && !timeout) {
                // the very last workgroup closes the directory and the header
                const unsigned long long all = excl + agg;
                uint32_t *dir = (uint32_t *)(a.payload + a.off_dir);
                dir[a.total_chunks] = (uint32_t)all;
                unsigned long long k_units = all;          // (this is the last K workgroup only if V has no chunks)
                if (IS_V)
                    k_units = a.k_wgs > 0 ? __hip_atomic_load(&a.ws.state[a.k_wgs - 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & kValueMask : 0;
                const unsigned long long total = (unsigned long long)a.off_bodies + all * 16;
                unsigned long long *h = (unsigned long long *)a.payload;
                h[5] = total;                                   // byte 40: total bytes
                h[13] = k_units * 16;                           // byte 104: K code bytes
                h[14] = (unsigned long long)a.off_bodies + k_units * 16;   // byte 112: V code offset
                h[15] = (all - k_units) * 16;                   // byte 120: V code bytes
                *a.out_bytes = total;
            }
        }
    }
    __syncthreads();
    const unsigned long long excl = s_excl;
    if (!live || excl == ~0ull) return;
    unsigned long long mine = excl;
    for (int w = 0; w < wave; ++w) mine += s_units[w];
    if (lane == 0) ((uint32_t *)(a.payload + a.off_dir))[a.chunk_base + chunk] = (uint32_t)mine;
    uint8_t *dst = a.payload + a.off_bodies + mine * 16;
    if ((long long)(a.off_bodies + (mine + body_units) * 16) > a.capacity) return;      // cannot happen: bodies never exceed raw size
    if (coded) {
        for (uint32_t o = lane * 16; o < body_units * 16; o += 64 * 16) *(u32x4 *)(dst + o) = *(const u32x4 *)(lds + o);
    } else {
        // raw chunk: each lane still holds its sub-block (2 rows) in registers
        const int have = min(max(rows - 2 * lane, 0), 2);
        u32x4 *p = (u32x4 *)(dst + lane * Geo::kSubBytes);
#pragma unroll
        for (int k = 0; k < W / 4; ++k)
            if (k * 2 < have * (W / 4)) {
                u32x4 v;
                v[0] = sym[4 * k]; v[1] = sym[4 * k + 1]; v[2] = sym[4 * k + 2]; v[3] = sym[4 * k + 3];
                p[k] = v;
            }
    }
}

// ---- launchers ----------------------------------------------------------------------------------

template <int BITS, int G, int DT, bool IS_V> static int encode_launch(const CoderBatch &b, hipStream_t s)
{
    const CoderArgs &a = b.item[0];
    const int NW = enc_waves(BITS, G, DT, a.q.dense != 0, IS_V, a.q.rotate || a.q.anchors != nullptr);
    CoderBatch placed = b;
    unsigned need = 0;
    for (int i = 0; i < b.n; ++i) {
        placed.start[i] = need;
        need += (unsigned)((b.item[i].chunks + NW - 1) / NW);
    }
    placed.start[b.n] = need;
    if (need == 0) return KVC_OK;
    const dim3 grid(need), block(NW * 64);
    // K token blocks of 64 and 128 rows, and V groups of 32 channels (the variant that is short of
    // registers), have a kernel of their own for launches without a transform
    constexpr bool kSplit = IS_V ? G == 32 : G >= 64;
    if (kSplit && !a.q.rotate && !a.q.anchors) {
        if (a.q.dense) hipLaunchKernelGGL((encode_kernel<BITS, G, DT, IS_V, true, !kSplit>), grid, block, 0, s, placed);
        else hipLaunchKernelGGL((encode_kernel<BITS, G, DT, IS_V, false, !kSplit>), grid, block, 0, s, placed);
        return launched();
    }
    if (a.q.dense) hipLaunchKernelGGL((encode_kernel<BITS, G, DT, IS_V, true, true>), grid, block, 0, s, placed);
    else hipLaunchKernelGGL((encode_kernel<BITS, G, DT, IS_V, false, true>), grid, block, 0, s, placed);
    return launched();
}

template <int DT, bool ISV> static int encode_g(int group, const CoderBatch &a, hipStream_t s)
{
    switch (group) {
    case 32: return encode_launch<KVC_BITS, 32, DT, ISV>(a, s);
    case 64: return encode_launch<KVC_BITS, 64, DT, ISV>(a, s);
    case 128: return encode_launch<KVC_BITS, 128, DT, ISV>(a, s);
    }
    return KVC_ERR_UNSUPPORTED;
}

#define KVC_PASTE2(a, b) a##b
#define KVC_PASTE(a, b) KVC_PASTE2(a, b)

int KVC_PASTE(launch_encode_bits, KVC_BITS)(int group, int dtype, const CoderBatch &a, hipStream_t s)
{
    if (a.item[0].is_v) return dtype == DT_F16 ? encode_g<DT_F16, true>(group, a, s) : encode_g<DT_BF16, true>(group, a, s);
    return dtype == DT_F16 ? encode_g<DT_F16, false>(group, a, s) : encode_g<DT_BF16, false>(group, a, s);
}

}  // namespace kvc
