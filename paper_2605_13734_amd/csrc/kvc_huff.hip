// Lossless stage (codec C of the pipeline, KVServe section 5.1) fused with the quantizer:
// canonical, length-limited Huffman coding of the packed code bytes.
//
// Format (per section K or V): chunks of 128 token rows of one head; a chunk body is
// 64 x u16 sub-block bit counts (a sub-block = 2 rows), then the code words, most
// significant bit first in 32-bit little-endian words, sub-blocks back to back, padded
// to 16 bytes -- or the raw packed bytes when that is not smaller.  Bodies are stored
// back to back; a directory of running offsets (16-byte units) locates them.
//
// One wave owns one chunk: it quantizes the chunk into LDS, every lane then codes one
// sub-block, and the body is copied to its final place, which comes from a single-pass
// prefix sum over workgroups (ticket order + look-back on a state word per workgroup).
// Decoding mirrors it: body -> LDS, every lane decodes one sub-block with a 4096-entry
// table, the packed rows are rebuilt in LDS and dequantized from there.

#include "kvc_internal.h"
#include "kvc_tile.h"
#include "../../include/kvc.h"

namespace kvc {

// Optional per-phase cycle counts of the coder kernels (development builds only: compile with
// -DKVC_PHASE_CLOCKS and read g_phase_clocks through kvc_phase_clocks).
#ifdef KVC_PHASE_CLOCKS
__device__ unsigned long long g_phase_clocks[1024][2][16];      // rows spread the atomics
#define PHASE_START()                                             \
    unsigned long long phase_t = clock64(), phase_acc[8] = {0, 0, 0, 0, 0, 0, 0, 0}
#define PHASE(k, i)                                               \
    do {                                                          \
        const unsigned long long phase_n = clock64();             \
        phase_acc[i] += phase_n - phase_t;                        \
        phase_t = phase_n;                                        \
    } while (0)
#define PHASE_END(k)                                                                              \
    do {                                                                                          \
        if (lane_id() == 0)                                                                       \
            for (int i = 0; i < 8; ++i)                                                           \
                if (phase_acc[i]) atomicAdd(&g_phase_clocks[blockIdx.x & 1023][k][i], phase_acc[i]); \
    } while (0)
#else
#define PHASE_START() do {} while (0)
#define PHASE(k, i) do {} while (0)
#define PHASE_END(k) do {} while (0)
#endif


// Scan state of a workgroup: bits 63:62 = 2 once its inclusive prefix (bits 0..39) is known.
// Before that, every wave adds its chunk's size to bits 0..39 and its share of kAggComplete to
// the arrival count in bits 40..47; the sum of sizes is the workgroup's aggregate once the
// count is complete.  Sizes and prefixes are in 16-byte units.
constexpr unsigned long long kFlagPrefix = 2ull << 62, kValueMask = (1ull << 40) - 1;
constexpr int kAggShift = 40, kAggComplete = 4;
constexpr int kSpinLimit = 1 << 20;

template <int BITS> struct ChunkGeom {
    static constexpr int kRowBytes = 16 * BITS;            // packed bytes of one token row
    static constexpr int kSubBytes = 2 * kRowBytes;        // one sub-block
    static constexpr int kSubStride = kSubBytes + 16;      // LDS stride (bank spread, 16-byte aligned)
    static constexpr int kWords = kSubBytes / 4;           // words a lane holds for its sub-block
    static constexpr int kLds = kSubs * kSubStride;        // LDS bytes per wave
    static constexpr int kWaves = BITS == 8 ? 2 : 4;       // encoder: waves (= chunks) per workgroup
    static constexpr int kDecWaves = BITS == 8 ? 2 : 4;    // decoder: waves per workgroup (they share the 8 KB table)
};

// The decoder's LDS layout of a chunk.  4-bit codes: sub-blocks without padding, pieces rotated
// (fetch_codes, LAYOUT 2), 8 KB per wave, so that four workgroups of four waves and their 8 KB
// tables fill a compute unit's 160 KB exactly.  Other widths: the encoder's padded layout.
template <int BITS> struct DecGeom {
    static constexpr bool kRotated = BITS == 4;
    static constexpr int kLayout = kRotated ? 2 : 1;
    static constexpr int kStride = kRotated ? ChunkGeom<BITS>::kSubBytes : ChunkGeom<BITS>::kSubStride;
    static constexpr int kLds = kSubs * kStride;
    // address of 16-byte piece `piece` of sub-block `sub`
    static __device__ __forceinline__ uint8_t *piece_ptr(uint8_t *lds, uint32_t sub, uint32_t piece)
    {
        if (kRotated) return lds + sub * kStride + (((piece + sub) & 7u) << 4);
        return lds + sub * kStride + piece * 16;
    }
};

// ---- chunk <-> LDS -------------------------------------------------------------------------

template <int BITS> __device__ __forceinline__ uint8_t *lds_row(uint8_t *lds, int r)
{
    return code_row<BITS, true>(lds, r);
}

struct ChunkPos {
    long long lh, cb, head_off, row0;
    int rows;
};

__device__ __forceinline__ ChunkPos chunk_pos(const QuantArgs &a, long long chunk)
{
    ChunkPos c;
    const long long cph = (a.tokens + kChunkRows - 1) / kChunkRows;
    c.lh = chunk / cph;
    c.cb = chunk - c.lh * cph;
    const long long l = c.lh / a.heads, h = c.lh - l * a.heads;
    c.head_off = l * a.x.stride_layer + h * a.x.stride_head;
    c.row0 = c.cb * kChunkRows;
    const long long left = a.tokens - c.row0;
    c.rows = left < kChunkRows ? (int)left : kChunkRows;
    return c;
}

// Quantize and pack the chunk's rows into the wave's LDS region (sub-block layout) and,
// when `write_meta`, store the group metadata to the payload.  K group parameters are
// exchanged through the 16 padding bytes that follow each sub-block.
// XF = false leaves the code of stage T out (for launches that have no transform): in one kernel
// with the plain path it costs the plain path its registers, most of all for token blocks of 64
// and 128 rows.
template <int BITS, int G, int DT, bool IS_V, bool DENSE, bool XF = true>
__device__ __forceinline__ void quantize_chunk(const QuantArgs &a, const ChunkPos &c, uint8_t *lds, bool write_meta,
                                               bool &bad)
{
    constexpr int RU = IS_V ? kPassRows : G, PU = RU / kPassRows, NU = kChunkRows / RU;
#pragma unroll 1
    for (int u = 0; u < NU; ++u) {
        if (u * RU >= c.rows) break;
        const long long row0 = c.row0 + u * RU;
        u32x4 raw[PU * 8];
#pragma unroll
        for (int p = 0; p < PU; ++p) load_pass<DENSE>(a.x, c.head_off, row0 + p * kPassRows, a.tokens, raw + p * 8, bad);
        if (XF && a.rotate) rotate_rows<DT, PU * 8>(raw);
        if (XF && a.anchors)
            delta_rows<DT, DENSE, PU * 8>(a.x, c.head_off, row0, a.tokens, a.anchor_shift,
                                          head_anchors(a.anchors, c.lh, a.tokens, a.anchor_shift), write_meta, raw, bad);
        if (!IS_V) {
            const long long nb = (a.tokens + G - 1) / G;
            KParams kp;
            uint8_t *meta_block = write_meta ? a.meta + (c.lh * nb + row0 / G) * (kDim * 4) : nullptr;
            k_group_params<BITS, DT, PU * 8, ChunkGeom<BITS>::kSubStride>(raw, lds + ChunkGeom<BITS>::kSubBytes, meta_block, kp);
            k_emit<BITS, DT, PU, true>(raw, kp, code_row<BITS, true>(lds, u * RU), c.rows - u * RU);
        } else {
            constexpr int NG = kDim / G;
            VParams vp;
            v_pass_params<BITS, G, DT>(raw, vp);
            uint32_t *meta = write_meta ? (uint32_t *)a.meta + (c.lh * a.tokens + row0) * NG : nullptr;
            v_emit<BITS, G, DT, true>(raw, vp, code_row<BITS, true>(lds, u * RU), c.rows - u * RU, meta);
        }
    }
}

// The lane's sub-block (rows 2*lane, 2*lane+1) from LDS into registers.
template <int BITS> __device__ __forceinline__ void load_sub(const uint8_t *lds, uint32_t *sym)
{
    constexpr int W = ChunkGeom<BITS>::kWords;
    const u32x4 *p = (const u32x4 *)(lds + lane_id() * ChunkGeom<BITS>::kSubStride);
#pragma unroll
    for (int k = 0; k < W / 4; ++k) {
        u32x4 v = p[k];
        sym[4 * k] = v[0]; sym[4 * k + 1] = v[1]; sym[4 * k + 2] = v[2]; sym[4 * k + 3] = v[3];
    }
}

template <int BITS> __device__ __forceinline__ void store_sub(uint8_t *lds, const uint32_t *sym)
{
    constexpr int W = ChunkGeom<BITS>::kWords;
    u32x4 *p = (u32x4 *)(lds + lane_id() * ChunkGeom<BITS>::kSubStride);
#pragma unroll
    for (int k = 0; k < W / 4; ++k) {
        u32x4 v;
        v[0] = sym[4 * k]; v[1] = sym[4 * k + 1]; v[2] = sym[4 * k + 2]; v[3] = sym[4 * k + 3];
        p[k] = v;
    }
}

// inclusive prefix sum over the 64 lanes
__device__ __forceinline__ uint32_t wave_inclusive_sum(uint32_t v)
{
    const int lane = lane_id();
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint32_t o = (uint32_t)__builtin_amdgcn_ds_bpermute((lane - d) << 2, (int)v);
        if (lane >= d) v += o;
    }
    return v;
}

// ---- table sample: histogram of up to 16 chunks per section ------------------------------------

template <int BITS, int G, int DT, bool IS_V>
__global__ __launch_bounds__(64) void hist_kernel(CoderArgs a)
{
    __shared__ __attribute__((aligned(16))) uint8_t lds[ChunkGeom<BITS>::kLds];
    __shared__ uint32_t hist[256];
    const int i = blockIdx.x, lane = lane_id();
    const long long n = a.chunks;
    const long long chunk = (long long)i * n / 16;
    if (i > 0 && (long long)(i - 1) * n / 16 == chunk) return;      // each chunk counted once
    for (int k = lane; k < 256; k += 64) hist[k] = 0;
    ChunkPos c = chunk_pos(a.q, chunk);
    bool bad = false;
    quantize_chunk<BITS, G, DT, IS_V, false>(a.q, c, lds, false, bad);
    wave_sync();
    constexpr int W = ChunkGeom<BITS>::kWords;
    uint32_t sym[W];
    load_sub<BITS>(lds, sym);
    const int valid = min(max(c.rows - 2 * lane, 0), 2) * (W / 2);
#pragma unroll
    for (int k = 0; k < W; ++k)
        if (k < valid) {
#pragma unroll
            for (int b = 0; b < 4; ++b) atomicAdd(&hist[(sym[k] >> (8 * b)) & 255u], 1u);
        }
    wave_sync();
    uint32_t *g = a.ws.hist + (IS_V ? 256 : 0);
    for (int k = lane; k < 256; k += 64)
        if (hist[k]) atomicAdd(&g[k], hist[k]);
}

// ---- code construction (one wave per section) ---------------------------------------------------

// Huffman code lengths of 256 symbols from weights w[] (LDS), joining the two nodes with the
// smallest (weight, id) each time: leaves have id = symbol, the k-th joined node id 256 + k.
// Leaves sorted by (weight, symbol) form one queue, joined nodes (created in non-decreasing
// weight order) the other; the heads of the two queues are the two candidates.  The joining
// itself is sequential (lane 0): it keeps the two front weights of either queue in registers
// and reads one position ahead, so that no step waits for LDS.  Weights stay far below 2^32
// (a table sample is at most 16 chunks of 16 KB).
struct BuildLds {
    uint32_t w[256];               // leaf weights by symbol
    uint32_t sw[258];              // leaf weights in queue order, then two sentinels
    uint32_t wi[256];              // weights of the joined nodes, in order of creation
    uint16_t parent_leaf[256];     // by queue position: index of the joined node above the leaf
    uint16_t parent_int[256];      // by joined node: index of the joined node above it
    uint8_t len[256];
    uint32_t count[16], first[16], start[16];
    uint16_t by_len[256];          // symbols by (length, symbol)
    int longest;
};

// Code lengths from the weights s.w[], by a workgroup of 256 threads (one symbol each): Huffman's
// algorithm with two queues, a leaf before a joined node of the same weight and the lower symbol
// first among equal leaves; while the longest code exceeds kMaxLen all weights are halved (rounded
// up) and the construction is repeated.  Sorting, depths and halving are spread over the threads;
// the 255 joins are one thread's work.
__device__ __forceinline__ void build_lengths(BuildLds &s)
{
    constexpr uint32_t kNone = 0xffffffffu;
    const int tid = threadIdx.x;
    for (;;) {
        // position of the thread's leaf among all leaves
        const uint32_t wk = s.w[tid];
        int pos = 0;
        for (int t = 0; t < 256; ++t) {
            const uint32_t wt = s.w[t];
            pos += (wt < wk || (wt == wk && t < tid)) ? 1 : 0;
        }
        s.sw[pos] = wk;
        if (tid < 2) s.sw[256 + tid] = kNone;
        if (tid == 0) s.longest = 0;
        __syncthreads();
        if (tid == 0) {
            uint32_t wl = s.sw[0], wl1 = s.sw[1];      // front of the leaf queue and the one behind it
            uint32_t wj = kNone, wj1 = kNone;          // same for the queue of joined nodes
            int lq = 0, jq = 0, made = 0;
            for (int k = 0; k < 255; ++k) {
                uint32_t sum = 0;
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    if (wl <= wj) {                    // a leaf wins a tie: its id is lower
                        sum += wl;
                        s.parent_leaf[lq] = (uint16_t)made;
                        ++lq;
                        wl = wl1;
                        wl1 = s.sw[lq + 1];
                    } else {
                        sum += wj;
                        s.parent_int[jq] = (uint16_t)made;
                        ++jq;
                        wj = wj1;
                        wj1 = jq + 1 < made ? s.wi[jq + 1] : kNone;
                    }
                }
                s.wi[made] = sum;
                if (made == jq) wj = sum;
                else if (made == jq + 1) wj1 = sum;
                ++made;
            }
        }
        __syncthreads();
        int d = 1;
        for (int i = s.parent_leaf[pos]; i != 254 && d < 256; i = s.parent_int[i]) ++d;
        s.len[tid] = (uint8_t)d;
        atomicMax(&s.longest, d);
        __syncthreads();
        if (s.longest <= kMaxLen) return;
        const uint32_t v = (wk + 1) >> 1;
        __syncthreads();                               // everyone has seen `longest` before it is cleared
        s.w[tid] = v < 1 ? 1 : v;
        __syncthreads();
    }
}

constexpr int kTableWaves = 8;      // waves that fill a decode table

// grid = 2 workgroups of 256 threads (one symbol each): 0 builds the K table, 1 the V table
__global__ __launch_bounds__(256) void build_tables_kernel(CoderArgs a)
{
    __shared__ BuildLds s;
    __shared__ uint32_t block_count[4][16];            // symbols of each length in each block of 64 symbols
    const int sec = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = lane_id();
    s.w[tid] = a.ws.hist[256 * sec + tid] + 1;
    __syncthreads();
    build_lengths(s);
    // canonical codes: first code of every length, and the symbol's place among the symbols of
    // its length (those of lower blocks, then the lower lanes of its own block)
    const int L = s.len[tid];
    int within = 0;
#pragma unroll
    for (int l = 1; l <= kMaxLen; ++l) {
        const unsigned long long same = __builtin_amdgcn_ballot_w64(L == l);
        if (lane == 0) block_count[wave][l] = (uint32_t)__builtin_popcountll(same);
        if (L == l) within = __builtin_popcountll(same & ((1ull << lane) - 1));
    }
    __syncthreads();
    if (tid == 0) {
        uint32_t next = 0;
        for (int l = 1; l <= kMaxLen; ++l) {
            s.first[l] = next;
            next = (next + block_count[0][l] + block_count[1][l] + block_count[2][l] + block_count[3][l]) << 1;
        }
    }
    __syncthreads();
    uint32_t rank = (uint32_t)within;
    for (int w = 0; w < wave; ++w) rank += block_count[w][L];
    a.payload[a.off_aux + 256 * sec + tid] = (uint8_t)L;
    a.ws.enc[256 * sec + tid] = (s.first[L] + rank) | ((uint32_t)L << 16);
}

// grid = 2 workgroups of kTableWaves waves: decode tables from the lengths stored in the payload
__global__ __launch_bounds__(kTableWaves * 64) void decode_prepare_kernel(CoderArgs a)
{
    __shared__ BuildLds s;
    __shared__ uint32_t block_count[4][16];            // symbols of each length in each block of 64 symbols
    __shared__ int s_ok;
    const int sec = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = lane_id();
    if (*a.q.status & KVC_DEV_BAD_HEADER) return;
    // canonical order: the first four waves hold one symbol per thread
    int mylen = 0, within = 0;
    if (tid < 256) {
        mylen = a.payload[a.off_aux + 256 * sec + tid];
#pragma unroll
        for (int l = 1; l <= kMaxLen; ++l) {
            const unsigned long long same = __builtin_amdgcn_ballot_w64(mylen == l);
            if (lane == 0) block_count[wave][l] = (uint32_t)__builtin_popcountll(same);
            if (mylen == l) within = __builtin_popcountll(same & ((1ull << lane) - 1));
        }
        const bool in_range = mylen >= 1 && mylen <= kMaxLen;
        if (lane == 0) block_count[wave][0] = __builtin_amdgcn_ballot_w64(!in_range) != 0 ? 1u : 0u;
    }
    __syncthreads();
    if (tid == 0) {
        uint32_t next = 0, at = 0, kraft = 0;
        for (int l = 1; l <= kMaxLen; ++l) {
            const uint32_t n = block_count[0][l] + block_count[1][l] + block_count[2][l] + block_count[3][l];
            s.count[l] = n;
            s.first[l] = next;
            s.start[l] = at;
            next = (next + n) << 1;
            at += n;
            kraft += n << (kMaxLen - l);
        }
        const bool bad_len = (block_count[0][0] | block_count[1][0] | block_count[2][0] | block_count[3][0]) != 0;
        const bool ok = !bad_len && kraft == (1u << kMaxLen);          // a complete prefix code
        s_ok = ok ? 1 : 0;
        if (!ok) atomicOr(a.q.status, KVC_DEV_BAD_TABLE);
    }
    __syncthreads();
    if (s_ok && tid < 256) {
        uint32_t rank = (uint32_t)within;
        for (int w = 0; w < wave; ++w) rank += block_count[w][mylen];
        s.by_len[s.start[mylen] + rank] = (uint16_t)tid;                    // symbols by (length, symbol)
    }
    __syncthreads();
    uint16_t *lut = a.ws.lut + 4096 * sec;
    if (!s_ok) {
        for (int i = tid; i < 4096; i += kTableWaves * 64) lut[i] = (uint16_t)(1u << 8);      // symbol 0, length 1
        return;
    }
    // entry i describes the code word that is a prefix of the 12-bit string i
    for (int i = tid; i < 4096; i += kTableWaves * 64) {
        uint16_t e = (uint16_t)(1u << 8);
        for (int L = 1; L <= kMaxLen; ++L) {
            const uint32_t c = (uint32_t)i >> (kMaxLen - L);
            if (c >= s.first[L] && c - s.first[L] < s.count[L]) {
                e = (uint16_t)(s.by_len[s.start[L] + c - s.first[L]] | (L << 8));
                break;
            }
        }
        lut[i] = e;
    }
}

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
// Waves per SIMD the register allocation must leave room for: four workgroups of the 2- to 4-bit
// group-32 encoders fit a compute unit's LDS, and for fp16 rows in the dense layout they fit its
// registers too without spilling (the other variants would spill, so they keep what they need).
template <int BITS, int G, int DT, bool DENSE> constexpr int enc_min_waves()
{
    return (BITS <= 4 && G == 32 && DT == DT_F16 && DENSE) ? 4 : 1;
}

template <int BITS, int G, int DT, bool IS_V, bool DENSE, bool XF>
__global__ __launch_bounds__(ChunkGeom<BITS>::kWaves * 64) __attribute__((amdgpu_waves_per_eu(enc_min_waves<BITS, G, DT, DENSE>())))
void encode_kernel(CoderArgs a)
{
    using Geo = ChunkGeom<BITS>;
    constexpr int W = Geo::kWords, NW = Geo::kWaves;
    __shared__ __attribute__((aligned(16))) uint8_t lds_all[NW * Geo::kLds];
    __shared__ EncTables enc;
    __shared__ uint32_t s_units[NW];
    __shared__ unsigned long long s_excl;
    __shared__ uint32_t s_ticket;

    const int tid = threadIdx.x, wave = tid >> 6, lane = lane_id();
    PHASE_START();
    if (tid == 0) s_ticket = atomicAdd(a.ws.ticket, 1u);
    for (int k = tid; k < 256; k += NW * 64) {
        const uint32_t e = a.ws.enc[(IS_V ? 256 : 0) + k];       // code | length << 16
        enc.len[k] = (uint8_t)(e >> 16);
        enc.code[k] = (uint16_t)((e & 0xfffu) | ((e >> 16) << 12));
    }
    __syncthreads();
    PHASE(0, 0);
    const long long ticket = s_ticket;                 // global order over K and V workgroups
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
        PHASE(0, 1);
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
        PHASE(0, 2);
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
    PHASE(0, 3);
    if (!live && lane == 0)
        __hip_atomic_fetch_add(&a.ws.state[ticket], (unsigned long long)(kAggComplete / NW) << kAggShift, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
    if (lane == 0) s_units[wave] = body_units;
    __syncthreads();
    PHASE(0, 4);

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
                uint32_t *dir = (uint32_t *)(a.payload + a.off_aux + 512);
                dir[a.total_chunks] = (uint32_t)all;
                unsigned long long k_units = 0;
                if (a.wg_base > 0)
                    k_units = __hip_atomic_load(&a.ws.state[a.wg_base - 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & kValueMask;
                else if (!IS_V)
                    k_units = all;
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
    if (wave == 0) PHASE(0, 5);
    __syncthreads();
    PHASE(0, 6);
    const unsigned long long excl = s_excl;
    if (!live || excl == ~0ull) return;
    unsigned long long mine = excl;
    for (int w = 0; w < wave; ++w) mine += s_units[w];
    if (lane == 0) ((uint32_t *)(a.payload + a.off_aux + 512))[a.chunk_base + chunk] = (uint32_t)mine;
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
    PHASE(0, 7);
    PHASE_END(0);
}

// ---- decoder ---------------------------------------------------------------------------------

struct BitReader {
    unsigned long long window;   // upcoming bits, left aligned
    int avail;
    const uint32_t *next;        // next word (LDS)
    const uint32_t *last;        // last readable word
};

__device__ __forceinline__ void refill(BitReader &br)
{
    if (br.avail <= 32) {
        br.window |= (unsigned long long)(*br.next) << (32 - br.avail);
        br.avail += 32;
        if (br.next < br.last) ++br.next;
    }
}

template <int W> __device__ __forceinline__ void decode_half(uint32_t *sym, const uint16_t *lut, int half, BitReader &br)
{
#pragma unroll
    for (int k = 0; k < W / 2; ++k) {
        uint32_t w = 0;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const uint32_t e = lut[(uint32_t)(br.window >> 52)];
            const uint32_t len = e >> 8;
            w = __builtin_amdgcn_alignbit(e, w, 8);      // symbol byte enters at the top; after 4 symbols the first is lowest
            br.window <<= len;
            br.avail -= (int)len;
            if (b & 1) refill(br);
        }
        sym[half * (W / 2) + k] = w;
    }
}

// metadata of the 32 rows starting at chunk row `r0`: K = the lane's 8 channels of that token
// block (two 16-byte loads), V = the lane's group in each of its 8 rows
__device__ __forceinline__ void load_meta_k(const QuantArgs &q, const ChunkPos &c, int r0, u32x4 &m0, u32x4 &m1)
{
    const int col = lane_id() & 15;
    const long long nb = (q.tokens + q.group - 1) / q.group;
    const u32x4 *m = (const u32x4 *)(q.meta + ((c.lh * nb + (c.row0 + r0) / q.group) * kDim + col * 8) * 4);
    m0 = m[0];
    m1 = m[1];
}

__device__ __forceinline__ void load_meta_v(const QuantArgs &q, const ChunkPos &c, int r0, uint32_t mv[8])
{
    const int lane = lane_id(), col = lane & 15, rsub = lane >> 4;
    const int ng = kDim / q.group, shift = q.group == 32 ? 2 : (q.group == 64 ? 3 : 4);
    const uint32_t *m = (const uint32_t *)q.meta + (c.lh * q.tokens + c.row0 + r0) * ng + (col >> shift);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int r = 4 * i + rsub;
        mv[i] = m[(r0 + r < c.rows ? r : 0) * ng];
    }
}

// Dequantize a decoded chunk from the wave's LDS region and store its rows; the metadata of a
// pass is in flight one pass ahead.  meta0 / meta1 (K) or metav (V): the first pass's metadata.
// first_anchor (delta transform): the first pass's anchor row.
template <int BITS, int DT, bool IS_V, bool DENSE, int TR>
__device__ __forceinline__ void dequant_chunk(const CoderArgs &a, const ChunkPos &c, uint8_t *lds, const u32x4 &meta0,
                                              const u32x4 &meta1, const uint32_t metav[8], const u32x4 &first_anchor, bool &bad)
{
    using Dec = DecGeom<BITS>;
    const uint16_t *anchors = TR == 2 ? head_anchors(a.q.anchors, c.lh, a.q.tokens, a.q.anchor_shift) : nullptr;
    constexpr bool one_anchor = TR == 2;
    u32x4 anchor = first_anchor, anchor_next = first_anchor;
    u32x4 mk0 = meta0, mk1 = meta1;
    uint32_t mv[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) mv[i] = metav[i];
#pragma unroll 1
    for (int p = 0; p < kChunkRows / kPassRows; ++p) {
        if (p * kPassRows >= c.rows) break;
        float scale[8], zero[8];
        const bool clamp = IS_V ? v_meta_floats<BITS, DT>(mv, scale, zero) : k_meta_floats<BITS, DT>(mk0, mk1, scale, zero);
        if ((p + 1) * kPassRows < c.rows) {
            if (!IS_V) load_meta_k(a.q, c, (p + 1) * kPassRows, mk0, mk1);
            else load_meta_v(a.q, c, (p + 1) * kPassRows, mv);
            if (one_anchor) anchor_next = load_anchor(anchors, a.q.anchor_shift, c.row0 + (p + 1) * kPassRows);
        }
        dequant_pass<BITS, DT, IS_V, DENSE, Dec::kLayout, TR>(lds, scale, zero, clamp, a.q.x, c.head_off, c.row0 + p * kPassRows,
                                                              c.rows - p * kPassRows, bad, p * kPassRows, anchors, a.q.anchor_shift,
                                                              one_anchor ? &anchor : nullptr);
        anchor = anchor_next;
    }
}

template <int BITS, int DT, bool IS_V, bool DENSE>
__global__ __launch_bounds__(ChunkGeom<BITS>::kDecWaves * 64) void decode_kernel(CoderArgs a)
{
    using Geo = ChunkGeom<BITS>;
    using Dec = DecGeom<BITS>;
    constexpr int W = Geo::kWords, NW = Geo::kDecWaves;
    __shared__ __attribute__((aligned(16))) uint8_t lds_all[NW * Dec::kLds];
    __shared__ uint16_t lut[4096];

    const int tid = threadIdx.x, wave = tid >> 6, lane = lane_id();
    const long long chunk = (long long)blockIdx.x * NW + wave;
    const bool live = chunk < a.chunks;
    uint8_t *lds = lds_all + wave * Dec::kLds;
    PHASE_START();
    // Register headroom.  On this GPU a 64-bit shift whose count sits in the last VGPR of the
    // wave's allocation shifts by the lane number instead, now and then, once three or four such
    // waves share a SIMD (LLVM knows and avoids the fault for gfx90a only).  A build of this
    // kernel that needed exactly 112 registers kept a code length in v111 for `window <<= len`
    // and decoded the last two symbols of a sub-block wrongly in one wave of seven at full size.
    // Naming a higher register keeps the allocation (128: still four waves per SIMD) above every
    // register the code touches; the build checks the assembly of all kernels for the pattern.
    asm volatile("" ::: "v127");

    // Round trip 1: the chunk's two directory entries and the status word, with the decode
    // table right behind them.
    unsigned long long d0 = 0, d1 = 0;
    int st = 0;
    if (live) {
        const uint32_t *dir = (const uint32_t *)(a.payload + a.off_aux + 512) + a.chunk_base + chunk;
        d0 = dir[0];
        d1 = dir[1];
        st = *a.q.status;
    }
    constexpr int LUTN = 512 / (NW * 64);
    u32x4 lutv[LUTN];
    {
        const u32x4 *src = (const u32x4 *)(a.ws.lut + (IS_V ? 4096 : 0));
#pragma unroll
        for (int i = 0; i < LUTN; ++i) lutv[i] = src[tid + i * NW * 64];
    }
    ChunkPos c = chunk_pos(a.q, live ? chunk : 0);
    const uint32_t raw_bytes = (uint32_t)c.rows * Geo::kRowBytes;
    const unsigned long long size = (d1 - d0) * 16;
    bool ok = live && !(st & (KVC_DEV_BAD_HEADER | KVC_DEV_BAD_TABLE));
    if (ok && (d1 < d0 || size > raw_bytes || (long long)(a.off_bodies + d1 * 16) > a.capacity ||
               (size != raw_bytes && size < 2 * kSubs + 16))) {
        if (lane == 0) atomicOr(a.q.status, KVC_DEV_BAD_CHUNK);
        ok = false;
    }
    // Round trip 2: the body (into registers) and the metadata of the first pass.
    constexpr int NB = 2 * BITS;                       // 16-byte pieces per lane of a full raw chunk
    u32x4 bodyv[NB];
    u32x4 meta0 = {0, 0, 0, 0}, meta1 = {0, 0, 0, 0};
    uint32_t metav[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    u32x4 anchor0 = {0, 0, 0, 0};                      // delta transform: the first pass's anchor row
    if (ok) {
        const uint8_t *body = a.payload + a.off_bodies + d0 * 16;
#pragma unroll
        for (int k = 0; k < NB; ++k) {
            const uint32_t o = (k * 64 + lane) * 16;
            if (o < size) bodyv[k] = __builtin_nontemporal_load((const u32x4 *)(body + o));
        }
        if (!IS_V) load_meta_k(a.q, c, 0, meta0, meta1);
        else load_meta_v(a.q, c, 0, metav);
        if (a.q.anchors)
            anchor0 = load_anchor(head_anchors(a.q.anchors, c.lh, a.q.tokens, a.q.anchor_shift), a.q.anchor_shift, c.row0);
    }
#pragma unroll
    for (int i = 0; i < LUTN; ++i) ((u32x4 *)lut)[tid + i * NW * 64] = lutv[i];
    __syncthreads();
    if (!ok) return;
    PHASE(1, 0);

    if (size == raw_bytes) {
        // stored raw: scatter the packed rows into the sub-block layout
#pragma unroll
        for (int k = 0; k < NB; ++k) {
            const uint32_t o = (k * 64 + lane) * 16;
            if (o < raw_bytes) {
                const uint32_t sub = o / Geo::kSubBytes, in = o - sub * Geo::kSubBytes;
                *(u32x4 *)Dec::piece_ptr(lds, sub, in / 16) = bodyv[k];
            }
        }
        wave_sync();
    } else {
#pragma unroll
        for (int k = 0; k < NB; ++k) {
            const uint32_t o = (k * 64 + lane) * 16;
            if (o < size) *(u32x4 *)(lds + o) = bodyv[k];
        }
        wave_sync();
        PHASE(1, 1);
        const uint32_t bits = ((const uint16_t *)lds)[lane];
        const uint32_t incl = wave_inclusive_sum(bits);
        const uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
        if (((2 * kSubs + 4 * ((total + 31) / 32) + 15) & ~15u) != size) {
            if (lane == 0) atomicOr(a.q.status, KVC_DEV_BAD_CHUNK);
            return;
        }
        const uint32_t start = incl - bits;
        const uint32_t *words = (const uint32_t *)(lds + 2 * kSubs);
        BitReader br;
        br.last = (const uint32_t *)(lds + size) - 1;
        const uint32_t *p = words + (start >> 5);
        p = p < br.last ? p : br.last;
        const uint32_t w0 = *p;
        p = p < br.last ? p + 1 : p;
        const uint32_t w1 = *p;
        p = p < br.last ? p + 1 : p;
        br.window = (((unsigned long long)w0 << 32) | w1) << (start & 31);
        br.avail = 64 - (int)(start & 31);
        br.next = p;
        uint32_t sym[W];
#pragma unroll
        for (int k = 0; k < W; ++k) sym[k] = 0;
        const int have = min(max(c.rows - 2 * lane, 0), 2);
        if (have > 0) decode_half<W>(sym, lut, 0, br);
        if (have > 1) decode_half<W>(sym, lut, 1, br);
        wave_sync();                                   // all lanes are done reading the coded words
        {
#pragma unroll
            for (int q = 0; q < W / 4; ++q) {
                u32x4 v;
                v[0] = sym[4 * q]; v[1] = sym[4 * q + 1]; v[2] = sym[4 * q + 2]; v[3] = sym[4 * q + 3];
                *(u32x4 *)Dec::piece_ptr(lds, lane, q) = v;
            }
        }
        wave_sync();
        PHASE(1, 2);
    }

    // dequantize the rows from LDS (one copy of the loop per transform; a launch runs one of them)
    bool bad = false;
    if (a.q.rotate) dequant_chunk<BITS, DT, IS_V, DENSE, 1>(a, c, lds, meta0, meta1, metav, anchor0, bad);
    else if (a.q.anchors) dequant_chunk<BITS, DT, IS_V, DENSE, 2>(a, c, lds, meta0, meta1, metav, anchor0, bad);
    else dequant_chunk<BITS, DT, IS_V, DENSE, 0>(a, c, lds, meta0, meta1, metav, anchor0, bad);
    if (bad) atomicOr(a.q.status, KVC_DEV_BAD_BLOCK);
    PHASE(1, 3);
    PHASE_END(1);
}

// ---- launchers ----------------------------------------------------------------------------------

static inline int launched() { return hipGetLastError() == hipSuccess ? KVC_OK : KVC_ERR_DEVICE; }

template <int BITS, int G, int DT, bool IS_V> static int hist_launch(const CoderArgs &a, hipStream_t s)
{
    if (a.chunks <= 0) return KVC_OK;
    hipLaunchKernelGGL((hist_kernel<BITS, G, DT, IS_V>), dim3(16), dim3(64), 0, s, a);
    return launched();
}

template <int BITS, int G, int DT, bool IS_V> static int encode_launch(const CoderArgs &a, hipStream_t s)
{
    constexpr int NW = ChunkGeom<BITS>::kWaves;
    const long long need = (a.chunks + NW - 1) / NW;
    if (need <= 0) return KVC_OK;
    // K token blocks of 64 and 128 rows, and V groups of 32 channels (the variant that is short of
    // registers), have a kernel of their own for launches without a transform
    constexpr bool kSplit = IS_V ? G == 32 : G >= 64;
    if (kSplit && !a.q.rotate && !a.q.anchors) {
        if (a.q.dense) hipLaunchKernelGGL((encode_kernel<BITS, G, DT, IS_V, true, !kSplit>), dim3((unsigned)need), dim3(NW * 64), 0, s, a);
        else hipLaunchKernelGGL((encode_kernel<BITS, G, DT, IS_V, false, !kSplit>), dim3((unsigned)need), dim3(NW * 64), 0, s, a);
        return launched();
    }
    if (a.q.dense) hipLaunchKernelGGL((encode_kernel<BITS, G, DT, IS_V, true, true>), dim3((unsigned)need), dim3(NW * 64), 0, s, a);
    else hipLaunchKernelGGL((encode_kernel<BITS, G, DT, IS_V, false, true>), dim3((unsigned)need), dim3(NW * 64), 0, s, a);
    return launched();
}

template <int BITS, int DT, bool IS_V> static int decode_launch(const CoderArgs &a, hipStream_t s)
{
    constexpr int NW = ChunkGeom<BITS>::kDecWaves;
    const long long need = (a.chunks + NW - 1) / NW;
    if (need <= 0) return KVC_OK;
    if (a.q.dense) hipLaunchKernelGGL((decode_kernel<BITS, DT, IS_V, true>), dim3((unsigned)need), dim3(NW * 64), 0, s, a);
    else hipLaunchKernelGGL((decode_kernel<BITS, DT, IS_V, false>), dim3((unsigned)need), dim3(NW * 64), 0, s, a);
    return launched();
}

#define KVC_BY_GROUP(FN, BITS, DT, ISV, group, ...)                    \
    switch (group) {                                                   \
    case 32: return FN<BITS, 32, DT, ISV>(__VA_ARGS__);                \
    case 64: return FN<BITS, 64, DT, ISV>(__VA_ARGS__);                \
    case 128: return FN<BITS, 128, DT, ISV>(__VA_ARGS__);              \
    }                                                                  \
    return KVC_ERR_UNSUPPORTED

template <int BITS, int DT, bool ISV> static int hist_g(int group, const CoderArgs &a, hipStream_t s) { KVC_BY_GROUP(hist_launch, BITS, DT, ISV, group, a, s); }
template <int BITS, int DT, bool ISV> static int encode_g(int group, const CoderArgs &a, hipStream_t s) { KVC_BY_GROUP(encode_launch, BITS, DT, ISV, group, a, s); }

template <int BITS, bool ISV> static int hist_d(int group, int dtype, const CoderArgs &a, hipStream_t s)
{
    return dtype == DT_F16 ? hist_g<BITS, DT_F16, ISV>(group, a, s) : hist_g<BITS, DT_BF16, ISV>(group, a, s);
}
template <int BITS, bool ISV> static int encode_d(int group, int dtype, const CoderArgs &a, hipStream_t s)
{
    return dtype == DT_F16 ? encode_g<BITS, DT_F16, ISV>(group, a, s) : encode_g<BITS, DT_BF16, ISV>(group, a, s);
}
template <int BITS, bool ISV> static int decode_d(int dtype, const CoderArgs &a, hipStream_t s)
{
    return dtype == DT_F16 ? decode_launch<BITS, DT_F16, ISV>(a, s) : decode_launch<BITS, DT_BF16, ISV>(a, s);
}

template <bool ISV> static int hist_b(int bits, int group, int dtype, const CoderArgs &a, hipStream_t s)
{
    switch (bits) {
    case 2: return hist_d<2, ISV>(group, dtype, a, s);
    case 3: return hist_d<3, ISV>(group, dtype, a, s);
    case 4: return hist_d<4, ISV>(group, dtype, a, s);
    case 8: return hist_d<8, ISV>(group, dtype, a, s);
    }
    return KVC_ERR_UNSUPPORTED;
}
template <bool ISV> static int encode_b(int bits, int group, int dtype, const CoderArgs &a, hipStream_t s)
{
    switch (bits) {
    case 2: return encode_d<2, ISV>(group, dtype, a, s);
    case 3: return encode_d<3, ISV>(group, dtype, a, s);
    case 4: return encode_d<4, ISV>(group, dtype, a, s);
    case 8: return encode_d<8, ISV>(group, dtype, a, s);
    }
    return KVC_ERR_UNSUPPORTED;
}
template <bool ISV> static int decode_b(int bits, int dtype, const CoderArgs &a, hipStream_t s)
{
    switch (bits) {
    case 2: return decode_d<2, ISV>(dtype, a, s);
    case 3: return decode_d<3, ISV>(dtype, a, s);
    case 4: return decode_d<4, ISV>(dtype, a, s);
    case 8: return decode_d<8, ISV>(dtype, a, s);
    }
    return KVC_ERR_UNSUPPORTED;
}

int launch_coder_tables(int bits_k, int bits_v, int group_k, int group_v, int dtype, const CoderArgs &k,
                        const CoderArgs &v, hipStream_t s)
{
    int rc = hist_b<false>(bits_k, group_k, dtype, k, s);
    if (rc) return rc;
    rc = hist_b<true>(bits_v, group_v, dtype, v, s);
    if (rc) return rc;
    hipLaunchKernelGGL(build_tables_kernel, dim3(2), dim3(256), 0, s, k);
    return launched();
}

int launch_encode_section(int bits, int group, int dtype, const CoderArgs &a, hipStream_t s)
{
    return a.is_v ? encode_b<true>(bits, group, dtype, a, s) : encode_b<false>(bits, group, dtype, a, s);
}

int launch_decode_prepare(const CoderArgs &k, hipStream_t s)
{
    hipLaunchKernelGGL(decode_prepare_kernel, dim3(2), dim3(kTableWaves * 64), 0, s, k);
    return launched();
}

int launch_decode_section(int bits, int group, int dtype, const CoderArgs &a, hipStream_t s)
{
    (void)group;
    return a.is_v ? decode_b<true>(bits, dtype, a, s) : decode_b<false>(bits, dtype, a, s);
}

}  // namespace kvc

#ifdef KVC_PHASE_CLOCKS
// out: HOST memory, 32 64-bit words (encoder phases 0..15, decoder phases 0..15); reset != 0 clears
extern "C" int kvc_phase_clocks(uint64_t *out, int reset)
{
    static uint64_t rows[1024][2][16];
    if (hipDeviceSynchronize() != hipSuccess) return -1;
    if (out) {
        if (hipMemcpyFromSymbol(rows, HIP_SYMBOL(kvc::g_phase_clocks), sizeof(rows)) != hipSuccess) return -1;
        for (int i = 0; i < 32; ++i) out[i] = 0;
        for (int r = 0; r < 1024; ++r)
            for (int i = 0; i < 32; ++i) out[i] += rows[r][i / 16][i % 16];
    }
    if (reset) {
        for (int r = 0; r < 1024; ++r)
            for (int i = 0; i < 32; ++i) rows[r][i / 16][i % 16] = 0;
        if (hipMemcpyToSymbol(HIP_SYMBOL(kvc::g_phase_clocks), rows, sizeof(rows)) != hipSuccess) return -1;
    }
    return 0;
}
#endif
