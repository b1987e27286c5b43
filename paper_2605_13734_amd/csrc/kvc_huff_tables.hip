// Lossless stage, set-up kernels: the table sample (byte histogram of up to 16 chunks per section),
// the code construction (Huffman lengths, canonical codes) and the decode tables.  See kvc_huff.h.

#include "kvc_huff.h"

namespace kvc {

// ---- table sample: histogram of up to 16 chunks per section ------------------------------------

// grid = 16 sample chunks x the units of a chunk, one wave each: the wave quantizes its unit (one
// load round trip) and counts the byte values of the packed rows.
template <int BITS, int G, int DT, bool IS_V>
__global__ __launch_bounds__(64) void hist_kernel(CoderBatch batch)
{
    const CoderArgs &a = batch.item[blockIdx.y];
    if (a.chunks <= 0) return;
    using Unit = UnitGeom<BITS, G, DT, IS_V>;
    constexpr int RW = 4 * BITS;                         // words of a packed row
    // (a whole chunk's region: the K group parameters travel through the padding of all 64 sub-blocks)
    __shared__ __attribute__((aligned(16))) uint8_t lds[ChunkGeom<BITS>::kLds];
    __shared__ uint32_t hist[256];
    const int i = blockIdx.x / Unit::kUnits, u = blockIdx.x - i * Unit::kUnits, lane = lane_id();
    const long long n = a.chunks;
    const long long chunk = (long long)i * n / 16;
    if (i > 0 && (long long)(i - 1) * n / 16 == chunk) return;      // each chunk counted once
    ChunkPos c = chunk_pos(a.q, chunk);
    if (u * Unit::kRows >= c.rows) return;
    for (int k = lane; k < 256; k += 64) hist[k] = 0;
    bool bad = false;
    quantize_unit<BITS, G, DT, IS_V, false>(a.q, c, u, lds, 0, false, bad);
    wave_sync();
    const int rows = min(c.rows - u * Unit::kRows, Unit::kRows);
    for (int w = lane; w < rows * RW; w += 64) {
        const int r = w / RW;
        const uint32_t word = *(const uint32_t *)(code_row<BITS, true>(lds, r) + (w - r * RW) * 4);
#pragma unroll
        for (int b = 0; b < 4; ++b) atomicAdd(&hist[(word >> (8 * b)) & 255u], 1u);
    }
    wave_sync();
    uint32_t *g = a.ws.hist + 256 * a.tab;
    for (int k = lane; k < 256; k += 64)
        if (hist[k]) atomicAdd(&g[k], hist[k]);
}

// ---- code construction (one wave per section) ---------------------------------------------------

// Huffman code lengths of 256 symbols from weights w[] (LDS), joining the two nodes with the
// smallest (weight, id) each time: leaves have id = symbol, the k-th joined node id 256 + k.
// Leaves sorted by (weight, symbol) form one queue, joined nodes (created in non-decreasing
// weight order) the other; the heads of the two queues are the two candidates.  The joining
// itself is sequential (lane 0).  Weights stay far below 2^32 (a table sample is at most 16
// chunks of 16 KB).
constexpr int kQueue = 260;

struct BuildLds {
    uint32_t w[256];               // leaf weights by symbol
    // The two queues of the join and, at one and the same distance behind each (kQueue words), the
    // parents of their entries: the join walks both queues with one byte offset each and reaches
    // weight and parent through constant displacements.
    uint32_t sw[kQueue];           // leaf weights in queue order, then two sentinels
    uint32_t parent_leaf[kQueue];  // by queue position: index of the joined node above the leaf
    uint32_t wi[kQueue];           // weights of the joined nodes, in order of creation
    uint32_t parent_int[kQueue];   // by joined node: index of the joined node above it
    uint8_t len[256];
    uint32_t count[16], first[16], start[16];
    uint16_t by_len[256];          // symbols by (length, symbol)
    int longest;
};

// One construction of code lengths from the weights s.w[], by a workgroup of 256 threads (one symbol
// each): Huffman's algorithm with two queues, a leaf before a joined node of the same weight and the
// lower symbol first among equal leaves.  Sorting and depths are spread over the threads; the 255
// joins are one thread's work.  Leaves s.len[] and s.longest; ends with a barrier.
__device__ __forceinline__ void build_once(BuildLds &s)
{
    constexpr uint32_t kNone = 0xffffffffu;
    const int tid = threadIdx.x;
    // position of the thread's leaf among all leaves
    const uint32_t wk = s.w[tid];
    int pos = 0;
    for (int t = 0; t < 256; ++t) {
        const uint32_t wt = s.w[t];
        pos += (wt < wk || (wt == wk && t < tid)) ? 1 : 0;
    }
    s.sw[pos] = wk;
    s.wi[tid] = kNone;                             // a joined node that does not exist yet never wins
    if (tid < 2) s.sw[256 + tid] = kNone;
    if (tid == 0) s.longest = 0;
    __syncthreads();
    if (tid == 0) {
        // Every join reads the two front entries of both queues in one go (one LDS round trip) and
        // decides in registers; the entries it writes are read by later joins only.
        uint8_t *base = (uint8_t *)&s;
        uint32_t lo = (uint32_t)__builtin_offsetof(BuildLds, sw), jo = (uint32_t)__builtin_offsetof(BuildLds, wi);
        constexpr uint32_t kParent = kQueue * 4;       // from a queue entry to its parent word
        for (uint32_t made = 0; made < 255; ++made) {
            const uint32_t a0 = *(const uint32_t *)(base + lo), a1 = *(const uint32_t *)(base + lo + 4);
            const uint32_t b0 = *(const uint32_t *)(base + jo), b1 = *(const uint32_t *)(base + jo + 4);
            const bool first_leaf = a0 <= b0;      // a leaf wins a tie: its id is lower
            const uint32_t la = first_leaf ? a1 : a0, jb = first_leaf ? b0 : b1;     // the fronts after the first pick
            const bool second_leaf = la <= jb;
            const uint32_t sum = (first_leaf ? a0 : b0) + (second_leaf ? la : jb);
            const uint32_t p0 = first_leaf ? lo : jo;
            lo += first_leaf ? 4 : 0;
            jo += first_leaf ? 0 : 4;
            const uint32_t p1 = second_leaf ? lo : jo;
            lo += second_leaf ? 4 : 0;
            jo += second_leaf ? 0 : 4;
            *(uint32_t *)(base + p0 + kParent) = made;
            *(uint32_t *)(base + p1 + kParent) = made;
            s.wi[made] = sum;
        }
    }
    __syncthreads();
    int d = 1;
    for (uint32_t i = s.parent_leaf[pos]; i != 254 && d < 256; i = s.parent_int[i]) ++d;
    s.len[tid] = (uint8_t)d;
    atomicMax(&s.longest, d);
    __syncthreads();
}

// The format's length limit: while the longest code exceeds kMaxLen all weights are halved (rounded
// up) and the construction is repeated.  k halvings turn a weight w into ceil(w / 2^k), so the
// constructions do not depend on each other: all of them run side by side, one workgroup each, and
// the one with the fewest halvings that meets the limit is the table.  (Groups along 128 tokens or
// channels give strongly peaked codes that need five or six halvings; one after the other they
// took 0.25 ms per call.)  A table sample is at most 16 chunks of 16 KB, so a weight is at most
// 2^18 + 1 and 19 halvings leave nothing but ones, whose code has 8 bits everywhere: the last
// candidate always meets the limit.
constexpr int kCandidates = 20;

__device__ __forceinline__ uint32_t halved(uint32_t w, int k) { return (w + ((1u << k) - 1u)) >> k; }

constexpr int kTableWaves = 8;      // waves that fill a decode table

// grid = kCandidates workgroups of 256 threads (one symbol each) per table slot of the format.
// A candidate leaves its lengths in the slot's decode-table space of the workspace (unused while
// compressing); the last one to finish picks and writes the table.
__global__ __launch_bounds__(256) void build_tables_kernel(CoderBatch batch)
{
    const CoderArgs &a = batch.item[blockIdx.y];
    const int sec = blockIdx.x / kCandidates, k = blockIdx.x - sec * kCandidates;
    const int tid = threadIdx.x, wave = tid >> 6, lane = lane_id();
    if (!((a.slot_mask >> sec) & 1)) {                 // a width the tensor does not use: an empty table
        if (k == 0) a.payload[a.off_aux + 256 * sec + tid] = 0;
        return;
    }
    __shared__ BuildLds s;
    __shared__ uint32_t block_count[4][16];            // symbols of each length in each block of 64 symbols
    __shared__ int s_pick;
    const uint32_t w0 = a.ws.hist[256 * sec + tid] + 1;
    s.w[tid] = halved(w0, k);
    __syncthreads();
    build_once(s);
    uint32_t *cand = (uint32_t *)(a.ws.lut + 4096 * sec);      // [kCandidates][64] words of lengths, then the longest of each
    if ((tid & 3) == 0) {
        const uint32_t word = (uint32_t)s.len[tid] | ((uint32_t)s.len[tid + 1] << 8) | ((uint32_t)s.len[tid + 2] << 16) |
                              ((uint32_t)s.len[tid + 3] << 24);
        __hip_atomic_store(cand + 64 * k + (tid >> 2), word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (tid == 0) __hip_atomic_store(cand + 64 * kCandidates + k, (uint32_t)s.longest, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __threadfence();
    __syncthreads();
    if (tid == 0) {
        // (the counters sit behind the ticket, in words that every call clears)
        const uint32_t done = __hip_atomic_fetch_add(a.ws.ticket + 8 + sec, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
        int pick = -1;                                 // not the last candidate: nothing more to do
        if (done == kCandidates - 1) {
            pick = kCandidates - 1;
            for (int j = kCandidates - 2; j >= 0; --j)
                if (__hip_atomic_load(cand + 64 * kCandidates + j, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) <= (uint32_t)kMaxLen) pick = j;
        }
        s_pick = pick;
    }
    __syncthreads();
    const int pick = s_pick;
    if (pick < 0) return;
    const uint32_t picked = __hip_atomic_load(cand + 64 * pick + (tid >> 2), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int L = (int)((picked >> (8 * (tid & 3))) & 255u);
    // canonical codes: first code of every length, and the symbol's place among the symbols of
    // its length (those of lower blocks, then the lower lanes of its own block)
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

// grid = one workgroup of kTableWaves waves per table slot: decode tables from the lengths stored in the payload
__global__ __launch_bounds__(kTableWaves * 64) void decode_prepare_kernel(CoderBatch batch)
{
    const CoderArgs &a = batch.item[blockIdx.y];
    if (!((a.slot_mask >> blockIdx.x) & 1)) return;
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

// ---- launchers ----------------------------------------------------------------------------------

template <int BITS, int G, int DT, bool IS_V> static int hist_launch(const CoderBatch &b, hipStream_t s)
{
    bool any = false;
    for (int i = 0; i < b.n; ++i) any |= b.item[i].chunks > 0;
    if (!any) return KVC_OK;
    hipLaunchKernelGGL((hist_kernel<BITS, G, DT, IS_V>), dim3(16 * UnitGeom<BITS, G, DT, IS_V>::kUnits, (unsigned)b.n), dim3(64), 0, s, b);
    return launched();
}

template <int BITS, int DT, bool ISV> static int hist_g(int group, const CoderBatch &a, hipStream_t s)
{
    switch (group) {
    case 32: return hist_launch<BITS, 32, DT, ISV>(a, s);
    case 64: return hist_launch<BITS, 64, DT, ISV>(a, s);
    case 128: return hist_launch<BITS, 128, DT, ISV>(a, s);
    }
    return KVC_ERR_UNSUPPORTED;
}

template <int BITS, bool ISV> static int hist_d(int group, int dtype, const CoderBatch &a, hipStream_t s)
{
    return dtype == DT_F16 ? hist_g<BITS, DT_F16, ISV>(group, a, s) : hist_g<BITS, DT_BF16, ISV>(group, a, s);
}

template <bool ISV> static int hist_b(int bits, int group, int dtype, const CoderBatch &a, hipStream_t s)
{
    switch (bits) {
    case 2: return hist_d<2, ISV>(group, dtype, a, s);
    case 3: return hist_d<3, ISV>(group, dtype, a, s);
    case 4: return hist_d<4, ISV>(group, dtype, a, s);
    case 8: return hist_d<8, ISV>(group, dtype, a, s);
    }
    return KVC_ERR_UNSUPPORTED;
}

int launch_table_sample(int bits, int group, int dtype, const CoderBatch &b, hipStream_t s)
{
    return b.item[0].is_v ? hist_b<true>(bits, group, dtype, b, s) : hist_b<false>(bits, group, dtype, b, s);
}

int launch_build_tables(const CoderBatch &b, hipStream_t s)
{
    hipLaunchKernelGGL(build_tables_kernel, dim3(b.item[0].slots * kCandidates, (unsigned)b.n), dim3(256), 0, s, b);
    return launched();
}

int launch_decode_prepare(const CoderBatch &b, hipStream_t s)
{
    hipLaunchKernelGGL(decode_prepare_kernel, dim3(b.item[0].slots, (unsigned)b.n), dim3(kTableWaves * 64), 0, s, b);
    return launched();
}

int launch_encode_section(int bits, int group, int dtype, const CoderBatch &a, hipStream_t s)
{
    switch (bits) {
    case 2: return launch_encode_bits2(group, dtype, a, s);
    case 3: return launch_encode_bits3(group, dtype, a, s);
    case 4: return launch_encode_bits4(group, dtype, a, s);
    case 8: return launch_encode_bits8(group, dtype, a, s);
    }
    return KVC_ERR_UNSUPPORTED;
}

int launch_decode_section(int bits, int group, int dtype, const CoderBatch &a, hipStream_t s)
{
    (void)group;
    switch (bits) {
    case 2: return launch_decode_bits2(dtype, a, s);
    case 3: return launch_decode_bits3(dtype, a, s);
    case 4: return launch_decode_bits4(dtype, a, s);
    case 8: return launch_decode_bits8(dtype, a, s);
    }
    return KVC_ERR_UNSUPPORTED;
}

}  // namespace kvc
