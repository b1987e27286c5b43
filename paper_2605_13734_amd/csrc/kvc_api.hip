// Host side of the C ABI (include/kvc.h): plan validation, payload geometry and header,
// and the launch sequences of kvc_compress / kvc_decompress.  No device allocation, no
// synchronisation; everything is enqueued on the caller's stream.

#include <stdlib.h>
#include <string.h>

#include <mutex>

#include "../../include/kvc.h"
#include "kvc_internal.h"

using namespace kvc;

struct kvc_plan_s {
    kvc_model model;
    kvc_strategy strat;
    int64_t max_tokens;
    int32_t max_batch;
    size_t ws_request;          // workspace bytes per request
    size_t ws_state_off;        // offset of the scan state inside a request's workspace
    // per-head bit widths (section 5.1: head-wise mixed precision; the MixHQ mechanism)
    int has_table[2];           // K, V
    uint8_t *blob;              // host image of the device tables, see table_layout
    size_t blob_bytes;          // multiple of 256; the workspace starts with a copy of it
    int width_count[2][4];      // heads per width 2, 3, 4, 8
    // measurement hook (kvc_trace): events recorded between the stages of a call
    hipEvent_t *trace;
    int trace_cap, trace_n;
};

static const int kWidths[4] = {2, 3, 4, 8};
// limits that keep every byte count of a payload below 2^63
static const long long kMaxHeads = 1ll << 20, kMaxTokens = 1ll << 32;

// Device tables of a plan with per-head widths, in this order (LH = layers * kv_heads):
//   aux image : the bytes of the payload's auxiliary section (K table, V table, zero padding
//               to 16 bytes)
//   per tensor: long long bits_before[LH], then int head_list[LH] (heads grouped by width, in
//               the order 2, 3, 4, 8; head order kept inside a group)
struct TableLayout {
    size_t aux_image, bits_before[2], head_list[2], total;
};
static TableLayout table_layout(long long LH, int tables)
{
    TableLayout t;
    size_t at = 0;
    t.aux_image = at;
    at += (size_t)((tables * LH + 15) & ~15ll);
    at = (at + 255) & ~(size_t)255;
    for (int i = 0; i < 2; ++i) {
        t.bits_before[i] = at;
        at += (size_t)LH * 8;
        t.head_list[i] = at;
        at += (((size_t)LH * 4) + 7) & ~(size_t)7;
    }
    t.total = (at + 255) & ~(size_t)255;
    return t;
}

static int width_at(const kvc_plan_t *p, int is_v, long long lh)
{
    const uint8_t *t = is_v ? p->strat.head_bits_v : p->strat.head_bits_k;
    return t ? t[lh] : (is_v ? p->strat.bits_v : p->strat.bits_k);
}

// Optional measurement hook (kvc_trace): events recorded between the stages of a call, four per
// request: before anything of the request is enqueued, after its set-up, after K, after V.  Requests
// that share their launches (see request_window) share the moments.
struct Marks {
    kvc_plan_t *p;
    hipStream_t s;
    int base;
    Marks(const kvc_plan_t *plan, hipStream_t stream) : p(const_cast<kvc_plan_t *>(plan)), s(stream), base(p->trace_n) {}
    void at(int request, int stage) const
    {
        const int idx = base + 4 * request + stage;
        if (p->trace && idx < p->trace_cap && hipEventRecord(p->trace[idx], s) == hipSuccess && p->trace_n < idx + 1) p->trace_n = idx + 1;
    }
    void window(int first, int end, int stage) const
    {
        if (!p->trace) return;
        for (int i = first; i < end; ++i)
            if (!(stage == 0 && i == 0)) at(i, stage);      // (the first request's first mark opens the call)
    }
};

extern "C" int kvc_trace(kvc_plan_t *plan, void **hip_events, int32_t capacity)
{
    if (!plan) return 0;
    const int recorded = plan->trace_n;
    plan->trace = (hipEvent_t *)hip_events;
    plan->trace_cap = hip_events ? capacity : 0;
    plan->trace_n = 0;
    return recorded;
}

static inline long long a16(long long n) { return (n + 15) & ~15ll; }
static inline size_t a256(size_t n) { return (n + 255) & ~(size_t)255; }

static bool bits_ok(int b) { return b == 2 || b == 3 || b == 4 || b == 8 || b == 16; }
static bool group_ok(int g) { return g == 32 || g == 64 || g == 128; }

static long long chunks_per_head(long long tokens) { return (tokens + kChunkRows - 1) / kChunkRows; }

// Payload = header | K meta | V meta | auxiliary section | K codes | V codes, each part on a
// 16-byte boundary; two fp16 values of metadata per group (section 7.3).  The auxiliary section
// holds the coder's tables and directory or the per-head width tables, then (delta transform, from
// the next 16-byte boundary) the anchor rows of K and of V, 16 bits per element.
static long long anchor_rows(const kvc_plan_t *p, int is_v, long long T)
{
    if (p->strat.transform != KVC_T_DELTA) return 0;
    if (!p->has_table[is_v] && (is_v ? p->strat.bits_v : p->strat.bits_k) == 16) return 0;
    return (T + p->strat.anchor_period - 1) / p->strat.anchor_period;
}

static void geometry(const kvc_plan_t *p, long long T, Geometry *g)
{
    const long long LH = (long long)p->model.layers * p->model.kv_heads, D = p->model.head_dim;
    const int bk = p->strat.bits_k, bv = p->strat.bits_v;
    g->meta_k = (bk == 16 && !p->has_table[0]) ? 0 : 4 * LH * ((T + p->strat.group_k - 1) / p->strat.group_k) * D;
    g->meta_v = (bv == 16 && !p->has_table[1]) ? 0 : 4 * LH * T * (D / p->strat.group_v);
    long long sum_k = LH * bk, sum_v = LH * bv;          // widths summed over the heads
    if (p->has_table[0]) {
        sum_k = 0;
        for (long long i = 0; p->strat.head_bits_k && i < LH; ++i) sum_k += p->strat.head_bits_k[i];
    }
    if (p->has_table[1]) {
        sum_v = 0;
        for (long long i = 0; p->strat.head_bits_v && i < LH; ++i) sum_v += p->strat.head_bits_v[i];
    }
    g->codes_k = sum_k * T * D / 8;
    g->codes_v = sum_v * T * D / 8;
    g->chunks_k = g->chunks_v = LH * chunks_per_head(T);
    // with the coder: its tables (one per tensor, or one per tensor and width when there are width
    // tables), then the directory; then the width tables
    g->code_tables = p->strat.codec ? 256 * ((p->has_table[0] || p->has_table[1]) ? kTableSlots : 2) : 0;
    g->aux = p->strat.codec ? g->code_tables + 4 * (g->chunks_k + g->chunks_v + 1) : 0;
    g->widths = (p->has_table[0] + p->has_table[1]) * LH;
    const long long widths_at = g->aux;
    g->aux += g->widths;
    g->aux_base = g->aux;
    g->anchors_k = 2 * LH * anchor_rows(p, 0, T) * D;
    g->anchors_v = 2 * LH * anchor_rows(p, 1, T) * D;
    if (p->strat.transform == KVC_T_DELTA) g->aux = a16(g->aux_base) + g->anchors_k + g->anchors_v;
    g->off_meta_k = kHeader;
    g->off_meta_v = g->off_meta_k + a16(g->meta_k);
    g->off_aux = g->off_meta_v + a16(g->meta_v);
    g->off_dir = g->off_aux + g->code_tables;
    g->off_widths = g->off_aux + widths_at;
    g->off_codes_k = g->off_aux + a16(g->aux);
    g->off_anchors_k = g->off_codes_k - g->anchors_v - g->anchors_k;
    g->off_anchors_v = g->off_codes_k - g->anchors_v;
    g->off_codes_v = g->off_codes_k + a16(g->codes_k);
    g->total = g->off_codes_v + a16(g->codes_v);
}

static void put16(uint8_t *p, unsigned v) { p[0] = (uint8_t)v; p[1] = (uint8_t)(v >> 8); }
static void put32(uint8_t *p, uint32_t v) { for (int i = 0; i < 4; ++i) p[i] = (uint8_t)(v >> (8 * i)); }
static void put64(uint8_t *p, uint64_t v) { for (int i = 0; i < 8; ++i) p[i] = (uint8_t)(v >> (8 * i)); }
static unsigned get16(const uint8_t *p) { return p[0] | (p[1] << 8); }
static uint32_t get32(const uint8_t *p) { uint32_t v = 0; for (int i = 0; i < 4; ++i) v |= (uint32_t)p[i] << (8 * i); return v; }
static uint64_t get64(const uint8_t *p) { uint64_t v = 0; for (int i = 0; i < 8; ++i) v |= (uint64_t)p[i] << (8 * i); return v; }

// 128-byte little-endian header.  With the coder, the four size-dependent fields (total,
// K code bytes, V code offset, V code bytes) are left zero here and patched on the device.
static void make_header(const kvc_plan_t *p, long long T, const Geometry &g, HeaderBytes *out)
{
    uint8_t h[kHeader];
    memset(h, 0, sizeof h);
    memcpy(h, "KVC1", 4);
    put16(h + 4, 1);
    h[6] = p->model.dtype;
    h[7] = p->strat.codec;
    put32(h + 8, (uint32_t)p->model.layers);
    put32(h + 12, (uint32_t)p->model.kv_heads);
    put32(h + 16, (uint32_t)p->model.head_dim);
    h[20] = p->has_table[0] ? 0 : p->strat.bits_k;
    h[21] = p->has_table[1] ? 0 : p->strat.bits_v;
    put16(h + 22, p->strat.group_k);
    put16(h + 24, p->strat.group_v);
    h[26] = p->strat.transform;
    h[27] = (uint8_t)(p->has_table[0] | (p->has_table[1] << 1));
    put16(h + 28, p->strat.anchor_period);
    put64(h + 32, (uint64_t)T);
    put64(h + 48, (uint64_t)g.off_meta_k); put64(h + 56, (uint64_t)g.meta_k);
    put64(h + 64, (uint64_t)g.off_meta_v); put64(h + 72, (uint64_t)g.meta_v);
    put64(h + 80, (uint64_t)g.off_aux);    put64(h + 88, (uint64_t)g.aux);
    put64(h + 96, (uint64_t)g.off_codes_k);
    if (!p->strat.codec) {
        put64(h + 40, (uint64_t)g.total);
        put64(h + 104, (uint64_t)g.codes_k);
        put64(h + 112, (uint64_t)g.off_codes_v);
        put64(h + 120, (uint64_t)g.codes_v);
    }
    memcpy(out->w, h, kHeader);
}

extern "C" const char *kvc_status_string(int s)
{
    switch (s) {
    case KVC_OK: return "ok";
    case KVC_ERR_ARG: return "invalid argument";
    case KVC_ERR_UNSUPPORTED: return "unsupported configuration";
    case KVC_ERR_CAPACITY: return "capacity too small";
    case KVC_ERR_FORMAT: return "malformed payload";
    case KVC_ERR_MISMATCH: return "payload does not match plan";
    case KVC_ERR_DEVICE: return "HIP error";
    }
    return "unknown status";
}

static int check_pair(const kvc_model *m, const kvc_strategy *s)
{
    if (!m || !s) return KVC_ERR_ARG;
    if (m->dtype != KVC_F16 && m->dtype != KVC_BF16) return KVC_ERR_ARG;
    if (m->layers < 1 || m->kv_heads < 1 || m->head_dim < 1) return KVC_ERR_ARG;
    if ((long long)m->layers * m->kv_heads > kMaxHeads) return KVC_ERR_ARG;      // sizes stay far below 2^63
    if ((!s->head_bits_k && !bits_ok(s->bits_k)) || (!s->head_bits_v && !bits_ok(s->bits_v))) return KVC_ERR_ARG;
    if (s->codec != KVC_CODEC_NONE && s->codec != KVC_CODEC_HUFF8) return KVC_ERR_ARG;
    if ((s->head_bits_k || s->bits_k != 16) && !group_ok(s->group_k)) return KVC_ERR_ARG;
    if ((s->head_bits_v || s->bits_v != 16) && !group_ok(s->group_v)) return KVC_ERR_ARG;
    const long long LH = (long long)m->layers * m->kv_heads;
    for (int is_v = 0; is_v < 2; ++is_v) {
        const uint8_t *t = is_v ? s->head_bits_v : s->head_bits_k;
        if (!t) continue;
        if ((is_v ? s->bits_v : s->bits_k) != 0) return KVC_ERR_ARG;        // the table replaces the uniform width
        for (long long i = 0; i < LH; ++i)
            if (t[i] != 2 && t[i] != 3 && t[i] != 4 && t[i] != 8) return KVC_ERR_ARG;
    }
    if (m->head_dim != kDim) return KVC_ERR_UNSUPPORTED;
    if (s->transform > KVC_T_DELTA) return KVC_ERR_UNSUPPORTED;
    if (s->transform == KVC_T_DELTA) {
        const int a = s->anchor_period;
        if (a < 8 || a > 128 || (a & (a - 1))) return KVC_ERR_ARG;
    } else if (s->anchor_period != 0) return KVC_ERR_ARG;
    if (s->codec && (s->bits_k == 16 || s->bits_v == 16)) return KVC_ERR_UNSUPPORTED;
    return KVC_OK;
}

extern "C" int kvc_plan(const kvc_model *model, const kvc_strategy *strategy, int64_t max_tokens,
                        int32_t max_batch, kvc_plan_t **out)
{
    if (!out) return KVC_ERR_ARG;
    *out = nullptr;
    int rc = check_pair(model, strategy);
    if (rc) return rc;
    if (max_tokens < 0 || max_tokens > kMaxTokens || max_batch < 1) return KVC_ERR_ARG;
    kvc_plan_t *p = (kvc_plan_t *)calloc(1, sizeof(kvc_plan_t));
    if (!p) return KVC_ERR_ARG;
    p->model = *model;
    p->strat = *strategy;
    if (p->strat.bits_k == 16) p->strat.group_k = 32;       // unused; keep the header canonical
    if (p->strat.bits_v == 16) p->strat.group_v = 32;
    p->max_tokens = max_tokens;
    p->max_batch = max_batch;
    p->has_table[0] = strategy->head_bits_k ? 1 : 0;
    p->has_table[1] = strategy->head_bits_v ? 1 : 0;
    p->strat.head_bits_k = p->strat.head_bits_v = nullptr;
    if (p->has_table[0] || p->has_table[1]) {
        // the plan owns copies of the tables, inside the image of the device tables
        const long long LH = (long long)model->layers * model->kv_heads;
        const TableLayout t = table_layout(LH, p->has_table[0] + p->has_table[1]);
        p->blob = (uint8_t *)calloc(1, t.total);
        if (!p->blob) { free(p); return KVC_ERR_ARG; }
        p->blob_bytes = t.total;
        uint8_t *aux = p->blob + t.aux_image;
        if (p->has_table[0]) { memcpy(aux, strategy->head_bits_k, (size_t)LH); p->strat.head_bits_k = aux; aux += LH; }
        if (p->has_table[1]) { memcpy(aux, strategy->head_bits_v, (size_t)LH); p->strat.head_bits_v = aux; }
        for (int is_v = 0; is_v < 2; ++is_v) {
            if (!p->has_table[is_v]) continue;
            long long *before = (long long *)(p->blob + t.bits_before[is_v]);
            int *list = (int *)(p->blob + t.head_list[is_v]);
            long long sum = 0, at = 0;
            for (long long i = 0; i < LH; ++i) { before[i] = sum; sum += width_at(p, is_v, i); }
            for (int w = 0; w < 4; ++w) {
                p->width_count[is_v][w] = 0;
                for (long long i = 0; i < LH; ++i)
                    if (width_at(p, is_v, i) == kWidths[w]) { list[at++] = (int)i; ++p->width_count[is_v][w]; }
            }
        }
    }
    if (strategy->codec) {
        // histograms, encode tables, decode tables, ticket, then the scan state
        // one scan-state word per chunk of K and of V
        const long long chunks = (long long)model->layers * model->kv_heads * chunks_per_head(max_tokens);
        p->ws_state_off = 2 * a256(kTableSlots * 256 * 4) + a256(kTableSlots * 4096 * 2) + 256;
        p->ws_request = p->ws_state_off + a256((size_t)(2 * chunks) * 8 + 8);
    }
    *out = p;
    return KVC_OK;
}

extern "C" void kvc_plan_free(kvc_plan_t *plan)
{
    if (plan) free(plan->blob);
    free(plan);
}

extern "C" int kvc_payload_size(const kvc_plan_t *plan, int64_t tokens, uint64_t *bytes, int *is_exact)
{
    if (!plan || !bytes || tokens < 0 || tokens > kMaxTokens) return KVC_ERR_ARG;
    Geometry g;
    geometry(plan, tokens, &g);
    *bytes = (uint64_t)g.total;
    if (is_exact) *is_exact = plan->strat.codec == 0;
    return KVC_OK;
}

extern "C" size_t kvc_workspace_size(const kvc_plan_t *plan)
{
    return plan ? plan->blob_bytes + plan->ws_request * (size_t)plan->max_batch : 0;
}

extern "C" int kvc_payload_inspect(const void *header128, kvc_model *model, kvc_strategy *strategy,
                                   int64_t *tokens, uint64_t *total_bytes, uint64_t *sections)
{
    const uint8_t *h = (const uint8_t *)header128;
    if (!h) return KVC_ERR_ARG;
    if (memcmp(h, "KVC1", 4) != 0 || get16(h + 4) != 1) return KVC_ERR_FORMAT;
    kvc_model m;
    kvc_strategy s;
    memset(&m, 0, sizeof m);
    memset(&s, 0, sizeof s);
    m.dtype = h[6];
    s.codec = h[7];
    m.layers = (int32_t)get32(h + 8);
    m.kv_heads = (int32_t)get32(h + 12);
    m.head_dim = (int32_t)get32(h + 16);
    s.bits_k = h[20];
    s.bits_v = h[21];
    s.group_k = (uint16_t)get16(h + 22);
    s.group_v = (uint16_t)get16(h + 24);
    s.transform = h[26];
    s.anchor_period = (uint16_t)get16(h + 28);
    const int64_t T = (int64_t)get64(h + 32);
    // a tensor with a per-head width table has width 0 in the header; the table itself is in the
    // auxiliary section, which this function does not see
    const int flags = h[27];
    if (flags & ~3) return KVC_ERR_FORMAT;
    kvc_strategy probe = s;
    if (flags & 1) { if (s.bits_k) return KVC_ERR_FORMAT; probe.bits_k = 4; }
    if (flags & 2) { if (s.bits_v) return KVC_ERR_FORMAT; probe.bits_v = 4; }
    int rc = check_pair(&m, &probe);
    if (rc == KVC_ERR_ARG || T < 0 || T > kMaxTokens) return KVC_ERR_FORMAT;
    if (h[30] | h[31]) return KVC_ERR_FORMAT;
    // the fixed part of the section table must be the closed form of the fields above
    kvc_plan_t tmp;
    memset(&tmp, 0, sizeof tmp);
    tmp.model = m;
    tmp.strat = s;
    tmp.has_table[0] = flags & 1;
    tmp.has_table[1] = (flags >> 1) & 1;
    Geometry g;
    geometry(&tmp, T, &g);
    const uint64_t want[7] = {(uint64_t)g.off_meta_k, (uint64_t)g.meta_k, (uint64_t)g.off_meta_v,
                              (uint64_t)g.meta_v, (uint64_t)g.off_aux, (uint64_t)g.aux,
                              (uint64_t)g.off_codes_k};
    for (int i = 0; i < 7; ++i)
        if (get64(h + 48 + 8 * i) != want[i]) return KVC_ERR_FORMAT;
    const uint64_t total = get64(h + 40), ck = get64(h + 104), ov = get64(h + 112), cv = get64(h + 120);
    // with width tables the code sizes follow from the tables, which are not in the header: only the
    // bounds that hold for any table (2 to 8 bits per element) are known here
    const uint64_t unit = (uint64_t)m.layers * m.kv_heads * (uint64_t)T * 16;      // bytes per bit of width
    const uint64_t lo_k = (flags & 1) ? 2 * unit : (uint64_t)s.bits_k * unit, hi_k = (flags & 1) ? 8 * unit : lo_k;
    const uint64_t lo_v = (flags & 2) ? 2 * unit : (uint64_t)s.bits_v * unit, hi_v = (flags & 2) ? 8 * unit : lo_v;
    if (flags && s.codec) {
        if (ov != (uint64_t)g.off_codes_k + ck || total != ov + cv || (ck & 15) || (cv & 15) || ck > hi_k || cv > hi_v)
            return KVC_ERR_FORMAT;
    } else if (flags) {
        if (ck < lo_k || ck > hi_k || cv < lo_v || cv > hi_v || ov != (uint64_t)g.off_codes_k + (uint64_t)a16((long long)ck) ||
            total != ov + (uint64_t)a16((long long)cv))
            return KVC_ERR_FORMAT;
    } else if (!s.codec) {
        if (total != (uint64_t)g.total || ck != (uint64_t)g.codes_k || ov != (uint64_t)g.off_codes_v ||
            cv != (uint64_t)g.codes_v)
            return KVC_ERR_FORMAT;
    } else {
        if (ov != (uint64_t)g.off_codes_k + ck || total != ov + cv || total > (uint64_t)g.total ||
            (ck & 15) || (cv & 15))
            return KVC_ERR_FORMAT;
    }
    if (model) *model = m;
    if (strategy) *strategy = s;
    if (tokens) *tokens = T;
    if (total_bytes) *total_bytes = total;
    if (sections) {
        for (int i = 0; i < 7; ++i) sections[i] = want[i];
        sections[7] = ck; sections[8] = ov; sections[9] = cv;
    }
    return rc;     // KVC_OK, or KVC_ERR_UNSUPPORTED for a well-formed header this build cannot run
}

extern "C" int kvc_check_block_table(const int32_t *table, int64_t entries, int32_t num_phys_blocks)
{
    if (!table || entries < 0 || num_phys_blocks < 1) return KVC_ERR_ARG;
    for (int64_t i = 0; i < entries; ++i)
        if (table[i] < 0 || table[i] >= num_phys_blocks) return KVC_ERR_ARG;
    return KVC_OK;
}

static bool aligned16(const void *p) { return ((uintptr_t)p & 15) == 0; }

static int check_request(const kvc_plan_t *p, const kvc_request *r)
{
    if (r->tokens < 0) return KVC_ERR_ARG;
    if (r->tokens > p->max_tokens) return KVC_ERR_CAPACITY;
    if (r->tokens == 0) return KVC_OK;
    if (!r->k || !r->v || !aligned16(r->k) || !aligned16(r->v)) return KVC_ERR_ARG;
    if ((r->stride_layer | r->stride_head | r->stride_token) & 7) return KVC_ERR_ARG;
    if (r->stride_token < kDim) return KVC_ERR_ARG;
    if (r->block_table) {
        if (r->block_tokens < 1 || (r->block_tokens & (r->block_tokens - 1))) return KVC_ERR_UNSUPPORTED;
        if (r->num_phys_blocks < 1 || (r->stride_block & 7) || r->stride_block < 1) return KVC_ERR_ARG;
        if (((uintptr_t)r->block_table & 3)) return KVC_ERR_ARG;
    }
    return KVC_OK;
}

static TensorView view_of(const kvc_request *r, int is_v)
{
    TensorView v;
    v.base = (uint16_t *)(is_v ? r->v : r->k);
    v.stride_layer = r->stride_layer;
    v.stride_head = r->stride_head;
    v.stride_token = r->stride_token;
    v.stride_block = r->stride_block;
    v.block_table = r->block_table;
    v.bt_shift = 0;
    if (r->block_table)
        while ((1 << v.bt_shift) < r->block_tokens) ++v.bt_shift;
    v.num_phys_blocks = r->num_phys_blocks;
    v.bt_wave = (r->block_table && r->block_tokens >= 4 && r->stride_token < (1ll << 24) &&
                 (long long)r->block_tokens * r->stride_token < (1ll << 31)) ? 1 : 0;
    return v;
}

static QuantArgs quant_args(const kvc_plan_t *p, const kvc_request *r, int is_v, uint8_t *payload,
                            const Geometry &g, int *status, bool compress)
{
    QuantArgs a;
    memset(&a, 0, sizeof a);
    const int bits = is_v ? p->strat.bits_v : p->strat.bits_k;
    const int group = is_v ? p->strat.group_v : p->strat.group_k;
    a.x = view_of(r, is_v);
    a.codes = payload + (is_v ? g.off_codes_v : g.off_codes_k);
    a.meta = payload + (is_v ? g.off_meta_v : g.off_meta_k);
    a.tokens = r->tokens;
    a.heads = p->model.kv_heads;
    a.group = group;
    a.dense = (!r->block_table && r->stride_token == kDim) ? 1 : 0;
    a.head_minor = (r->stride_head < r->stride_token && !p->has_table[is_v]) ? 1 : 0;
    a.rotate = (p->strat.transform == KVC_T_HADAMARD && bits != 16) ? 1 : 0;
    if (anchor_rows(p, is_v, r->tokens) > 0) {
        a.anchors = (uint16_t *)(payload + (is_v ? g.off_anchors_v : g.off_anchors_k));
        while ((1 << a.anchor_shift) < p->strat.anchor_period) ++a.anchor_shift;
    }
    const long long rows_per_unit = (compress && !is_v && bits != 16) ? group : kPassRows;
    a.units_per_head = (r->tokens + rows_per_unit - 1) / rows_per_unit;
    a.total_units = a.units_per_head * p->model.layers * p->model.kv_heads;
    a.status = status;
    return a;
}

// One tensor of the requests of a window without the coder: one launch, or one per width present in
// the head table.
static int launch_tensor(const kvc_plan_t *p, int is_v, bool compress, QuantBatch b, const uint8_t *dev_tables, hipStream_t s)
{
    const int dt = p->model.dtype;
    const int group = is_v ? p->strat.group_v : p->strat.group_k;
    if (!p->has_table[is_v]) {
        const int bits = is_v ? p->strat.bits_v : p->strat.bits_k;
        return compress ? launch_compress_tensor(is_v, bits, group, dt, b, s) : launch_decompress_tensor(is_v, bits, group, dt, b, s);
    }
    const long long LH = (long long)p->model.layers * p->model.kv_heads;
    const TableLayout t = table_layout(LH, p->has_table[0] + p->has_table[1]);
    const int *list = (const int *)(dev_tables + t.head_list[is_v]);
    for (int w = 0; w < 4; ++w) {
        const int n = p->width_count[is_v][w];
        if (n > 0) {
            for (int i = 0; i < b.n; ++i) {
                b.item[i].bits_before = (const long long *)(dev_tables + t.bits_before[is_v]);
                b.item[i].head_list = list;
                b.item[i].total_units = b.item[i].units_per_head * n;
            }
            const int rc = compress ? launch_compress_tensor(is_v, kWidths[w], group, dt, b, s)
                                    : launch_decompress_tensor(is_v, kWidths[w], group, dt, b, s);
            if (rc) return rc;
        }
        list += n;
    }
    return KVC_OK;
}

// The requests [first, end) that share their launches: at most `limit`, of one layout class (the
// kernels for rows that are contiguous per head are not the ones for strided or paged rows), and
// small ones only -- a request that fills the chip many times over gains nothing from company, and
// finding its item costs every workgroup of a shared launch a look at the batch (measured: a batch of
// four 20k- to 30k-token requests ran 4 % slower shared than one after the other).  Empty requests
// have no work in any launch and fit every window.
static bool dense_layout(const kvc_request *r) { return !r->block_table && r->stride_token == kDim; }

static int request_window(const kvc_plan_t *p, const kvc_request *reqs, int n, int first, int limit, int *lead)
{
    const long long heads = (long long)p->model.layers * p->model.kv_heads;
    const long long kSmallRows = 1ll << 21;              // token rows per tensor: 64 Ki work units of 32 rows
    int end = first, leader = -1;
    while (end < n && end - first < limit) {
        if (reqs[end].tokens > 0) {
            const bool small = heads * reqs[end].tokens < kSmallRows;
            if (leader < 0) leader = end;
            else if (!small || heads * reqs[leader].tokens >= kSmallRows ||
                     dense_layout(&reqs[end]) != dense_layout(&reqs[leader])) break;
        }
        ++end;
    }
    *lead = leader < 0 ? first : leader;
    return end;
}

// the k-th request of a window in launch order: the leader (a request that has rows) first, because
// the launchers read the kernel variant off the first item, then the others in their order
static int window_item(int first, int end, int lead, int k)
{
    (void)end;
    if (k == 0) return lead;
    return first + k - 1 < lead ? first + k - 1 : first + k;
}

// the window's tensor as one batch
static QuantBatch quant_batch(const kvc_plan_t *plan, const kvc_request *reqs, int first, int end, int lead, int is_v,
                              void *payload, const uint64_t *payload_off, int32_t *dev_status, bool compress)
{
    QuantBatch b;
    memset(&b, 0, sizeof b);
    for (int k = 0; k < end - first; ++k) {
        const int i = window_item(first, end, lead, k);
        Geometry g;
        geometry(plan, reqs[i].tokens, &g);
        b.item[b.n++] = quant_args(plan, &reqs[i], is_v, (uint8_t *)payload + payload_off[i], g, dev_status + i, compress);
    }
    return b;
}

extern "C" size_t kvc_table_bytes(const kvc_plan_t *plan) { return plan ? plan->blob_bytes : 0; }

extern "C" int kvc_workspace_init(const kvc_plan_t *plan, void *workspace, void *hip_stream)
{
    if (!plan) return KVC_ERR_ARG;
    if (!plan->blob_bytes) return KVC_OK;
    if (!workspace || ((uintptr_t)workspace & 15)) return KVC_ERR_ARG;
    return hipMemcpyAsync(workspace, plan->blob, plan->blob_bytes, hipMemcpyHostToDevice, (hipStream_t)hip_stream) == hipSuccess
               ? KVC_OK : KVC_ERR_DEVICE;
}

// The coder launches of one request, in chunk order: K before V; a tensor with a width table is one
// launch per width present (2, 3, 4, 8) over the heads of that width, otherwise one launch.
struct CoderLaunch {
    CoderArgs a;
    int bits, group;
};

// launch j of the first n requests of a window as one batch
static CoderBatch coder_batch(const CoderLaunch cl[][kTableSlots], int n, int j)
{
    CoderBatch b;
    memset(&b, 0, sizeof b);
    for (int k = 0; k < n; ++k) b.item[k] = cl[k][j].a;
    b.n = n;
    return b;
}

static int coder_launches(const kvc_plan_t *p, const kvc_request *r, uint8_t *payload, const Geometry &g, uint8_t *ws,
                          long long capacity, uint64_t *out_bytes, int *status, bool compress, const uint8_t *dev_tables,
                          CoderLaunch out[kTableSlots])
{
    const bool any_table = p->has_table[0] || p->has_table[1];
    const long long LH = (long long)p->model.layers * p->model.kv_heads, cph = chunks_per_head(r->tokens);
    const TableLayout t = table_layout(LH, p->has_table[0] + p->has_table[1]);
    CoderArgs base;
    memset(&base, 0, sizeof base);
    base.payload = payload;
    base.off_aux = g.off_aux;
    base.off_dir = g.off_dir;
    base.off_bodies = g.off_codes_k;
    base.capacity = capacity;
    base.total_chunks = g.chunks_k + g.chunks_v;
    base.slots = any_table ? kTableSlots : 2;
    base.ws.hist = (uint32_t *)ws;
    base.ws.enc = (uint32_t *)(ws + a256(kTableSlots * 256 * 4));
    base.ws.lut = (uint16_t *)(ws + 2 * a256(kTableSlots * 256 * 4));
    base.ws.ticket = (uint32_t *)(ws + 2 * a256(kTableSlots * 256 * 4) + a256(kTableSlots * 4096 * 2));
    base.ws.state = (unsigned long long *)(ws + p->ws_state_off);
    base.out_bytes = (unsigned long long *)out_bytes;
    int n = 0, mask = 0;
    long long chunk_at = 0, wg_at = 0, k_wgs = 0;
    for (int is_v = 0; is_v < 2; ++is_v) {
        const QuantArgs q = quant_args(p, r, is_v, payload, g, status, compress);
        const int group = is_v ? p->strat.group_v : p->strat.group_k;
        const int *list = p->has_table[is_v] ? (const int *)(dev_tables + t.head_list[is_v]) : nullptr;
        for (int w = 0; w < 4; ++w) {
            long long heads = 0;
            if (p->has_table[is_v]) heads = p->width_count[is_v][w];
            else if (kWidths[w] == (is_v ? p->strat.bits_v : p->strat.bits_k)) heads = LH;
            if (heads == 0) continue;
            CoderLaunch &L = out[n++];
            L.a = base;
            L.a.q = q;
            L.a.q.head_list = list;                    // (null without a table: the heads in their own order)
            if (list) {
                L.a.q.bits_before = (const long long *)(dev_tables + t.bits_before[is_v]);
                list += heads;
            }
            L.bits = kWidths[w];
            L.group = group;
            L.a.is_v = is_v;
            L.a.tab = any_table ? 4 * is_v + w : is_v;
            L.a.chunks = heads * cph;
            L.a.chunk_base = chunk_at;
            L.a.wg_base = wg_at;
            const int nw = enc_waves(L.bits, group, p->model.dtype, q.dense != 0, is_v != 0, q.rotate || q.anchors != nullptr);
            chunk_at += L.a.chunks;
            wg_at += (L.a.chunks + nw - 1) / nw;
            mask |= 1 << L.a.tab;
        }
        if (!is_v) k_wgs = wg_at;
    }
    for (int i = 0; i < n; ++i) {
        out[i].a.k_wgs = k_wgs;
        out[i].a.total_wgs = wg_at;
        out[i].a.slot_mask = mask;
    }
    return n;
}

static int check_batch(const kvc_plan_t *p, const kvc_request *reqs, int32_t n, const void *payload,
                       const uint64_t *off, const void *workspace)
{
    if (!p || !reqs || n < 1 || !payload || !off || !aligned16(payload)) return KVC_ERR_ARG;
    if (n > p->max_batch) return KVC_ERR_CAPACITY;
    if ((p->ws_request || p->blob_bytes) && (!workspace || !aligned16(workspace))) return KVC_ERR_ARG;
    for (int i = 0; i < n; ++i) {
        int rc = check_request(p, &reqs[i]);
        if (rc) return rc;
        if ((off[i] & 15) || off[i + 1] < off[i]) return KVC_ERR_ARG;
    }
    return KVC_OK;
}

#define KVC_TRY(expr) do { int rc__ = (expr); if (rc__ != KVC_OK) return rc__; } while (0)

// The launch sequence of kvc_compress on a given workspace (the caller's, or the library's own
// static one): one service launch for all requests, then per request the coder's tables and one
// pass per tensor.
static int compress_on(const kvc_plan_t *plan, const kvc_request *reqs, int32_t n, void *payload,
                       const uint64_t *payload_off, uint64_t *out_bytes, int32_t *dev_status,
                       void *workspace, hipStream_t s)
{
    KVC_TRY(check_batch(plan, reqs, n, payload, payload_off, workspace));
    if (!out_bytes || !dev_status || ((uintptr_t)out_bytes & 7) || ((uintptr_t)dev_status & 3)) return KVC_ERR_ARG;
    for (int i = 0; i < n; ++i) {
        Geometry g;
        geometry(plan, reqs[i].tokens, &g);
        if (payload_off[i + 1] - payload_off[i] < (uint64_t)g.total) return KVC_ERR_CAPACITY;
    }
    const kvc_strategy &st = plan->strat;
    const int dt = plan->model.dtype;
    const Marks marks(plan, s);
    marks.at(0, 0);
    for (int first = 0; first < n; first += kPrologueBatch) {
        PrologueArgs pa;
        memset(&pa, 0, sizeof pa);
        pa.n = n - first < kPrologueBatch ? n - first : kPrologueBatch;
        for (int j = 0; j < pa.n; ++j) {
            const int i = first + j;
            Geometry g;
            geometry(plan, reqs[i].tokens, &g);
            uint8_t *pl = (uint8_t *)payload + payload_off[i];
            PrologueItem &it = pa.item[j];
            it.payload = (uint32_t *)pl;
            make_header(plan, reqs[i].tokens, g, &it.header);
            // alignment padding after the V metadata and after the coder's or the width tables is zero
            it.pad_off[0] = g.off_meta_v + g.meta_v;
            it.pad_words[0] = (a16(g.meta_v) - g.meta_v) / 4;
            it.pad_off[1] = g.off_aux + g.aux_base;
            it.pad_words[1] = (a16(g.aux_base) - g.aux_base) / 4;
            if (plan->blob_bytes) {
                // the width tables: a copy of the image at the start of the workspace (whole words; the
                // image is zero behind the tables), then zero up to the next 16-byte boundary
                it.aux_src = (const uint32_t *)workspace;
                it.aux_off = g.off_widths;
                it.aux_words = (g.widths + 3) / 4;
                it.pad_off[1] = g.off_widths + 4 * it.aux_words;
                it.pad_words[1] = (g.off_aux + a16(g.aux_base) - it.pad_off[1]) / 4;
            }
            it.out_bytes = (unsigned long long *)(out_bytes + i);
            it.status = dev_status + i;
            if (!st.codec) {
                it.total = (unsigned long long)g.total;
                it.write_total = 1;
            } else {
                uint8_t *ws = (uint8_t *)workspace + plan->blob_bytes + (size_t)i * plan->ws_request;
                CoderLaunch cl[kTableSlots];
                const int launches = coder_launches(plan, &reqs[i], pl, g, ws, 0, nullptr, dev_status + i, true,
                                                    (const uint8_t *)workspace, cl);
                const CoderArgs &c = cl[0].a;              // (a request has at least one K and one V launch)
                (void)launches;
                // histograms, ticket and scan state start from zero
                it.zero[0] = c.ws.hist;
                it.zero_words[0] = kTableSlots * 256;
                it.zero[1] = c.ws.ticket;
                it.zero_words[1] = 64 + 2 * c.total_wgs + 2;
                if (c.total_chunks == 0) {
                    // empty request: no workgroup runs that could close the directory and header
                    put64((uint8_t *)it.header.w + 40, (uint64_t)g.off_codes_k);
                    put64((uint8_t *)it.header.w + 112, (uint64_t)g.off_codes_k);
                    it.dir0 = (uint32_t *)(pl + g.off_dir);
                    it.total = (unsigned long long)g.off_codes_k;
                    it.write_total = 1;
                }
            }
        }
        KVC_TRY(launch_compress_prologue(pa, s));
    }
    for (int first = 0; first < n;) {
        int lead;
        const int end = request_window(plan, reqs, n, first, st.codec ? kCoderBatch : kQuantBatch, &lead);
        marks.window(first, end, 0);
        if (!st.codec) {
            marks.window(first, end, 1);
            KVC_TRY(launch_tensor(plan, 0, true, quant_batch(plan, reqs, first, end, lead, 0, payload, payload_off, dev_status, true),
                                  (const uint8_t *)workspace, s));
            marks.window(first, end, 2);
            KVC_TRY(launch_tensor(plan, 1, true, quant_batch(plan, reqs, first, end, lead, 1, payload, payload_off, dev_status, true),
                                  (const uint8_t *)workspace, s));
            marks.window(first, end, 3);
        } else {
            // the coder launches of every request of the window (the same list for all: K before V,
            // widths ascending), then launch by launch over the requests together
            CoderLaunch cl[kCoderBatch][kTableSlots];
            int launches = 0;
            for (int k = 0; k < end - first; ++k) {
                const int i = window_item(first, end, lead, k);
                Geometry g;
                geometry(plan, reqs[i].tokens, &g);
                uint8_t *ws = (uint8_t *)workspace + plan->blob_bytes + (size_t)i * plan->ws_request;
                launches = coder_launches(plan, &reqs[i], (uint8_t *)payload + payload_off[i], g, ws,
                                          (long long)(payload_off[i + 1] - payload_off[i]), out_bytes + i, dev_status + i, true,
                                          (const uint8_t *)workspace, cl[k]);
            }
            for (int j = 0; j < launches; ++j)
                KVC_TRY(launch_table_sample(cl[0][j].bits, cl[0][j].group, dt, coder_batch(cl, end - first, j), s));
            KVC_TRY(launch_build_tables(coder_batch(cl, end - first, 0), s));
            marks.window(first, end, 1);
            for (int j = 0; j < launches; ++j)
                if (!cl[0][j].a.is_v) KVC_TRY(launch_encode_section(cl[0][j].bits, cl[0][j].group, dt, coder_batch(cl, end - first, j), s));
            marks.window(first, end, 2);
            for (int j = 0; j < launches; ++j)
                if (cl[0][j].a.is_v) KVC_TRY(launch_encode_section(cl[0][j].bits, cl[0][j].group, dt, coder_batch(cl, end - first, j), s));
            marks.window(first, end, 3);
        }
        first = end;
    }
    return KVC_OK;
}

extern "C" int kvc_compress(const kvc_plan_t *plan, const kvc_request *reqs, int32_t n, void *payload,
                            const uint64_t *payload_off, uint64_t *out_bytes, int32_t *dev_status,
                            void *workspace, void *hip_stream)
{
    return compress_on(plan, reqs, n, payload, payload_off, out_bytes, dev_status, workspace, (hipStream_t)hip_stream);
}

// ---- kvc_compress for callers that cannot allocate: the workspace is a static device array ----

// Every GPU the library runs on holds its own copy of this array until the process ends.  In host
// code the name is only a handle for hipGetSymbolAddress; the address it returns, one per device,
// is what the kernels and fills receive.
static __device__ __align__(256) unsigned char scratch[KVC_STATIC_WORKSPACE_BYTES];

static const int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_lock;

// the current device's copy of `scratch` (looked up once per device)
static int static_workspace(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return KVC_ERR_DEVICE;
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return KVC_ERR_DEVICE;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return KVC_OK;
}

extern "C" int kvc_compress_static(const kvc_plan_t *plan, const kvc_request *reqs, int32_t n, void *payload,
                                   const uint64_t *payload_off, uint64_t *out_bytes, int32_t *dev_status,
                                   void *hip_stream)
{
    if (!plan) return KVC_ERR_ARG;
    if (plan->blob_bytes) return KVC_ERR_UNSUPPORTED;      // width tables live in a caller workspace (kvc_workspace_init)
    if (kvc_workspace_size(plan) > (size_t)KVC_STATIC_WORKSPACE_BYTES) return KVC_ERR_CAPACITY;
    void *ws = nullptr;
    KVC_TRY(static_workspace(&ws));
    return compress_on(plan, reqs, n, payload, payload_off, out_bytes, dev_status, ws, (hipStream_t)hip_stream);
}

extern "C" int kvc_decompress(const kvc_plan_t *plan, const void *payload, const uint64_t *payload_off,
                              const kvc_request *dst, int32_t n, int32_t *dev_status, void *workspace,
                              void *hip_stream)
{
    KVC_TRY(check_batch(plan, dst, n, payload, payload_off, workspace));
    if (!dev_status || ((uintptr_t)dev_status & 3)) return KVC_ERR_ARG;
    const kvc_strategy &st = plan->strat;
    for (int i = 0; i < n; ++i) {
        Geometry g;
        geometry(plan, dst[i].tokens, &g);
        const long long cap = (long long)(payload_off[i + 1] - payload_off[i]);
        if (cap < kHeader || (!st.codec && cap < g.total) || (st.codec && cap < g.off_codes_k)) return KVC_ERR_CAPACITY;
    }
    hipStream_t s = (hipStream_t)hip_stream;
    const int dt = plan->model.dtype;
    const Marks marks(plan, s);
    marks.at(0, 0);
    for (int first = 0; first < n; first += kCheckBatch) {
        CheckArgs ca;
        memset(&ca, 0, sizeof ca);
        ca.n = n - first < kCheckBatch ? n - first : kCheckBatch;
        for (int j = 0; j < ca.n; ++j) {
            const int i = first + j;
            Geometry g;
            geometry(plan, dst[i].tokens, &g);
            const uint8_t *pl = (const uint8_t *)payload + payload_off[i];
            CheckItem &it = ca.item[j];
            it.payload = (const uint32_t *)pl;
            make_header(plan, dst[i].tokens, g, &it.expect);
            // words 10/11 (total), 26..31 (code sizes) depend on the data when the coder is on
            it.mask = st.codec ? 0x03fff3ffu : 0xffffffffu;
            if (plan->blob_bytes) {       // the payload's width tables must be the plan's
                it.tables = pl + g.off_widths;
                it.plan_tables = (const uint8_t *)workspace;
                it.table_bytes = g.widths;
            }
            it.status = dev_status + i;
        }
        KVC_TRY(launch_decompress_prologue(ca, s));
    }
    for (int first = 0; first < n;) {
        int lead;
        const int end = request_window(plan, dst, n, first, st.codec ? kCoderBatch : kQuantBatch, &lead);
        marks.window(first, end, 0);
        if (!st.codec) {
            marks.window(first, end, 1);
            KVC_TRY(launch_tensor(plan, 0, false, quant_batch(plan, dst, first, end, lead, 0, const_cast<void *>(payload), payload_off, dev_status, false),
                                  (const uint8_t *)workspace, s));
            marks.window(first, end, 2);
            KVC_TRY(launch_tensor(plan, 1, false, quant_batch(plan, dst, first, end, lead, 1, const_cast<void *>(payload), payload_off, dev_status, false),
                                  (const uint8_t *)workspace, s));
            marks.window(first, end, 3);
        } else {
            CoderLaunch cl[kCoderBatch][kTableSlots];
            int launches = 0;
            for (int k = 0; k < end - first; ++k) {
                const int i = window_item(first, end, lead, k);
                Geometry g;
                geometry(plan, dst[i].tokens, &g);
                uint8_t *ws = (uint8_t *)workspace + plan->blob_bytes + (size_t)i * plan->ws_request;
                launches = coder_launches(plan, &dst[i], (uint8_t *)payload + payload_off[i], g, ws,
                                          (long long)(payload_off[i + 1] - payload_off[i]), nullptr, dev_status + i, false,
                                          (const uint8_t *)workspace, cl[k]);
            }
            KVC_TRY(launch_decode_prepare(coder_batch(cl, end - first, 0), s));
            marks.window(first, end, 1);
            for (int j = 0; j < launches; ++j)
                if (!cl[0][j].a.is_v) KVC_TRY(launch_decode_section(cl[0][j].bits, cl[0][j].group, dt, coder_batch(cl, end - first, j), s));
            marks.window(first, end, 2);
            for (int j = 0; j < launches; ++j)
                if (cl[0][j].a.is_v) KVC_TRY(launch_decode_section(cl[0][j].bits, cl[0][j].group, dt, coder_batch(cl, end - first, j), s));
            marks.window(first, end, 3);
        }
        first = end;
    }
    return KVC_OK;
}
