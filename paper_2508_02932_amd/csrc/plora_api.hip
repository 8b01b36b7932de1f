// Host side of libplora: argument validation, the segment-packing metadata builder, workspace
// layout and the launch sequences of the forward and backward calls.  No arithmetic of the layer
// happens here; every step runs in the HIP kernels.
#include "plora_internal.h"
#include "plora_bench.h"
#include "plora_debug.h"

#include <cmath>
#include <cstring>
#include <algorithm>
#include <memory>
#include <mutex>
#include <new>
#include <vector>

namespace plora {

// Limits that keep every index of every kernel inside the type it is computed in: 32-bit byte offsets inside a
// GEMM tile (255 rows x d x 2 bytes), int tile counts, 65535 workgroups along y in the fp32 kernels.
constexpr int64_t kMaxHidden = 1 << 22;
constexpr int64_t kMaxTiles = 1 << 30;

static plora_status validate(const plora_desc *d)
{
    if (!d) return PLORA_ERR_NULL;
    if (d->dtype != PLORA_BF16 && d->dtype != PLORA_F32) return PLORA_ERR_UNSUPPORTED;
    if (d->w_layout != PLORA_W_IN_OUT && d->w_layout != PLORA_W_OUT_IN) return PLORA_ERR_UNSUPPORTED;
    if (d->T < 0 || d->d_in <= 0 || d->d_out <= 0) return PLORA_ERR_SHAPE;
    if (d->T > INT32_MAX || d->d_in > kMaxHidden || d->d_out > kMaxHidden) return PLORA_ERR_SHAPE;
    if (d->dtype == PLORA_BF16 && (d->d_in % 8 != 0 || d->d_out % 8 != 0)) return PLORA_ERR_SHAPE;
    {
        const int64_t tm = (d->T + kGemmTileRows - 1) / kGemmTileRows;
        const int64_t tn = (std::max(d->d_in, d->d_out) + 255) / 256;
        if (tm * tn > kMaxTiles) return PLORA_ERR_SHAPE;
        if (d->dtype == PLORA_F32 && (d->T + 63) / 64 > 65535) return PLORA_ERR_SHAPE;
    }
    if (d->n_seg < 0 || d->n_seg > PLORA_MAX_SEGMENTS) return PLORA_ERR_SEGMENTS;
    if (d->n_adapters < 0 || d->n_adapters > PLORA_MAX_ADAPTERS) return PLORA_ERR_ADAPTER;
    if (d->n_seg == 0) return d->T == 0 ? PLORA_OK : PLORA_ERR_SEGMENTS;
    if (!d->seg_off || !d->seg_adapter) return PLORA_ERR_NULL;
    if (d->n_adapters > 0 && (!d->rank || !d->scale)) return PLORA_ERR_NULL;
    for (int32_t k = 0; k < d->n_adapters; ++k)
        if (d->rank[k] < 1 || d->rank[k] > PLORA_MAX_RANK) return PLORA_ERR_RANK;
    if (d->seg_off[0] != 0 || d->seg_off[d->n_seg] != d->T) return PLORA_ERR_SEGMENTS;
    for (int32_t s = 0; s < d->n_seg; ++s) {
        if (d->seg_off[s + 1] < d->seg_off[s]) return PLORA_ERR_SEGMENTS;
        if (d->seg_adapter[s] < -1 || d->seg_adapter[s] >= d->n_adapters) return PLORA_ERR_ADAPTER;
    }
    return PLORA_OK;
}

// Compact description of a call (the words the preparation kernel receives).  Pointer tables may be null.
// at_base: device address of the packed-A^T region of the workspace (null when only the layout matters).
static void fill_desc_words(const plora_desc *d, int32_t n_blocks, const void *const *A, const void *const *B,
                            float *const *dA, float *const *dB, const void *at_base, bool order_is_identity, uint32_t *w)
{
    auto put64 = [&](int i, uint64_t v) { w[i] = (uint32_t)v; w[i + 1] = (uint32_t)(v >> 32); };
    put64(0, (uint64_t)d->T); put64(2, (uint64_t)d->d_in); put64(4, (uint64_t)d->d_out);
    w[6] = (uint32_t)d->n_seg; w[7] = (uint32_t)d->n_adapters; w[8] = (uint32_t)n_blocks;
    w[9] = (d->w_layout == PLORA_W_OUT_IN ? 1u : 0u) | (order_is_identity ? 2u : 0u);
    put64(10, (uint64_t)(uintptr_t)at_base);
    uint32_t *p = w + kDescHeadWords;
    for (int32_t s = 0; s < d->n_seg; ++s) { *p++ = (uint32_t)d->seg_off[s + 1]; *p++ = (uint32_t)d->seg_adapter[s]; }
    for (int32_t k = 0; k < d->n_adapters; ++k) {
        const int i = (int)(p - w);
        put64(i + 0, (uint64_t)(uintptr_t)(A ? A[k] : nullptr));
        put64(i + 2, (uint64_t)(uintptr_t)(B ? B[k] : nullptr));
        put64(i + 4, (uint64_t)(uintptr_t)(dA ? dA[k] : nullptr));
        put64(i + 6, (uint64_t)(uintptr_t)(dB ? dB[k] : nullptr));
        w[i + 8] = (uint32_t)d->rank[k];
        std::memcpy(&w[i + 9], &d->scale[k], 4);
        p += kDescAdWords;
    }
}

// Everything the host derives from a description: the tables (same code as the device runs), the
// launch plans and the workspace layout.  Depends on the description only (not on pointers or scales),
// so it is kept in a small cache and shared by the calls that repeat a layout - the seven linears of a
// decoder layer, every layer, forward and backward.
struct HostMeta {
    TableLayout layout;
    std::vector<char> image;          // the tables as the device lays them out (pointer fields null)
    Tables t;
    MetaHeader hdr;
    WorkspaceLayout ws;               // plora_linear_fwd / _bwd
    WorkspaceLayout ws_lora;          // plora_lora_fwd / _bwd: the padded small-matrix region holds [max(d_in, d_out)][rp]
    size_t h_elems = 0, hb_elems = 0, zt_elems = 0, at_elems = 0, ap_elems = 0;
    int r16_total = 0, n_active = 0, split_dA = 1, split_dB = 1, bc_dA = 256, bc_dB = 256;
    int split_shrink = 1, split_dh = 1;
    int n_words = 0;
    bool order_is_identity = false;   // the sorted order of the GEMM row tiles is 0, 1, 2, ...: the device need not sort
};

static void build_meta(const plora_desc *d, HostMeta &m)
{
    int32_t n_blocks = 0;
    for (int32_t s = 0; s < d->n_seg; ++s)
        if (d->seg_adapter[s] >= 0) n_blocks += (d->seg_off[s + 1] - d->seg_off[s] + kSkinnyRows - 1) / kSkinnyRows;
    m.n_words = desc_words(d->n_seg, d->n_adapters);
    std::vector<uint32_t> words((size_t)m.n_words);
    fill_desc_words(d, n_blocks, nullptr, nullptr, nullptr, nullptr, nullptr, false, words.data());
    m.layout = table_layout(d->T, d->n_seg, d->n_adapters, n_blocks);
    m.image.assign(m.layout.bytes, 0);
    m.t = tables_at(m.image.data(), m.layout);
    const DescReader<WordsInMemory> in{WordsInMemory{words.data()}};
    std::vector<int32_t> scratch(3 * (size_t)d->n_adapters + 1);
    derive_phase1(in, m.t, scratch.data(), nullptr, nullptr, nullptr);
    derive_phase2(m.t, *m.t.hdr, m.t.seg, m.t.ad, scratch.data() /* tokens */, 0, 1);
    {
        int32_t counts[kSortKeys], starts[kSortKeys];
        derive_phase3_count(m.t, m.layout.n_tiles, 0, 1, counts);
        derive_phase3_scan(0, 1, counts, starts);
        derive_phase3_place(m.t, m.layout.n_tiles, 0, 1, starts);
    }
    m.order_is_identity = true;
    for (int64_t i = 0; i < m.layout.n_tiles; ++i) m.order_is_identity = m.order_is_identity && m.t.tile_order[i] == (int32_t)i;
    m.hdr = *m.t.hdr;

    int64_t h = 0, hb = 0, zt = 0, at = 0, ap = 0;
    for (int32_t s = 0; s < d->n_seg; ++s) {
        const SegInfo &g = m.t.seg[s];
        if (g.adapter < 0) continue;
        const int64_t len = g.row1 - g.row0;
        h += len * g.r; hb += len * g.rp; zt += (int64_t)g.r16 * g.lp;
    }
    m.r16_total = 0; m.n_active = 0;
    for (int32_t k = 0; k < d->n_adapters; ++k) {
        const AdapterInfo &a = m.t.ad[k];
        at += (int64_t)a.r16 * d->d_in;
        ap += (int64_t)a.rp * (m.hdr.w_out_in ? d->d_out : d->d_in);
        m.r16_total += a.r16;
        m.n_active += a.tokens > 0;
    }
    m.h_elems = (size_t)h; m.hb_elems = (size_t)hb; m.zt_elems = (size_t)zt;
    m.at_elems = (size_t)at; m.ap_elems = (size_t)ap;
    m.split_dA = tokc_splits(m.hdr, d->d_in, m.n_active);
    m.split_dB = tokc_splits(m.hdr, d->d_out, m.n_active);
    m.bc_dA = tokc_tile_columns(m.hdr, d->d_in, m.n_active);
    m.bc_dB = tokc_tile_columns(m.hdr, d->d_out, m.n_active);
    m.split_shrink = skinny_splits(m.hdr, d->d_in);
    m.split_dh = skinny_splits(m.hdr, d->d_out);

    const bool bf = d->dtype == PLORA_BF16;
    auto lay_out = [&](WorkspaceLayout &w, size_t ap_elems) {
        size_t o = 0;
        w.zero = o; o += kZeroBytes;
        w.meta_bytes = m.layout.bytes;
        w.meta = o; o = align_up(o + w.meta_bytes, 256);
        w.desc = o; o = align_up(o + (m.n_words > kChunkWords ? (size_t)m.n_words * 4 : 0), 256);
        w.at = o;   o = align_up(o + (bf ? m.at_elems * 2 : 0), 256);
        w.ap = o;   o = align_up(o + (bf ? ap_elems * 2 : 0), 256);
        w.hb = o;   o = align_up(o + (bf ? m.hb_elems * 2 : 0), 256);
        w.zt_h = o; o = align_up(o + (bf ? m.zt_elems * 2 : 0), 256);
        w.zt_g = o; o = align_up(o + (bf ? m.zt_elems * 2 : 0), 256);
        w.hf = o;   o = align_up(o + m.h_elems * 4, 256);
        w.gf = o;   o = align_up(o + (bf ? 0 : m.h_elems * 4), 256);
        w.part = o; o = align_up(o + (bf ? (size_t)kSkinnyMaxSplits * m.hdr.n_blocks * kSkinnyRows * m.hdr.max_r16 * 4 : 0), 256);
        const size_t a_bytes = m.split_dA > 1 ? (size_t)m.split_dA * m.r16_total * d->d_in * 4 : 0;
        const size_t b_bytes = m.split_dB > 1 ? (size_t)m.split_dB * m.r16_total * d->d_out * 4 : 0;
        w.wpart = o; o = align_up(o + (bf ? (a_bytes > b_bytes ? a_bytes : b_bytes) : 0), 256);
        w.total = o + 256;
    };
    lay_out(m.ws, m.ap_elems);
    int64_t rp_total = 0;
    for (int32_t k = 0; k < d->n_adapters; ++k) rp_total += m.t.ad[k].rp;
    lay_out(m.ws_lora, (size_t)(rp_total * std::max(d->d_in, d->d_out)));
}

// ---- metadata cache: the last few descriptions and what was derived from them ---------------------
struct CacheEntry {
    std::vector<int64_t> key;
    std::shared_ptr<const HostMeta> meta;
    uint64_t stamp = 0;
};
constexpr int kCacheEntries = 16;
static std::mutex g_cache_mu;
static CacheEntry g_cache[kCacheEntries];
static uint64_t g_cache_clock = 0;

static void key_of(const plora_desc *d, std::vector<int64_t> &k)
{
    k.clear();
    k.reserve(6 + 2 * (size_t)d->n_seg + (size_t)d->n_adapters);
    k.push_back(d->T); k.push_back(d->d_in); k.push_back(d->d_out); k.push_back(d->dtype + 16 * (int64_t)d->w_layout);
    k.push_back(d->n_seg); k.push_back(d->n_adapters);
    for (int32_t s = 0; s < d->n_seg; ++s) { k.push_back(d->seg_off[s + 1]); k.push_back(d->seg_adapter[s]); }
    for (int32_t a = 0; a < d->n_adapters; ++a) k.push_back(d->rank[a]);
}

// The derived metadata of a valid description (from the cache when the same layout was seen lately).
static std::shared_ptr<const HostMeta> meta_of(const plora_desc *d)
{
    thread_local std::vector<int64_t> key;
    key_of(d, key);
    {
        std::lock_guard<std::mutex> lock(g_cache_mu);
        for (CacheEntry &e : g_cache)
            if (e.meta && e.key == key) { e.stamp = ++g_cache_clock; return e.meta; }
    }
    auto fresh = std::make_shared<HostMeta>();
    build_meta(d, *fresh);
    std::lock_guard<std::mutex> lock(g_cache_mu);
    CacheEntry *victim = &g_cache[0];
    for (CacheEntry &e : g_cache)
        if (e.stamp < victim->stamp) victim = &e;
    victim->key = key; victim->meta = fresh; victim->stamp = ++g_cache_clock;
    return fresh;
}

// ---- bench-only kernel timing (declared in plora_bench.h) -------------------------------------------
// Every kernel class of a call is bracketed by a pair of HIP events recorded on the call's own
// stream; pairs come from a pool that is filled while timing is enabled and summed on request.
constexpr int kClasses = 10;
constexpr int kMaxPairs = 16384;
static int g_timing = 0;
static std::vector<hipEvent_t> g_pool;            // 2 events per pair, created on demand
static std::vector<int> g_pair_class;             // class of each recorded pair

struct Bracket {
    int pair; hipStream_t st;
    Bracket(int cls, hipStream_t s) : pair(-1), st(s)
    {
        if (!g_timing || (int)g_pair_class.size() >= kMaxPairs) return;
        pair = (int)g_pair_class.size();
        if ((int)g_pool.size() < 2 * (pair + 1)) {
            hipEvent_t a, b;
            if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) { pair = -1; return; }
            g_pool.push_back(a); g_pool.push_back(b);
        }
        g_pair_class.push_back(cls);
        (void)hipEventRecord(g_pool[2 * pair], st);
    }
    ~Bracket() { if (pair >= 0) (void)hipEventRecord(g_pool[2 * pair + 1], st); }
};

#define PL_TRY(expr) do { hipError_t e__ = (expr); if (e__ != hipSuccess) return PLORA_ERR_HIP; } while (0)

static bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// One call's host state: the cached metadata and the compact description with this call's pointers.
struct Call {
    std::shared_ptr<const HostMeta> m;
    const WorkspaceLayout *L = nullptr;      // the workspace layout of this kind of call (inside *m)
    uint32_t small[kChunkWords];
    std::vector<uint32_t> large;
    const uint32_t *words = nullptr;
};

// Checks shared by forward and backward.  lora_only: the stand-alone low-rank calls (no W, their own workspace layout).
static plora_status prepare(const plora_desc *d, const void *x, const void *W, const void *const *A,
                            const void *const *B, float *const *dA, float *const *dB, void *workspace, size_t ws_bytes,
                            bool lora_only, Call &c)
{
    plora_status st = validate(d);
    if (st != PLORA_OK) return st;
    if (!x && d->T > 0) return PLORA_ERR_NULL;
    if (!W && !lora_only) return PLORA_ERR_NULL;
    if (d->n_adapters > 0 && (!A || !B)) return PLORA_ERR_NULL;
    for (int32_t k = 0; k < d->n_adapters; ++k) {
        if (!A[k] || !B[k]) return PLORA_ERR_NULL;
        if (misaligned(A[k]) || misaligned(B[k])) return PLORA_ERR_ALIGN;
    }
    if (misaligned(x) || misaligned(W)) return PLORA_ERR_ALIGN;
    c.m = meta_of(d);
    c.L = lora_only ? &c.m->ws_lora : &c.m->ws;
    if (!workspace || ws_bytes < c.L->total) return PLORA_ERR_WORKSPACE;
    if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return PLORA_ERR_ALIGN;
    uint32_t *w = c.small;
    if (c.m->n_words > kChunkWords) { c.large.resize((size_t)c.m->n_words); w = c.large.data(); }
    fill_desc_words(d, c.m->hdr.n_blocks, A, B, dA, dB, static_cast<const char *>(workspace) + c.L->at, c.m->order_is_identity, w);
    c.words = w;
    return PLORA_OK;
}

static MetaView device_view(const HostMeta &m, const WorkspaceLayout &L, char *ws)
{
    return view_of(tables_at(ws + L.meta, m.layout));
}

// Steps of a call, so that a grouped call can run a fused pass of its own between them (a plain call runs them all).
enum : unsigned {
    kStepPrep = 1u, kStepShrink = 2u, kStepMain = 4u,      // forward: prep, shrink, GEMM (or stand-alone update)
    kStepDh = 8u, kStepDb = 16u, kStepDa = 32u, kStepDx = 64u,   // backward: prep, shrink, dH, dB, dA, dX
    kStepsAll = 127u
};

static plora_status forward_impl(const plora_desc *desc, const void *x, const void *W, const void *const *A,
                                 const void *const *B, void *y, float *h_saved, void *workspace, size_t ws_bytes,
                                 void *hip_stream, bool lora_only = false, bool check_only = false, unsigned steps = kStepsAll)
{
    Call c;
    plora_status ps = prepare(desc, x, W, A, B, nullptr, nullptr, workspace, ws_bytes, lora_only, c);
    if (ps != PLORA_OK) return ps;
    const HostMeta &m = *c.m;
    const WorkspaceLayout &L = *c.L;
    if (!y && desc->T > 0) return PLORA_ERR_NULL;
    if (misaligned(y) || misaligned(h_saved)) return PLORA_ERR_ALIGN;
    if (desc->T == 0 || check_only) return PLORA_OK;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    char *ws = static_cast<char *>(workspace);

    const MetaView mv = device_view(m, L, ws);
    const bool lora = m.hdr.n_blocks > 0;
    const bool bf = desc->dtype == PLORA_BF16;
    const bool w_out_in = m.hdr.w_out_in != 0;
    if (steps & kStepPrep) {
        Bracket b(6, st);
        PL_TRY(launch_prep(c.words, m.n_words, m.hdr, ws + L.meta, reinterpret_cast<uint32_t *>(ws + L.desc), ws + L.zero,
                           ws + L.at, ws + L.ap, bf && lora, false, bf && lora && (w_out_in || lora_only), nullptr, nullptr, st));
    }
    float *hf = h_saved ? h_saved : reinterpret_cast<float *>(ws + L.hf);

    if (desc->dtype == PLORA_F32) {
        const float *xf = static_cast<const float *>(x);
        if (lora && (steps & kStepShrink)) { Bracket b(2, st); PL_TRY(launch_f32_lowrank(mv, m.hdr, 0, xf, desc->d_in, hf, st)); }
        if (!(steps & kStepMain)) return PLORA_OK;
        if (lora_only) {
            Bracket b(8, st);
            PL_TRY(launch_f32_expand(mv, m.hdr, true, static_cast<float *>(y), hf, st));
            return PLORA_OK;
        }
        { Bracket b(0, st);
          PL_TRY(launch_f32_gemm(mv, m.hdr, true, xf, static_cast<const float *>(W), hf, static_cast<float *>(y), false, st)); }
        return PLORA_OK;
    }

    void *at = ws + L.at, *hb = ws + L.hb;
    float *part = reinterpret_cast<float *>(ws + L.part);
    if (lora && (steps & kStepShrink)) {
        Bracket b(2, st);
        PL_TRY(launch_skinny_bf16(mv, m.hdr, 0, x, desc->d_in, at, ws + L.zero, part, h_saved, hb, nullptr, false, st));
    }
    if (!(steps & kStepMain)) return PLORA_OK;
    if (lora_only) {
        // the padded buffer holds B_k^T [d_out][rp]; the tables carry its offsets for d_in rows unless W's layout says d_out
        Bracket b(8, st);
        PL_TRY(launch_expand_bf16(mv, m.hdr, y, desc->d_out, hb, ws + L.ap, w_out_in ? desc->d_out : desc->d_in, ws + L.zero, st));
        return PLORA_OK;
    }
    { Bracket b(0, st);
      PL_TRY(launch_gemm_bf16(mv, m.hdr, !w_out_in, desc->d_in, desc->d_out, x, W, hb, ws + L.ap, ws + L.zero, y, false, st)); }
    return PLORA_OK;
}

static plora_status backward_impl(const plora_desc *desc, const void *x, const void *W, const void *const *A,
                                  const void *const *B, const void *dy, const float *h_saved, void *dx, float *const *dA,
                                  float *const *dB, void *workspace, size_t ws_bytes, void *hip_stream, bool lora_only = false,
                                  bool check_only = false, unsigned steps = kStepsAll, bool dx_accumulate = false)
{
    const bool want_w = (dA != nullptr) || (dB != nullptr);
    if (desc && want_w && desc->n_adapters > 0 && (!dA || !dB)) {
        plora_status v = validate(desc);
        return v != PLORA_OK ? v : PLORA_ERR_NULL;
    }
    Call c;
    plora_status ps = prepare(desc, x, W, A, B, want_w ? dA : nullptr, want_w ? dB : nullptr, workspace, ws_bytes, lora_only, c);
    if (ps != PLORA_OK) return ps;
    const HostMeta &m = *c.m;
    const WorkspaceLayout &L = *c.L;
    if (!dy && desc->T > 0) return PLORA_ERR_NULL;
    if (misaligned(dy) || misaligned(dx) || misaligned(h_saved)) return PLORA_ERR_ALIGN;
    if (want_w && desc->n_adapters > 0) {
        for (int32_t k = 0; k < desc->n_adapters; ++k) {
            if (!dA[k] || !dB[k]) return PLORA_ERR_NULL;
            if (misaligned(dA[k]) || misaligned(dB[k])) return PLORA_ERR_ALIGN;
        }
    }
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    char *ws = static_cast<char *>(workspace);
    const bool lora = m.hdr.n_blocks > 0;
    const bool any_w = want_w && desc->n_adapters > 0;
    if ((desc->T == 0 && !any_w) || check_only) return PLORA_OK;

    const MetaView mv = device_view(m, L, ws);
    if (steps & kStepPrep) {
        const bool bf = desc->dtype == PLORA_BF16;
        const bool need_shrink = any_w && !h_saved;
        const bool tr = bf && lora && any_w && h_saved;
        // the low-rank operand of the dX GEMM: padded A_k, or - W stored [d_out][d_in] - the packed A_k^T
        // (the stand-alone low-rank update always reads the padded A_k)
        const bool dx_ap = dx != nullptr && (lora_only || !m.hdr.w_out_in), dx_at = dx != nullptr && !lora_only && m.hdr.w_out_in;
        Bracket b(6, st);
        PL_TRY(launch_prep(c.words, m.n_words, m.hdr, ws + L.meta, reinterpret_cast<uint32_t *>(ws + L.desc), ws + L.zero,
                           ws + L.at, ws + L.ap, bf && lora && (need_shrink || dx_at), bf && lora && dx_ap, false,
                           tr ? h_saved : nullptr, tr ? ws + L.zt_h : nullptr, st));
    }

    if (desc->dtype == PLORA_F32) {
        const float *xf = static_cast<const float *>(x), *dyf = static_cast<const float *>(dy);
        float *gf = reinterpret_cast<float *>(ws + L.gf);
        const float *hf = h_saved;
        if (lora && any_w && !hf) {
            float *hw = reinterpret_cast<float *>(ws + L.hf);
            if (steps & kStepShrink) { Bracket b(2, st); PL_TRY(launch_f32_lowrank(mv, m.hdr, 0, xf, desc->d_in, hw, st)); }
            hf = hw;
        }
        if (lora && (steps & kStepDh)) { Bracket b(3, st); PL_TRY(launch_f32_lowrank(mv, m.hdr, 1, dyf, desc->d_out, gf, st)); }
        if (any_w) {
            if (steps & kStepDb) { Bracket b(4, st); PL_TRY(launch_f32_wgrad(mv, m.hdr, false, dyf, desc->d_out, hf, st)); }
            if (steps & kStepDa) { Bracket b(5, st); PL_TRY(launch_f32_wgrad(mv, m.hdr, true, xf, desc->d_in, gf, st)); }
        }
        if (!(steps & kStepDx)) return PLORA_OK;
        if (dx && desc->T > 0 && lora_only) {
            Bracket b(8, st);
            PL_TRY(launch_f32_expand(mv, m.hdr, false, static_cast<float *>(dx), gf, st));
        } else if (dx && desc->T > 0) {
            Bracket b(1, st);
            PL_TRY(launch_f32_gemm(mv, m.hdr, false, dyf, static_cast<const float *>(W), gf, static_cast<float *>(dx), dx_accumulate, st));
        }
        return PLORA_OK;
    }

    void *at = ws + L.at, *ap = ws + L.ap, *gb = ws + L.hb;
    void *zt_h = ws + L.zt_h, *zt_g = ws + L.zt_g;
    float *part = reinterpret_cast<float *>(ws + L.part);
    float *wpart = reinterpret_cast<float *>(ws + L.wpart);
    if (lora) {
        if (any_w && !h_saved && (steps & kStepShrink)) {
            Bracket b(2, st);
            PL_TRY(launch_skinny_bf16(mv, m.hdr, 0, x, desc->d_in, at, ws + L.zero, part, nullptr, nullptr, zt_h, false, st));
        }
        if (steps & kStepDh) {
            Bracket b(3, st);
            PL_TRY(launch_skinny_bf16(mv, m.hdr, 1, dy, desc->d_out, nullptr, ws + L.zero, part, nullptr, gb, any_w ? zt_g : nullptr, true, st));
        }
    }
    if (any_w) {
        if (steps & kStepDb) { Bracket b(4, st); PL_TRY(launch_tokcontract_bf16(mv, m.hdr, false, dy, desc->d_out, zt_h, ws + L.zero, wpart, m.split_dB, m.r16_total, m.n_active, st)); }
        if (steps & kStepDa) { Bracket b(5, st); PL_TRY(launch_tokcontract_bf16(mv, m.hdr, true, x, desc->d_in, zt_g, ws + L.zero, wpart, m.split_dA, m.r16_total, m.n_active, st)); }
    }
    if (!(steps & kStepDx)) return PLORA_OK;
    if (dx && desc->T > 0 && lora_only) {
        // padded A_k [d_in][rp]; the tables carry its offsets for d_in rows unless W's layout says d_out
        Bracket b(8, st);
        PL_TRY(launch_expand_bf16(mv, m.hdr, dx, desc->d_in, gb, ap, m.hdr.w_out_in ? desc->d_out : desc->d_in, ws + L.zero, st));
    } else if (dx && desc->T > 0) {
        Bracket b(1, st);
        PL_TRY(launch_gemm_bf16(mv, m.hdr, m.hdr.w_out_in != 0, desc->d_out, desc->d_in, dy, W, gb, ap, ws + L.zero, dx, dx_accumulate, st));
    }
    return PLORA_OK;
}

// ---- grouped calls: several projections on one x -------------------------------------------------------
// Each projection keeps a workspace of its own inside the group's (so every table and side buffer is where the plain
// call would put it); behind them lies the partial-tile region of the fused passes.  Projections are fused in cells:
// consecutive projections whose ranks, each padded to 16, sum to at most PLORA_MAX_RANK for every adapter.
struct GroupPlan {
    int n = 0;
    std::shared_ptr<const HostMeta> m[kMaxGroup];
    size_t ws_off[kMaxGroup] = {};
    int cell_of[kMaxGroup] = {};      // cell index of each projection
    int n_cells = 0;
    size_t part_off = 0, total = 0;
};

struct CellShape { int max_r16 = 0, r16_total = 0; };

// Fused ranks of the projections in `members` (indices into the plan).
static CellShape cell_shape(const GroupPlan &gp, const int *members, int n_members)
{
    CellShape c;
    const int n_ad = gp.m[0]->hdr.n_adapters;
    for (int k = 0; k < n_ad; ++k) {
        int sum = 0;
        for (int i = 0; i < n_members; ++i) sum += gp.m[members[i]]->t.ad[k].r16;
        c.max_r16 = std::max(c.max_r16, sum);
        c.r16_total += sum;
    }
    return c;
}

static size_t cell_part_bytes(const GroupPlan &gp, const plora_desc *d0, const CellShape &c)
{
    MetaHeader hv = gp.m[0]->hdr;
    hv.max_r16 = c.max_r16;
    const size_t shrink = (size_t)skinny_splits(hv, d0->d_in) * hv.n_blocks * kSkinnyRows * c.max_r16 * 4;
    const int sp = tokc_splits(hv, d0->d_in, gp.m[0]->n_active);
    const size_t da = sp > 1 ? (size_t)sp * c.r16_total * d0->d_in * 4 : 0;
    return std::max(shrink, da);
}

static plora_status plan_group(const plora_group *g, GroupPlan &gp)
{
    if (!g) return PLORA_ERR_NULL;
    if (g->n_proj < 1 || g->n_proj > PLORA_MAX_GROUP) return PLORA_ERR_GROUP;
    if (!g->desc) return PLORA_ERR_NULL;
    const plora_desc *d0 = &g->desc[0];
    for (int p = 0; p < g->n_proj; ++p) {
        const plora_desc *d = &g->desc[p];
        plora_status st = validate(d);
        if (st != PLORA_OK) return st;
        if (d->dtype != d0->dtype || d->T != d0->T || d->d_in != d0->d_in || d->n_seg != d0->n_seg || d->n_adapters != d0->n_adapters)
            return PLORA_ERR_GROUP;
        for (int32_t s = 0; s < d->n_seg; ++s)
            if (d->seg_off[s + 1] != d0->seg_off[s + 1] || d->seg_adapter[s] != d0->seg_adapter[s]) return PLORA_ERR_GROUP;
    }
    gp.n = g->n_proj;
    size_t o = 0;
    for (int p = 0; p < gp.n; ++p) {
        gp.m[p] = meta_of(&g->desc[p]);
        gp.ws_off[p] = o;
        o = align_up(o + gp.m[p]->ws.total, 256);
    }
    // cells (bf16 with adapters only: the fp32 path is not fused)
    const bool fuse = d0->dtype == PLORA_BF16 && gp.m[0]->hdr.n_blocks > 0;
    int members[kMaxGroup], nm = 0, cell = 0;
    size_t part = 0;
    for (int p = 0; p < gp.n; ++p) {
        members[nm] = p;
        if (nm > 0 && (!fuse || cell_shape(gp, members, nm + 1).max_r16 > PLORA_MAX_RANK)) {
            if (nm > 1) part = std::max(part, cell_part_bytes(gp, d0, cell_shape(gp, members, nm)));
            ++cell; members[0] = p; nm = 0;
        }
        gp.cell_of[p] = cell;
        ++nm;
    }
    if (nm > 1) part = std::max(part, cell_part_bytes(gp, d0, cell_shape(gp, members, nm)));
    gp.n_cells = cell + 1;
    gp.part_off = o;
    gp.total = align_up(o + part, 256) + 256;
    return PLORA_OK;
}

// The fused view of the projections `members` of the plan (all of one cell); small: which side buffer the pass gathers.
static void group_view(const GroupPlan &gp, char *ws, const int *members, int nm, bool small_is_at, GroupView &gv, MetaHeader &hv)
{
    const CellShape c = cell_shape(gp, members, nm);
    gv.n_proj = nm; gv.max_r16 = c.max_r16; gv.r16_total = c.r16_total; gv.reserved = 0;
    for (int i = 0; i < kMaxGroup; ++i) {
        const int p = members[i < nm ? i : 0];
        const HostMeta &m = *gp.m[p];
        char *w = ws + gp.ws_off[p];
        gv.mv[i] = device_view(m, m.ws, w);
        gv.small[i] = reinterpret_cast<const uint16_t *>(w + (small_is_at ? m.ws.at : m.ws.zt_g));
    }
    hv = gp.m[members[0]]->hdr;
    hv.max_r16 = c.max_r16;
}

static plora_status group_forward(const plora_group *g, const void *x, const void *const *W, const void *const *const *A,
                                  const void *const *const *B, void *const *y, float *const *h_saved, void *workspace,
                                  size_t ws_bytes, void *hip_stream)
{
    GroupPlan gp;
    plora_status ps = plan_group(g, gp);
    if (ps != PLORA_OK) return ps;
    if (!W || !y || (g->desc[0].n_adapters > 0 && (!A || !B))) return PLORA_ERR_NULL;
    if (!workspace || ws_bytes < gp.total) return PLORA_ERR_WORKSPACE;
    if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return PLORA_ERR_ALIGN;
    char *ws = static_cast<char *>(workspace);
    auto run = [&](int p, bool check, unsigned steps) {
        return forward_impl(&g->desc[p], x, W[p], A ? A[p] : nullptr, B ? B[p] : nullptr, y[p], h_saved ? h_saved[p] : nullptr,
                            ws + gp.ws_off[p], gp.m[p]->ws.total, hip_stream, false, check, steps);
    };
    for (int p = 0; p < gp.n; ++p)
        if ((ps = run(p, true, kStepsAll)) != PLORA_OK) return ps;
    if (g->desc[0].T == 0) return PLORA_OK;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    bool fused[kMaxGroup] = {};
    for (int p = 0; p < gp.n; ++p)
        for (int q = 0; q < gp.n; ++q) fused[p] = fused[p] || (q != p && gp.cell_of[q] == gp.cell_of[p]);
    for (int p = 0; p < gp.n; ++p)
        if ((ps = run(p, false, kStepPrep | (fused[p] ? 0u : kStepShrink))) != PLORA_OK) return ps;
    for (int c = 0; c < gp.n_cells; ++c) {
        int members[kMaxGroup], nm = 0;
        for (int p = 0; p < gp.n; ++p)
            if (gp.cell_of[p] == c && fused[p]) members[nm++] = p;
        if (nm < 2) continue;
        GroupView gv; MetaHeader hv;
        group_view(gp, ws, members, nm, true, gv, hv);
        float *hf[kMaxGroup] = {}; void *hb[kMaxGroup] = {}; void *zt[kMaxGroup] = {};
        for (int i = 0; i < nm; ++i) {
            hf[i] = h_saved ? h_saved[members[i]] : nullptr;
            hb[i] = ws + gp.ws_off[members[i]] + gp.m[members[i]]->ws.hb;
        }
        Bracket b(2, st);
        PL_TRY(launch_skinny_group(gv, hv, x, g->desc[0].d_in, ws + gp.ws_off[members[0]] + gp.m[members[0]]->ws.zero,
                                   reinterpret_cast<float *>(ws + gp.part_off), hf, hb, zt, st));
    }
    for (int p = 0; p < gp.n; ++p)
        if ((ps = run(p, false, kStepMain)) != PLORA_OK) return ps;
    return PLORA_OK;
}

static plora_status group_backward(const plora_group *g, const void *x, const void *const *W, const void *const *const *A,
                                   const void *const *const *B, const void *const *dy, const float *const *h_saved,
                                   void *const *dx, void *dx_sum, float *const *const *dA, float *const *const *dB,
                                   void *workspace, size_t ws_bytes, void *hip_stream)
{
    GroupPlan gp;
    plora_status ps = plan_group(g, gp);
    if (ps != PLORA_OK) return ps;
    if (!W || !dy || (g->desc[0].n_adapters > 0 && (!A || !B))) return PLORA_ERR_NULL;
    if (dx && dx_sum) return PLORA_ERR_GROUP;            // one or the other
    if (!workspace || ws_bytes < gp.total) return PLORA_ERR_WORKSPACE;
    if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return PLORA_ERR_ALIGN;
    char *ws = static_cast<char *>(workspace);
    // dx_sum: every projection's dX GEMM targets the one tensor, the first overwriting it, the others adding to it
    auto run = [&](int p, bool check, unsigned steps) {
        return backward_impl(&g->desc[p], x, W[p], A ? A[p] : nullptr, B ? B[p] : nullptr, dy[p], h_saved ? h_saved[p] : nullptr,
                             dx_sum ? dx_sum : (dx ? dx[p] : nullptr), dA ? dA[p] : nullptr, dB ? dB[p] : nullptr, ws + gp.ws_off[p],
                             gp.m[p]->ws.total, hip_stream, false, check, steps, dx_sum != nullptr && p > 0);
    };
    for (int p = 0; p < gp.n; ++p)
        if ((ps = run(p, true, kStepsAll)) != PLORA_OK) return ps;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const plora_desc *d0 = &g->desc[0];
    // which projections want weight gradients, and which of those have to recompute x A_k
    bool want_w[kMaxGroup] = {}, shrink[kMaxGroup] = {}, fuse_s[kMaxGroup] = {}, fuse_a[kMaxGroup] = {};
    for (int p = 0; p < gp.n; ++p) {
        want_w[p] = d0->n_adapters > 0 && ((dA && dA[p]) || (dB && dB[p]));
        shrink[p] = want_w[p] && !(h_saved && h_saved[p]);
    }
    for (int p = 0; p < gp.n; ++p)
        for (int q = 0; q < gp.n; ++q) {
            if (q == p || gp.cell_of[q] != gp.cell_of[p]) continue;
            fuse_s[p] = fuse_s[p] || (shrink[p] && shrink[q]);
            fuse_a[p] = fuse_a[p] || (want_w[p] && want_w[q]);
        }
    for (int p = 0; p < gp.n; ++p)
        if ((ps = run(p, false, kStepPrep | (fuse_s[p] ? 0u : kStepShrink))) != PLORA_OK) return ps;
    for (int c = 0; c < gp.n_cells; ++c) {
        int members[kMaxGroup], nm = 0;
        for (int p = 0; p < gp.n; ++p)
            if (gp.cell_of[p] == c && fuse_s[p]) members[nm++] = p;
        if (nm < 2) continue;
        GroupView gv; MetaHeader hv;
        group_view(gp, ws, members, nm, true, gv, hv);
        float *hf[kMaxGroup] = {}; void *hb[kMaxGroup] = {}; void *zt[kMaxGroup] = {};
        for (int i = 0; i < nm; ++i) zt[i] = ws + gp.ws_off[members[i]] + gp.m[members[i]]->ws.zt_h;
        Bracket b(2, st);
        PL_TRY(launch_skinny_group(gv, hv, x, d0->d_in, ws + gp.ws_off[members[0]] + gp.m[members[0]]->ws.zero,
                                   reinterpret_cast<float *>(ws + gp.part_off), hf, hb, zt, st));
    }
    for (int p = 0; p < gp.n; ++p)
        if ((ps = run(p, false, kStepDh | kStepDb | (fuse_a[p] ? 0u : kStepDa) | kStepDx)) != PLORA_OK) return ps;
    for (int c = 0; c < gp.n_cells; ++c) {
        int members[kMaxGroup], nm = 0;
        for (int p = 0; p < gp.n; ++p)
            if (gp.cell_of[p] == c && fuse_a[p]) members[nm++] = p;
        if (nm < 2) continue;
        GroupView gv; MetaHeader hv;
        group_view(gp, ws, members, nm, false, gv, hv);
        Bracket b(5, st);
        PL_TRY(launch_tokc_group_dA(gv, hv, x, d0->d_in, ws + gp.ws_off[members[0]] + gp.m[members[0]]->ws.zero,
                                    reinterpret_cast<float *>(ws + gp.part_off), tokc_splits(hv, d0->d_in, gp.m[0]->n_active),
                                    gp.m[0]->n_active, st));
    }
    return PLORA_OK;
}

// Scratch memory of plora_linear_fwd_noalloc: one array per GPU, resident from the first use of the
// library on that GPU until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress; kernels and copies get the device address looked up once per device.
__device__ __align__(256) unsigned char g_noalloc_scratch[PLORA_NOALLOC_SCRATCH_BYTES];

static plora_status noalloc_scratch(void **out)
{
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void *ptr[kMaxDevices] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return PLORA_ERR_HIP;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_noalloc_scratch)) != hipSuccess || !p) return PLORA_ERR_HIP;
        ptr[dev] = p;
    }
    *out = ptr[dev];
    return PLORA_OK;
}

}  // namespace plora

using namespace plora;

// No exception leaves the library: host allocation failures and anything else thrown on the way become a status.
#define PL_GUARDED(fallback, ...) \
    try { __VA_ARGS__ } catch (const std::bad_alloc &) { return fallback; } catch (...) { return fallback; }

extern "C" {

const char *plora_status_string(plora_status st)
{
    switch (st) {
    case PLORA_OK: return "ok";
    case PLORA_ERR_NULL: return "a required pointer is NULL";
    case PLORA_ERR_SHAPE: return "bad T / d_in / d_out (bf16 needs multiples of 8; sizes above the supported range)";
    case PLORA_ERR_SEGMENTS: return "segment offsets must start at 0, end at T and not decrease";
    case PLORA_ERR_ADAPTER: return "adapter id out of range or too many adapters";
    case PLORA_ERR_RANK: return "rank outside [1, PLORA_MAX_RANK]";
    case PLORA_ERR_ALIGN: return "device pointer not 16-byte aligned (workspace: 256)";
    case PLORA_ERR_WORKSPACE: return "workspace missing or too small";
    case PLORA_ERR_UNSUPPORTED: return "unsupported dtype";
    case PLORA_ERR_HIP: return "HIP launch failed";
    case PLORA_ERR_INTERNAL: return "host memory allocation failed or internal error";
    case PLORA_ERR_GROUP: return "grouped call: bad number of projections, or they differ in dtype, T, d_in, segments or adapters";
    }
    return "unknown status";
}

plora_status plora_validate(const plora_desc *desc) { return validate(desc); }

size_t plora_h_elems(const plora_desc *desc)
{
    PL_GUARDED(0,
        if (validate(desc) != PLORA_OK) return 0;
        return meta_of(desc)->h_elems;
    )
}

size_t plora_workspace_bytes(const plora_desc *desc)
{
    PL_GUARDED(0,
        if (validate(desc) != PLORA_OK) return 0;
        return meta_of(desc)->ws.total;
    )
}

int64_t plora_build_metadata(const plora_desc *desc, int32_t block_rows, int64_t *h_off_out,
                             int32_t *blocks_out, int64_t blocks_cap)
{
    PL_GUARDED(-1,
        if (validate(desc) != PLORA_OK || block_rows < 1) return -1;
        const std::shared_ptr<const HostMeta> m = meta_of(desc);
        if (h_off_out) {
            for (int32_t s = 0; s < desc->n_seg; ++s) h_off_out[s] = m->t.seg[s].h_off;
            h_off_out[desc->n_seg] = (int64_t)m->h_elems;
        }
        int64_t n = 0;
        for (int32_t s = 0; s < desc->n_seg; ++s) {
            const SegInfo &g = m->t.seg[s];
            for (int32_t r0 = g.row0; r0 < g.row1; r0 += block_rows) {
                if (blocks_out && n < blocks_cap) {
                    blocks_out[4 * n + 0] = r0;
                    blocks_out[4 * n + 1] = (g.row1 - r0 < block_rows) ? g.row1 - r0 : block_rows;
                    blocks_out[4 * n + 2] = s;
                    blocks_out[4 * n + 3] = g.adapter;
                }
                ++n;
            }
        }
        return n;
    )
}

int plora_debug_metadata(const plora_desc *desc, plora_debug_info *info, void *tables_out, size_t cap)
{
    PL_GUARDED(-1,
        if (validate(desc) != PLORA_OK || !info) return -1;
        HostMeta m;                      // built afresh: the export must not depend on what the cache holds
        build_meta(desc, m);
        std::memset(info, 0, sizeof(*info));
        info->n_tiles = m.layout.n_tiles;
        info->n_seg = m.hdr.n_seg; info->n_adapters = m.hdr.n_adapters;
        info->n_blocks = m.hdr.n_blocks; info->max_r16 = m.hdr.max_r16;
        info->seg_stride = (int32_t)sizeof(SegInfo); info->ad_stride = (int32_t)sizeof(AdapterInfo);
        info->tile_stride = (int32_t)sizeof(GemmTile);
        info->off_hdr = m.layout.hdr; info->off_seg = m.layout.seg; info->off_ad = m.layout.ad;
        info->off_tile = m.layout.tile; info->off_blk_seg = m.layout.blk_seg; info->off_seg_list = m.layout.seg_list;
        info->off_tile_order = m.layout.tile_order;
        info->table_bytes = m.layout.bytes;
        info->shrink_splits = m.split_shrink; info->dh_splits = m.split_dh;
        info->da_splits = m.split_dA; info->da_tile_cols = m.bc_dA;
        info->db_splits = m.split_dB; info->db_tile_cols = m.bc_dB;
        info->r16_total = m.r16_total; info->n_active = m.n_active;
        info->ws_zero = m.ws.zero; info->ws_meta = m.ws.meta; info->ws_desc = m.ws.desc; info->ws_at = m.ws.at;
        info->ws_ap = m.ws.ap; info->ws_hb = m.ws.hb; info->ws_zt_h = m.ws.zt_h; info->ws_zt_g = m.ws.zt_g;
        info->ws_hf = m.ws.hf; info->ws_gf = m.ws.gf; info->ws_part = m.ws.part; info->ws_wpart = m.ws.wpart;
        info->ws_total = m.ws.total;
        info->h_elems = m.h_elems;
        info->desc_words = m.n_words;
        if (tables_out) {
            if (cap < m.layout.bytes) return -1;
            std::memcpy(tables_out, m.image.data(), m.layout.bytes);
        }
        return 0;
    )
}

void plora_set_kernel_timing(int enabled)
{
    g_timing = enabled;
    g_pair_class.clear();
}

int plora_kernel_time(int cls, float *total_ms, int *count)
{
    if (cls < 0 || cls >= kClasses || !total_ms || !count) return -1;
    float tot = 0.f; int n = 0;
    for (size_t p = 0; p < g_pair_class.size(); ++p) {
        if (g_pair_class[p] != cls) continue;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, g_pool[2 * p], g_pool[2 * p + 1]) != hipSuccess) return -1;
        tot += ms; ++n;
    }
    *total_ms = tot; *count = n;
    return 0;
}

plora_status plora_linear_fwd(const plora_desc *desc, const void *x, const void *W,
                              const void *const *A, const void *const *B, void *y, float *h_saved,
                              void *workspace, size_t ws_bytes, void *hip_stream)
{
    PL_GUARDED(PLORA_ERR_INTERNAL,
        return forward_impl(desc, x, W, A, B, y, h_saved, workspace, ws_bytes, hip_stream);
    )
}

plora_status plora_linear_fwd_noalloc(const plora_desc *desc, const void *x, const void *W,
                                      const void *const *A, const void *const *B, void *y, float *h_saved,
                                      void *hip_stream)
{
    PL_GUARDED(PLORA_ERR_INTERNAL,
        const plora_status v = validate(desc);
        if (v != PLORA_OK) return v;
        if (meta_of(desc)->ws.total > (size_t)PLORA_NOALLOC_SCRATCH_BYTES) return PLORA_ERR_WORKSPACE;
        void *scratch = nullptr;
        const plora_status ps = noalloc_scratch(&scratch);
        if (ps != PLORA_OK) return ps;
        return forward_impl(desc, x, W, A, B, y, h_saved, scratch, PLORA_NOALLOC_SCRATCH_BYTES, hip_stream);
    )
}

static plora_status adamw_collect(const plora_desc *d, const plora_adamw_side *s, bool is_A, const plora_adamw_hparams *hp,
                                  std::vector<AdamwTensor> &out)
{
    if (!s || !s->grad || !s->m || !s->v) return PLORA_ERR_NULL;
    if (!s->param && !s->master) return PLORA_ERR_NULL;
    if (!s->master && d->dtype != PLORA_F32) return PLORA_ERR_NULL;
    for (int32_t k = 0; k < d->n_adapters; ++k) {
        AdamwTensor t;
        t.param = s->param ? s->param[k] : nullptr;
        t.master = s->master ? s->master[k] : nullptr;
        t.grad = s->grad[k]; t.m = s->m[k]; t.v = s->v[k];
        if (!t.grad || !t.m || !t.v || (s->param && !t.param) || (s->master && !t.master)) return PLORA_ERR_NULL;
        if (misaligned(t.param) || misaligned(t.master) || misaligned(t.grad) || misaligned(t.m) || misaligned(t.v))
            return PLORA_ERR_ALIGN;
        t.numel = (uint64_t)d->rank[k] * (uint64_t)(is_A ? d->d_in : d->d_out);
        t.lr = hp[k].lr; t.beta1 = hp[k].beta1; t.beta2 = hp[k].beta2; t.eps = hp[k].eps;
        t.weight_decay = hp[k].weight_decay; t.step = hp[k].step; t.grad_scale = hp[k].grad_scale;
        out.push_back(t);
    }
    return PLORA_OK;
}

plora_status plora_adamw_step(const plora_desc *desc, const plora_adamw_side *A, const plora_adamw_side *B,
                              const plora_adamw_hparams *hp, void *hip_stream)
{
    PL_GUARDED(PLORA_ERR_INTERNAL,
        const plora_status v = validate(desc);
        if (v != PLORA_OK) return v;
        if (desc->n_adapters == 0) return PLORA_OK;
        if (!hp) return PLORA_ERR_NULL;
        for (int32_t k = 0; k < desc->n_adapters; ++k)
            if (hp[k].step < 1 || !(hp[k].beta1 >= 0.f && hp[k].beta1 < 1.f) || !(hp[k].beta2 >= 0.f && hp[k].beta2 < 1.f) ||
                !std::isfinite(hp[k].grad_scale))
                return PLORA_ERR_SHAPE;
        std::vector<AdamwTensor> jobs;
        jobs.reserve(2 * (size_t)desc->n_adapters);
        plora_status ps = adamw_collect(desc, A, true, hp, jobs);
        if (ps != PLORA_OK) return ps;
        ps = adamw_collect(desc, B, false, hp, jobs);
        if (ps != PLORA_OK) return ps;
        { Bracket b(7, static_cast<hipStream_t>(hip_stream));
          PL_TRY(launch_adamw(jobs.data(), (int)jobs.size(), desc->dtype == PLORA_BF16, static_cast<hipStream_t>(hip_stream))); }
        return PLORA_OK;
    )
}

plora_status plora_linear_bwd(const plora_desc *desc, const void *x, const void *W,
                              const void *const *A, const void *const *B, const void *dy,
                              const float *h_saved, void *dx, float *const *dA, float *const *dB,
                              void *workspace, size_t ws_bytes, void *hip_stream)
{
    PL_GUARDED(PLORA_ERR_INTERNAL,
        return backward_impl(desc, x, W, A, B, dy, h_saved, dx, dA, dB, workspace, ws_bytes, hip_stream);
    )
}

// Workspace of the NF4 calls: the ordinary workspace, then the expanded weight.
static size_t nf4_weight_offset(const HostMeta &m) { return align_up(m.ws.total, 256); }
static size_t nf4_weight_bytes(const plora_desc *d) { return (size_t)d->d_in * (size_t)d->d_out * (d->dtype == PLORA_BF16 ? 2 : 4); }

size_t plora_nf4_workspace_bytes(const plora_desc *desc)
{
    PL_GUARDED(0,
        if (validate(desc) != PLORA_OK || (desc->d_in * desc->d_out) % 64 != 0) return 0;
        return nf4_weight_offset(*meta_of(desc)) + nf4_weight_bytes(desc);
    )
}

plora_status plora_nf4_dequantize(const void *W_codes, const float *W_absmax, int64_t n_elems, int32_t dtype, void *out,
                                  void *hip_stream)
{
    PL_GUARDED(PLORA_ERR_INTERNAL,
        if (dtype != PLORA_BF16 && dtype != PLORA_F32) return PLORA_ERR_UNSUPPORTED;
        if (n_elems < 0 || n_elems % 64 != 0) return PLORA_ERR_SHAPE;
        if (n_elems == 0) return PLORA_OK;
        if (!W_codes || !W_absmax || !out) return PLORA_ERR_NULL;
        if (misaligned(W_codes) || misaligned(W_absmax) || misaligned(out)) return PLORA_ERR_ALIGN;
        hipStream_t st = static_cast<hipStream_t>(hip_stream);
        Bracket b(9, st);
        PL_TRY(launch_nf4_dequant(W_codes, W_absmax, n_elems, dtype == PLORA_BF16, out, st));
        return PLORA_OK;
    )
}

// Checks of the NF4 calls that come before anything is enqueued; *w_out = where the expanded weight goes.
static plora_status nf4_prepare(const plora_desc *desc, const void *codes, const float *absmax, void *workspace,
                                size_t ws_bytes, void **w_out, size_t *inner_bytes)
{
    const plora_status v = validate(desc);
    if (v != PLORA_OK) return v;
    if ((desc->d_in * desc->d_out) % 64 != 0) return PLORA_ERR_SHAPE;
    if (!codes || !absmax) return PLORA_ERR_NULL;
    if (misaligned(codes) || misaligned(absmax)) return PLORA_ERR_ALIGN;
    const size_t off = nf4_weight_offset(*meta_of(desc));
    if (!workspace || ws_bytes < off + nf4_weight_bytes(desc)) return PLORA_ERR_WORKSPACE;
    if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return PLORA_ERR_ALIGN;
    *w_out = static_cast<char *>(workspace) + off;
    *inner_bytes = off;
    return PLORA_OK;
}

plora_status plora_linear_fwd_nf4(const plora_desc *desc, const void *x, const void *W_codes, const float *W_absmax,
                                  const void *const *A, const void *const *B, void *y, float *h_saved, void *workspace,
                                  size_t ws_bytes, void *hip_stream)
{
    PL_GUARDED(PLORA_ERR_INTERNAL,
        void *W = nullptr;
        size_t inner = 0;
        plora_status ps = nf4_prepare(desc, W_codes, W_absmax, workspace, ws_bytes, &W, &inner);
        if (ps != PLORA_OK) return ps;
        // every other argument is checked before the weight is expanded, so that an error enqueues nothing
        ps = forward_impl(desc, x, W, A, B, y, h_saved, workspace, inner, hip_stream, false, true);
        if (ps != PLORA_OK) return ps;
        if (desc->T > 0) {
            ps = plora_nf4_dequantize(W_codes, W_absmax, desc->d_in * desc->d_out, desc->dtype, W, hip_stream);
            if (ps != PLORA_OK) return ps;
        }
        return forward_impl(desc, x, W, A, B, y, h_saved, workspace, inner, hip_stream);
    )
}

plora_status plora_linear_bwd_nf4(const plora_desc *desc, const void *x, const void *W_codes, const float *W_absmax,
                                  const void *const *A, const void *const *B, const void *dy, const float *h_saved, void *dx,
                                  float *const *dA, float *const *dB, void *workspace, size_t ws_bytes, void *hip_stream)
{
    PL_GUARDED(PLORA_ERR_INTERNAL,
        void *W = nullptr;
        size_t inner = 0;
        plora_status ps = nf4_prepare(desc, W_codes, W_absmax, workspace, ws_bytes, &W, &inner);
        if (ps != PLORA_OK) return ps;
        ps = backward_impl(desc, x, W, A, B, dy, h_saved, dx, dA, dB, workspace, inner, hip_stream, false, true);
        if (ps != PLORA_OK) return ps;
        if (dx && desc->T > 0) {
            ps = plora_nf4_dequantize(W_codes, W_absmax, desc->d_in * desc->d_out, desc->dtype, W, hip_stream);
            if (ps != PLORA_OK) return ps;
        }
        return backward_impl(desc, x, W, A, B, dy, h_saved, dx, dA, dB, workspace, inner, hip_stream);
    )
}

size_t plora_lora_workspace_bytes(const plora_desc *desc)
{
    PL_GUARDED(0,
        if (validate(desc) != PLORA_OK) return 0;
        return meta_of(desc)->ws_lora.total;
    )
}

plora_status plora_lora_fwd(const plora_desc *desc, const void *x, const void *const *A, const void *const *B, void *y,
                            float *h_saved, void *workspace, size_t ws_bytes, void *hip_stream)
{
    PL_GUARDED(PLORA_ERR_INTERNAL,
        return forward_impl(desc, x, nullptr, A, B, y, h_saved, workspace, ws_bytes, hip_stream, true);
    )
}

plora_status plora_lora_bwd(const plora_desc *desc, const void *x, const void *const *A, const void *const *B,
                            const void *dy, const float *h_saved, void *dx, float *const *dA, float *const *dB,
                            void *workspace, size_t ws_bytes, void *hip_stream)
{
    PL_GUARDED(PLORA_ERR_INTERNAL,
        return backward_impl(desc, x, nullptr, A, B, dy, h_saved, dx, dA, dB, workspace, ws_bytes, hip_stream, true);
    )
}

size_t plora_group_workspace_bytes(const plora_group *group)
{
    PL_GUARDED(0,
        GroupPlan gp;
        if (plan_group(group, gp) != PLORA_OK) return 0;
        return gp.total;
    )
}

plora_status plora_group_fwd(const plora_group *group, const void *x, const void *const *W, const void *const *const *A,
                             const void *const *const *B, void *const *y, float *const *h_saved, void *workspace,
                             size_t ws_bytes, void *hip_stream)
{
    PL_GUARDED(PLORA_ERR_INTERNAL,
        return group_forward(group, x, W, A, B, y, h_saved, workspace, ws_bytes, hip_stream);
    )
}

plora_status plora_group_bwd(const plora_group *group, const void *x, const void *const *W, const void *const *const *A,
                             const void *const *const *B, const void *const *dy, const float *const *h_saved,
                             void *const *dx, void *dx_sum, float *const *const *dA, float *const *const *dB,
                             void *workspace, size_t ws_bytes, void *hip_stream)
{
    PL_GUARDED(PLORA_ERR_INTERNAL,
        return group_backward(group, x, W, A, B, dy, h_saved, dx, dx_sum, dA, dB, workspace, ws_bytes, hip_stream);
    )
}

}  // extern "C"
