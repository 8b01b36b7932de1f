// Host side of libplora: argument validation, the segment-packing metadata builder, workspace
// layout and the launch sequences of the forward and backward calls.  No arithmetic of the layer
// happens here; every step runs in the HIP kernels.
#include "plora_internal.h"

#include <cstring>
#include <algorithm>
#include <mutex>
#include <vector>

namespace plora {

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static inline int32_t pad_to(int32_t v, int32_t a) { return (v + a - 1) / a * a; }

static plora_status validate(const plora_desc *d)
{
    if (!d) return PLORA_ERR_NULL;
    if (d->dtype != PLORA_BF16 && d->dtype != PLORA_F32) return PLORA_ERR_UNSUPPORTED;
    if (d->T < 0 || d->d_in <= 0 || d->d_out <= 0) return PLORA_ERR_SHAPE;
    if (d->T > INT32_MAX || d->d_in > (1 << 24) || d->d_out > (1 << 24)) return PLORA_ERR_SHAPE;
    if (d->dtype == PLORA_BF16 && (d->d_in % 8 != 0 || d->d_out % 8 != 0)) return PLORA_ERR_SHAPE;
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

// Host copy of the metadata blob plus the workspace layout derived from it.
struct HostMeta {
    MetaHeader hdr;
    std::vector<SegInfo> seg;
    std::vector<AdapterInfo> ad;
    std::vector<TileExt> tile_ext;
    std::vector<int32_t> blk_seg, seg_list;
    WorkspaceLayout ws;
    size_t h_elems = 0, hb_elems = 0, zt_elems = 0, at_elems = 0, ap_elems = 0;
    int r16_total = 0, n_active = 0, split_dA = 1, split_dB = 1;
};

// The segment-packing metadata builder (host).  Pure integer work.
static void build_meta(const plora_desc *d, HostMeta &m)
{
    m.hdr.T = d->T; m.hdr.D = d->d_in; m.hdr.K = d->d_out;
    m.hdr.n_seg = d->n_seg; m.hdr.n_adapters = d->n_adapters; m.hdr.max_r16 = 0;
    m.seg.resize(d->n_seg);
    m.ad.resize(d->n_adapters);
    int64_t at = 0, ap = 0;
    int32_t r16_off = 0;
    for (int32_t k = 0; k < d->n_adapters; ++k) {
        AdapterInfo &a = m.ad[k];
        std::memset(&a, 0, sizeof(a));
        a.r = d->rank[k];
        a.rp = pad_to(a.r, kRankPadGemm);
        a.r16 = pad_to(a.r, kRankPadMfma);
        a.scale = d->scale[k];
        a.at_off = at; at += (int64_t)a.r16 * d->d_in;
        a.ap_off = ap; ap += (int64_t)a.rp * d->d_in;
        a.r16_off = r16_off; r16_off += a.r16;
    }
    int64_t h = 0, hb = 0, zt = 0;
    int32_t blk = 0;
    for (int32_t s = 0; s < d->n_seg; ++s) {
        SegInfo &g = m.seg[s];
        g.row0 = d->seg_off[s]; g.row1 = d->seg_off[s + 1];
        g.adapter = d->seg_adapter[s];
        const int32_t len = g.row1 - g.row0;
        g.r = g.adapter >= 0 ? m.ad[g.adapter].r : 0;
        g.rp = g.adapter >= 0 ? m.ad[g.adapter].rp : 0;
        g.r16 = g.adapter >= 0 ? m.ad[g.adapter].r16 : 0;
        g.lp = pad_to(len, kTokPad);
        g.blk0 = blk;
        g.h_off = h; g.hb_off = hb; g.zt_off = zt;
        if (g.adapter >= 0) {
            blk += (len + kSkinnyRows - 1) / kSkinnyRows;
            if (len > 0 && g.r16 > m.hdr.max_r16) m.hdr.max_r16 = g.r16;
            h += (int64_t)len * g.r;
            hb += (int64_t)len * g.rp;
            zt += (int64_t)g.r16 * g.lp;
        }
    }
    m.hdr.n_blocks = blk;
    m.r16_total = r16_off;
    m.blk_seg.assign(blk, 0);
    for (int32_t s = 0; s < d->n_seg; ++s) {
        const SegInfo &g = m.seg[s];
        if (g.adapter < 0) continue;
        const int32_t nb = (g.row1 - g.row0 + kSkinnyRows - 1) / kSkinnyRows;
        for (int32_t b = 0; b < nb; ++b) m.blk_seg[g.blk0 + b] = s;
    }
    m.seg_list.clear();
    for (int32_t k = 0; k < d->n_adapters; ++k) {
        m.ad[k].seg_list0 = (int32_t)m.seg_list.size();
        for (int32_t s = 0; s < d->n_seg; ++s)
            if (m.seg[s].adapter == k && m.seg[s].row1 > m.seg[s].row0) m.seg_list.push_back(s);
        m.ad[k].n_own = (int32_t)m.seg_list.size() - m.ad[k].seg_list0;
    }
    {
        const int64_t tiles = (d->T + kGemmTileRows - 1) / kGemmTileRows;
        m.tile_ext.assign((size_t)tiles, TileExt{d->n_seg, 0});
        for (int32_t s = 0; s < d->n_seg; ++s) {
            const SegInfo &g = m.seg[s];
            if (g.adapter < 0 || g.row1 <= g.row0) continue;
            for (int64_t t = g.row0 / kGemmTileRows; t <= (g.row1 - 1) / kGemmTileRows; ++t) {
                if (m.tile_ext[t].first_seg == d->n_seg) m.tile_ext[t].first_seg = s;
                m.tile_ext[t].n_ext += g.rp / kRankPadGemm;
            }
        }
    }
    {
        std::vector<char> seen(d->n_adapters, 0);
        for (int32_t s = 0; s < d->n_seg; ++s)
            if (m.seg[s].adapter >= 0 && m.seg[s].row1 > m.seg[s].row0) seen[m.seg[s].adapter] = 1;
        m.n_active = 0;
        for (char c : seen) m.n_active += c;
    }
    {
        // the weight-gradient kernels hand out adapters longest first, so the last workgroups are short
        std::vector<int64_t> tokens(d->n_adapters, 0);
        for (int32_t s = 0; s < d->n_seg; ++s)
            if (m.seg[s].adapter >= 0) tokens[m.seg[s].adapter] += m.seg[s].row1 - m.seg[s].row0;
        std::vector<int32_t> order(d->n_adapters);
        for (int32_t k = 0; k < d->n_adapters; ++k) order[k] = k;
        std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return tokens[a] > tokens[b]; });
        for (int32_t k = 0; k < d->n_adapters; ++k) m.ad[k].by_tokens = order[k];
    }
    m.split_dA = tokc_splits(m.hdr, d->d_in, m.n_active);
    m.split_dB = tokc_splits(m.hdr, d->d_out, m.n_active);
    m.h_elems = (size_t)h; m.hb_elems = (size_t)hb; m.zt_elems = (size_t)zt;
    m.at_elems = (size_t)at; m.ap_elems = (size_t)ap;

    WorkspaceLayout &w = m.ws;
    size_t o = 0;
    w.zero = o; o += kZeroBytes;
    w.meta_bytes = sizeof(MetaHeader) + m.seg.size() * sizeof(SegInfo) + m.ad.size() * sizeof(AdapterInfo) +
                   m.tile_ext.size() * sizeof(TileExt) + (m.blk_seg.size() + m.seg_list.size()) * sizeof(int32_t);
    w.meta = o; o = align_up(o + w.meta_bytes, 256);
    const bool bf = d->dtype == PLORA_BF16;
    w.at = o;   o = align_up(o + (bf ? m.at_elems * 2 : 0), 256);
    w.ap = o;   o = align_up(o + (bf ? m.ap_elems * 2 : 0), 256);
    w.hb = o;   o = align_up(o + (bf ? m.hb_elems * 2 : 0), 256);
    w.zt_h = o; o = align_up(o + (bf ? m.zt_elems * 2 : 0), 256);
    w.zt_g = o; o = align_up(o + (bf ? m.zt_elems * 2 : 0), 256);
    w.hf = o;   o = align_up(o + m.h_elems * 4, 256);
    w.gf = o;   o = align_up(o + (bf ? 0 : m.h_elems * 4), 256);
    w.part = o; o = align_up(o + (bf ? (size_t)kSkinnyMaxSplits * blk * kSkinnyRows * m.hdr.max_r16 * 4 : 0), 256);
    {
        const size_t a_bytes = m.split_dA > 1 ? (size_t)m.split_dA * m.r16_total * d->d_in * 4 : 0;
        const size_t b_bytes = m.split_dB > 1 ? (size_t)m.split_dB * m.r16_total * d->d_out * 4 : 0;
        w.wpart = o; o = align_up(o + (bf ? (a_bytes > b_bytes ? a_bytes : b_bytes) : 0), 256);
    }
    w.total = o + 256;
}

// ---- bench-only kernel timing ------------------------------------------------------------------
// Every kernel class of a call is bracketed by a pair of HIP events recorded on the call's own
// stream; pairs come from a pool that is filled while timing is enabled and summed on request.
constexpr int kClasses = 8;
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

// Checks shared by forward and backward; fills the adapter pointer fields.
static plora_status prepare(const plora_desc *d, const void *x, const void *W, const void *const *A,
                            const void *const *B, void *workspace, size_t ws_bytes, HostMeta &m)
{
    plora_status st = validate(d);
    if (st != PLORA_OK) return st;
    if (!x && d->T > 0) return PLORA_ERR_NULL;
    if (!W) return PLORA_ERR_NULL;
    if (d->n_adapters > 0 && (!A || !B)) return PLORA_ERR_NULL;
    for (int32_t k = 0; k < d->n_adapters; ++k) {
        if (!A[k] || !B[k]) return PLORA_ERR_NULL;
        if (misaligned(A[k]) || misaligned(B[k])) return PLORA_ERR_ALIGN;
    }
    if (misaligned(x) || misaligned(W)) return PLORA_ERR_ALIGN;
    build_meta(d, m);
    if (!workspace || ws_bytes < m.ws.total) return PLORA_ERR_WORKSPACE;
    if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return PLORA_ERR_ALIGN;
    for (int32_t k = 0; k < d->n_adapters; ++k) { m.ad[k].A = A[k]; m.ad[k].B = B[k]; }
    return PLORA_OK;
}

static void build_blob(const HostMeta &m, char *ws, std::vector<char> &blob, MetaView &mv)
{
    blob.resize(m.ws.meta_bytes);
    char *p = blob.data();
    std::memcpy(p, &m.hdr, sizeof(MetaHeader)); p += sizeof(MetaHeader);
    if (!m.seg.empty()) std::memcpy(p, m.seg.data(), m.seg.size() * sizeof(SegInfo));
    p += m.seg.size() * sizeof(SegInfo);
    if (!m.ad.empty()) std::memcpy(p, m.ad.data(), m.ad.size() * sizeof(AdapterInfo));
    p += m.ad.size() * sizeof(AdapterInfo);
    if (!m.tile_ext.empty()) std::memcpy(p, m.tile_ext.data(), m.tile_ext.size() * sizeof(TileExt));
    p += m.tile_ext.size() * sizeof(TileExt);
    if (!m.blk_seg.empty()) std::memcpy(p, m.blk_seg.data(), m.blk_seg.size() * sizeof(int32_t));
    p += m.blk_seg.size() * sizeof(int32_t);
    if (!m.seg_list.empty()) std::memcpy(p, m.seg_list.data(), m.seg_list.size() * sizeof(int32_t));
    char *dev = ws + m.ws.meta;
    size_t off = 0;
    mv.hdr = reinterpret_cast<const MetaHeader *>(dev); off += sizeof(MetaHeader);
    mv.seg = reinterpret_cast<const SegInfo *>(dev + off); off += m.seg.size() * sizeof(SegInfo);
    mv.ad = reinterpret_cast<const AdapterInfo *>(dev + off); off += m.ad.size() * sizeof(AdapterInfo);
    mv.tile_ext = reinterpret_cast<const TileExt *>(dev + off); off += m.tile_ext.size() * sizeof(TileExt);
    mv.blk_seg = reinterpret_cast<const int32_t *>(dev + off); off += m.blk_seg.size() * sizeof(int32_t);
    mv.seg_list = reinterpret_cast<const int32_t *>(dev + off);
}

// The small jobs in front of the heavy kernels: metadata blob and zero page into the workspace,
// packing of A_k (bf16 path), transposed bf16 copy of a saved activation (bf16 backward).  One
// launch when the blob fits a kernel argument, separate launches otherwise.
static hipError_t prepare_device(const HostMeta &m, char *ws, hipStream_t st, MetaView &mv, void *at, void *ap,
                                 bool want_at, bool want_ap, const float *hf, void *zt)
{
    std::vector<char> blob;
    build_blob(m, ws, blob, mv);
    const bool pack = m.hdr.n_adapters > 0 && (want_at || want_ap);
    const bool tr = hf && zt && m.hdr.n_blocks > 0;
    if (prep_fits(blob.size())) {
        Bracket b(6, st);
        return launch_prep(m.hdr, ws + m.ws.meta, blob.data(), blob.size(), ws + m.ws.zero, at, ap, pack && want_at,
                           pack && want_ap, tr ? hf : nullptr, tr ? zt : nullptr, st);
    }
    hipError_t e = clear_zero_page(ws + m.ws.zero, st);
    if (e != hipSuccess) return e;
    e = upload_blob(ws + m.ws.meta, blob.data(), blob.size(), st);
    if (e != hipSuccess) return e;
    if (pack) {
        Bracket b(6, st);
        e = launch_pack_bf16(mv, m.hdr, at, ap, want_at, want_ap, st);
        if (e != hipSuccess) return e;
    }
    if (tr) {
        Bracket b(7, st);
        e = launch_h_to_zt(mv, m.hdr, hf, zt, st);
    }
    return e;
}

}  // namespace plora

using namespace plora;

extern "C" {

const char *plora_status_string(plora_status st)
{
    switch (st) {
    case PLORA_OK: return "ok";
    case PLORA_ERR_NULL: return "a required pointer is NULL";
    case PLORA_ERR_SHAPE: return "bad T / d_in / d_out (bf16 needs multiples of 8)";
    case PLORA_ERR_SEGMENTS: return "segment offsets must start at 0, end at T and not decrease";
    case PLORA_ERR_ADAPTER: return "adapter id out of range or too many adapters";
    case PLORA_ERR_RANK: return "rank outside [1, PLORA_MAX_RANK]";
    case PLORA_ERR_ALIGN: return "device pointer not 16-byte aligned (workspace: 256)";
    case PLORA_ERR_WORKSPACE: return "workspace missing or too small";
    case PLORA_ERR_UNSUPPORTED: return "unsupported dtype";
    case PLORA_ERR_HIP: return "HIP launch failed";
    }
    return "unknown status";
}

plora_status plora_validate(const plora_desc *desc) { return validate(desc); }

size_t plora_h_elems(const plora_desc *desc)
{
    if (validate(desc) != PLORA_OK) return 0;
    HostMeta m; build_meta(desc, m);
    return m.h_elems;
}

size_t plora_workspace_bytes(const plora_desc *desc)
{
    if (validate(desc) != PLORA_OK) return 0;
    HostMeta m; build_meta(desc, m);
    return m.ws.total;
}

int64_t plora_build_metadata(const plora_desc *desc, int32_t block_rows, int64_t *h_off_out,
                             int32_t *blocks_out, int64_t blocks_cap)
{
    if (validate(desc) != PLORA_OK || block_rows < 1) return -1;
    HostMeta m; build_meta(desc, m);
    if (h_off_out) {
        for (int32_t s = 0; s < desc->n_seg; ++s) h_off_out[s] = m.seg[s].h_off;
        h_off_out[desc->n_seg] = (int64_t)m.h_elems;
    }
    int64_t n = 0;
    for (int32_t s = 0; s < desc->n_seg; ++s) {
        const SegInfo &g = m.seg[s];
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

plora_status plora_linear_fwd_noalloc(const plora_desc *desc, const void *x, const void *W,
                                      const void *const *A, const void *const *B, void *y, float *h_saved,
                                      void *hip_stream)
{
    const size_t need = plora_workspace_bytes(desc);
    if (need == 0) return validate(desc) == PLORA_OK ? PLORA_ERR_WORKSPACE : validate(desc);
    if (need > (size_t)PLORA_NOALLOC_SCRATCH_BYTES) return PLORA_ERR_WORKSPACE;
    void *scratch = nullptr;
    plora_status ps = noalloc_scratch(&scratch);
    if (ps != PLORA_OK) return ps;
    return plora_linear_fwd(desc, x, W, A, B, y, h_saved, scratch, PLORA_NOALLOC_SCRATCH_BYTES, hip_stream);
}

plora_status plora_linear_fwd(const plora_desc *desc, const void *x, const void *W,
                              const void *const *A, const void *const *B, void *y, float *h_saved,
                              void *workspace, size_t ws_bytes, void *hip_stream)
{
    HostMeta m;
    plora_status ps = prepare(desc, x, W, A, B, workspace, ws_bytes, m);
    if (ps != PLORA_OK) return ps;
    if (!y && desc->T > 0) return PLORA_ERR_NULL;
    if (misaligned(y) || misaligned(h_saved)) return PLORA_ERR_ALIGN;
    if (desc->T == 0) return PLORA_OK;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    char *ws = static_cast<char *>(workspace);

    MetaView mv;
    const bool lora = m.hdr.n_blocks > 0;
    const bool bf = desc->dtype == PLORA_BF16;
    PL_TRY(prepare_device(m, ws, st, mv, ws + m.ws.at, nullptr, bf && lora, false, nullptr, nullptr));
    float *hf = h_saved ? h_saved : reinterpret_cast<float *>(ws + m.ws.hf);

    if (desc->dtype == PLORA_F32) {
        const float *xf = static_cast<const float *>(x);
        if (lora) { Bracket b(2, st); PL_TRY(launch_f32_lowrank(mv, m.hdr, 0, xf, desc->d_in, hf, st)); }
        { Bracket b(0, st);
          PL_TRY(launch_f32_gemm(mv, m.hdr, true, xf, static_cast<const float *>(W), hf, static_cast<float *>(y), st)); }
        return PLORA_OK;
    }

    void *at = ws + m.ws.at, *hb = ws + m.ws.hb;
    float *part = reinterpret_cast<float *>(ws + m.ws.part);
    if (lora) {
        Bracket b(2, st);
        PL_TRY(launch_skinny_bf16(mv, m.hdr, 0, x, desc->d_in, at, ws + m.ws.zero, part, h_saved, hb, nullptr, false, st));
    }
    { Bracket b(0, st);
      PL_TRY(launch_gemm_bf16(mv, m.hdr, true, x, W, hb, nullptr, ws + m.ws.zero, y, st)); }
    return PLORA_OK;
}

plora_status plora_linear_bwd(const plora_desc *desc, const void *x, const void *W,
                              const void *const *A, const void *const *B, const void *dy,
                              const float *h_saved, void *dx, float *const *dA, float *const *dB,
                              void *workspace, size_t ws_bytes, void *hip_stream)
{
    HostMeta m;
    plora_status ps = prepare(desc, x, W, A, B, workspace, ws_bytes, m);
    if (ps != PLORA_OK) return ps;
    if (!dy && desc->T > 0) return PLORA_ERR_NULL;
    if (misaligned(dy) || misaligned(dx) || misaligned(h_saved)) return PLORA_ERR_ALIGN;
    const bool want_w = (dA != nullptr) || (dB != nullptr);
    if (want_w && desc->n_adapters > 0) {
        if (!dA || !dB) return PLORA_ERR_NULL;
        for (int32_t k = 0; k < desc->n_adapters; ++k) {
            if (!dA[k] || !dB[k]) return PLORA_ERR_NULL;
            if (misaligned(dA[k]) || misaligned(dB[k])) return PLORA_ERR_ALIGN;
            m.ad[k].dA = dA[k]; m.ad[k].dB = dB[k];
        }
    }
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    char *ws = static_cast<char *>(workspace);
    const bool lora = m.hdr.n_blocks > 0;
    const bool any_w = want_w && desc->n_adapters > 0;
    if (desc->T == 0 && !any_w) return PLORA_OK;

    MetaView mv;
    {
        const bool bf = desc->dtype == PLORA_BF16;
        const bool need_shrink = any_w && !h_saved;
        PL_TRY(prepare_device(m, ws, st, mv, ws + m.ws.at, ws + m.ws.ap, bf && lora && need_shrink,
                              bf && lora && dx != nullptr, (bf && lora && any_w) ? h_saved : nullptr, ws + m.ws.zt_h));
    }

    if (desc->dtype == PLORA_F32) {
        const float *xf = static_cast<const float *>(x), *dyf = static_cast<const float *>(dy);
        float *gf = reinterpret_cast<float *>(ws + m.ws.gf);
        const float *hf = h_saved;
        if (lora && any_w && !hf) {
            Bracket b(2, st);
            float *hw = reinterpret_cast<float *>(ws + m.ws.hf);
            PL_TRY(launch_f32_lowrank(mv, m.hdr, 0, xf, desc->d_in, hw, st));
            hf = hw;
        }
        if (lora) { Bracket b(3, st); PL_TRY(launch_f32_lowrank(mv, m.hdr, 1, dyf, desc->d_out, gf, st)); }
        if (any_w) {
            { Bracket b(4, st); PL_TRY(launch_f32_wgrad(mv, m.hdr, false, dyf, desc->d_out, hf, st)); }
            { Bracket b(5, st); PL_TRY(launch_f32_wgrad(mv, m.hdr, true, xf, desc->d_in, gf, st)); }
        }
        if (dx && desc->T > 0) {
            Bracket b(1, st);
            PL_TRY(launch_f32_gemm(mv, m.hdr, false, dyf, static_cast<const float *>(W), gf, static_cast<float *>(dx), st));
        }
        return PLORA_OK;
    }

    void *at = ws + m.ws.at, *ap = ws + m.ws.ap, *gb = ws + m.ws.hb;
    void *zt_h = ws + m.ws.zt_h, *zt_g = ws + m.ws.zt_g;
    float *part = reinterpret_cast<float *>(ws + m.ws.part);
    float *wpart = reinterpret_cast<float *>(ws + m.ws.wpart);
    if (lora) {
        if (any_w && !h_saved) {
            Bracket b(2, st);
            PL_TRY(launch_skinny_bf16(mv, m.hdr, 0, x, desc->d_in, at, ws + m.ws.zero, part, nullptr, nullptr, zt_h, false, st));
        }
        { Bracket b(3, st);
          PL_TRY(launch_skinny_bf16(mv, m.hdr, 1, dy, desc->d_out, nullptr, ws + m.ws.zero, part, nullptr, gb, any_w ? zt_g : nullptr, true, st)); }
    }
    if (any_w) {
        { Bracket b(4, st); PL_TRY(launch_tokcontract_bf16(mv, m.hdr, false, dy, desc->d_out, zt_h, ws + m.ws.zero, wpart, m.split_dB, m.r16_total, m.n_active, st)); }
        { Bracket b(5, st); PL_TRY(launch_tokcontract_bf16(mv, m.hdr, true, x, desc->d_in, zt_g, ws + m.ws.zero, wpart, m.split_dA, m.r16_total, m.n_active, st)); }
    }
    if (dx && desc->T > 0) {
        Bracket b(1, st);
        PL_TRY(launch_gemm_bf16(mv, m.hdr, false, dy, W, gb, ap, ws + m.ws.zero, dx, st));
    }
    return PLORA_OK;
}

}  // extern "C"
