// Internal declarations shared by the host entry points and the HIP kernels of libplora.
// Not part of the public interface (that is include/plora.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "plora.h"

namespace plora {

constexpr int kSkinnyRows = 128;   // token block of the shrink / dH kernel (never straddles a segment)
constexpr int kRankPadGemm = 64;   // ranks are padded to one K-step of the GEMM in the bf16 side buffers
constexpr int kRankPadMfma = 16;   // ranks are padded to one MFMA block in the skinny kernels
constexpr int kTokPad = 64;        // segment lengths are padded to this in the transposed side buffers
constexpr int kZeroBytes = 1024;   // zero page at the head of the workspace
constexpr int kTokMaxSplits = 8;    // the dA / dB kernels split the token walk over at most this many workgroups
constexpr int kSkinnyMaxSplits = 8; // the skinny kernels split the contraction over at most this many workgroups
constexpr int kGemmTileRows = 256;  // row tile of the base GEMMs
constexpr int kGemmGroupRows = 4;   // row tiles that the GEMM's tile order keeps together on one XCD (they share W columns in its L2)

// ---------------------------------------------------------------------------------------------
// Segment-packing metadata (section 2.4: which rows belong to which adapter).
//
// The host validates the description and ships it to the device in a compact form (a few 32-bit
// words per segment and adapter, passed by value as a kernel argument).  The tables the kernels
// read are derived from it by one set of routines (derive_phase1, derive_phase2) compiled for both sides: the
// device runs them inside the preparation kernel and writes the tables into the workspace; the
// host runs the very same code to size the workspace, to plan the launches and to export the
// tables for the brute-force tests.
// ---------------------------------------------------------------------------------------------

// One entry per segment of the call (empty and base-only segments included).
struct SegInfo {
    int32_t row0, row1;   // token rows [row0, row1)
    int32_t adapter;      // -1: base weight only
    int32_t r;            // rank of the adapter (0 if none)
    int32_t rp;           // rank padded to kRankPadGemm: row pitch of the bf16 side buffer (0 if none)
    int32_t r16;          // rank padded to kRankPadMfma
    int32_t blk0;         // index of this segment's first token block (blocks of kSkinnyRows rows)
    int32_t lp;           // segment length padded to kTokPad: row pitch of the transposed side buffers
    int64_t h_off;        // element offset of the segment in the fp32 activation  [len][r]
    int64_t hb_off;       // element offset in the bf16 side buffer                [len][rp]
    int64_t zt_off;       // element offset in the transposed bf16 side buffers    [r16][lp]
};

// One entry per adapter.
struct AdapterInfo {
    const void *A;        // [d_in][r]
    const void *B;        // [r][d_out]
    float *dA;            // [d_in][r]   (backward only)
    float *dB;            // [r][d_out]  (backward only)
    int32_t r, rp, r16;
    float scale;
    int64_t at_off;       // element offset of A^T  [r16][d_in]  in the packed-A^T buffer
    int64_t ap_off;       // element offset of A    [d_in][rp]   in the padded-A buffer; with W stored [d_out][d_in]:
                          // of B^T [d_out][rp] in that same buffer
    int32_t r16_off;      // sum of r16 over the adapters before this one (row offset in dA / dB partial tiles)
    int32_t by_tokens;    // entry i: the adapter with the i-th largest token count (ties by index)
    int32_t seg_list0;    // this adapter's non-empty segments: seg_list[seg_list0 .. seg_list0 + n_own), in segment order
    int32_t n_own;
    int32_t tokens;       // tokens of this adapter over all its segments
    int32_t reserved;
    const void *ext_b;    // what GemmSeg::B is for this adapter's segments: B, or the packed A^T when W is [d_out][d_in]
};

struct MetaHeader {
    int64_t T, D, K;
    int32_t n_seg, n_adapters;
    int32_t n_blocks;     // token blocks of kSkinnyRows rows over all segments
    int32_t max_r16;      // largest rank (padded to 16) among segments with tokens
    int32_t w_out_in;     // 1: W is stored [d_out][d_in]
    int32_t reserved;
    const void *at_base;  // device address of the packed-A^T buffer (only used when w_out_in)
};

// What a 256-row tile of the base GEMMs needs to know about one segment whose low-rank term it adds.
struct GemmSeg {
    int32_t row0, row1;   // rows of the segment
    int32_t rp, r;        // padded and true rank
    int64_t hb_off;       // element offset of the segment in the bf16 low-rank factor [len][rp]
    const void *B;        // operand of the GEMM that reads W with the contraction index as row index, [r][N]:
                          // W[d_in][d_out]: forward, B_k;  W[d_out][d_in]: backward, the packed A_k^T
    int64_t ap_off;       // operand of the other GEMM, [N][rp], as element offset in the padded buffer:
                          // W[d_in][d_out]: backward, padded A_k;  W[d_out][d_in]: forward, padded B_k^T
};

// One entry per 256-row tile of the base GEMMs.  The low-rank term enters the GEMM as extra steps of
// the contraction loop, one per 64 padded rank columns of every segment with an adapter that
// overlaps the tile.  The first two such segments are spelled out, so that a tile gets all it needs
// with one fetch, issued a whole tile ahead.
struct GemmTile {
    int32_t n_ext;        // extension steps of the tile: sum of rp / 64 over the segments counted in n_own
    int32_t n_own;        // segments with an adapter and rows that overlap the tile
    int32_t first_seg;    // the first of them (n_seg if none)
    int32_t third_seg;    // the third of them (n_seg if fewer): where the walk over the segment table resumes
    GemmSeg s[2];
};

// Device view of the derived tables (all pointers into the workspace, laid out by table_layout).
struct MetaView {
    const MetaHeader *hdr;
    const SegInfo *seg;
    const AdapterInfo *ad;
    const GemmTile *tile;     // one per 256-row tile
    const int32_t *blk_seg;   // segment of each token block of kSkinnyRows rows
    const int32_t *seg_list;  // non-empty segments grouped by adapter (see AdapterInfo)
    const int32_t *tile_order;  // the GEMM row tiles ordered by extension steps, most first (ties: lower tile first)
};

// Several projections that read the same x (q / k / v, gate / up), fused along the rank: for adapter k the fused pass
// treats the rows of the projections' small factors, each padded to 16, as one factor of sum_p r16_{k,p} <= PLORA_MAX_RANK
// rows (appendix C.2's concatenation of adapters, applied across projections).  The rows stay where each projection's
// own kernels keep them; the fused kernels gather them 8 rows at a time.  The projections share the segments, so the
// token blocks, the per-adapter segment lists and the order by token count are those of projection 0.
constexpr int kMaxGroup = PLORA_MAX_GROUP;
struct GroupView {
    int32_t n_proj;               // projections fused in this launch (>= 2)
    int32_t max_r16;              // largest fused rank among the adapters with tokens
    int32_t r16_total;            // sum of the fused ranks over all adapters (rows of the dA partial tiles)
    int32_t reserved;
    MetaView mv[kMaxGroup];       // each projection's own tables
    const uint16_t *small[kMaxGroup];   // shrink: its packed-A^T buffer;  dA: its transposed bf16 g
};
struct NoGroup { int32_t unused; };

// ---- compact description -----------------------------------------------------------------------
// 32-bit words: [0,1] T  [2,3] D  [4,5] K  [6] n_seg  [7] n_adapters  [8] n_blocks (computed by the host, fixes the
// table layout)  [9] bit 0: W is stored [d_out][d_in], bit 1: the sorted order of the GEMM row tiles is the identity (the
// host knows from its own derivation; the device then skips the sort)  [10,11] device address of the packed-A^T buffer; then per segment
// {row1, adapter}; then per adapter {A lo, A hi, B lo, B hi, dA lo, dA hi, dB lo, dB hi, r, scale bits}.
constexpr int kDescHeadWords = 12, kDescSegWords = 2, kDescAdWords = 10;
constexpr int kChunkWords = 896;   // 3584 bytes: what one launch carries by value, below the 4 KB kernel-argument limit
struct DescChunk { uint32_t w[kChunkWords]; };

#define PLORA_HD __host__ __device__ inline

PLORA_HD int desc_words(int n_seg, int n_adapters) { return kDescHeadWords + kDescSegWords * n_seg + kDescAdWords * n_adapters; }

// Where the compact description lies: word(i) returns word i.
struct WordsInMemory {
    const uint32_t *p;
    PLORA_HD uint32_t word(int i) const { return p[i]; }
};

template <class Src> struct DescReader {
    Src src;
    PLORA_HD int64_t w64(int i) const { return (int64_t)((uint64_t)src.word(i) | ((uint64_t)src.word(i + 1) << 32)); }
    PLORA_HD int64_t T() const { return w64(0); }
    PLORA_HD int64_t D() const { return w64(2); }
    PLORA_HD int64_t K() const { return w64(4); }
    PLORA_HD int n_seg() const { return (int)src.word(6); }
    PLORA_HD int n_adapters() const { return (int)src.word(7); }
    PLORA_HD int n_blocks() const { return (int)src.word(8); }
    PLORA_HD int w_out_in() const { return (int)(src.word(9) & 1u); }
    PLORA_HD int order_is_identity() const { return (int)((src.word(9) >> 1) & 1u); }
    PLORA_HD const void *at_base() const { return reinterpret_cast<const void *>((uintptr_t)w64(10)); }
    PLORA_HD int seg_row1(int s) const { return (int)src.word(kDescHeadWords + kDescSegWords * s); }
    PLORA_HD int seg_row0(int s) const { return s ? seg_row1(s - 1) : 0; }
    PLORA_HD int seg_adapter(int s) const { return (int)src.word(kDescHeadWords + kDescSegWords * s + 1); }
    PLORA_HD int ad_base(int k) const { return kDescHeadWords + kDescSegWords * n_seg() + kDescAdWords * k; }
    PLORA_HD const void *ad_ptr(int k, int which) const { return reinterpret_cast<const void *>((uintptr_t)w64(ad_base(k) + 2 * which)); }
    PLORA_HD int ad_rank(int k) const { return (int)src.word(ad_base(k) + 8); }
    PLORA_HD float ad_scale(int k) const
    {
        union { uint32_t u; float f; } c;
        c.u = src.word(ad_base(k) + 9);
        return c.f;
    }
};

PLORA_HD int32_t pad_to(int32_t v, int32_t a) { return (v + a - 1) / a * a; }
PLORA_HD size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Byte offsets of the derived tables inside the metadata region of the workspace.
struct TableLayout {
    size_t hdr, seg, ad, tile, blk_seg, seg_list, tile_order, bytes;
    int64_t n_tiles;
};

PLORA_HD TableLayout table_layout(int64_t T, int n_seg, int n_adapters, int n_blocks)
{
    TableLayout l;
    size_t o = 0;
    l.n_tiles = (T + kGemmTileRows - 1) / kGemmTileRows;
    l.hdr = o;      o = align_up(o + sizeof(MetaHeader), 64);
    l.seg = o;      o = align_up(o + (size_t)n_seg * sizeof(SegInfo), 64);
    l.ad = o;       o = align_up(o + (size_t)n_adapters * sizeof(AdapterInfo), 64);
    l.tile = o;     o = align_up(o + (size_t)l.n_tiles * sizeof(GemmTile), 64);
    l.blk_seg = o;  o = align_up(o + (size_t)n_blocks * sizeof(int32_t), 64);
    l.seg_list = o; o = align_up(o + (size_t)n_seg * sizeof(int32_t), 64);
    l.tile_order = o; o = align_up(o + (size_t)l.n_tiles * sizeof(int32_t), 64);
    l.bytes = o;
    return l;
}

// Mutable pointers to the tables (a host buffer or the workspace).
struct Tables {
    MetaHeader *hdr;
    SegInfo *seg;
    AdapterInfo *ad;
    GemmTile *tile;
    int32_t *blk_seg;
    int32_t *seg_list;
    int32_t *tile_order;
};

PLORA_HD Tables tables_at(char *base, const TableLayout &l)
{
    Tables t;
    t.hdr = reinterpret_cast<MetaHeader *>(base + l.hdr);
    t.seg = reinterpret_cast<SegInfo *>(base + l.seg);
    t.ad = reinterpret_cast<AdapterInfo *>(base + l.ad);
    t.tile = reinterpret_cast<GemmTile *>(base + l.tile);
    t.blk_seg = reinterpret_cast<int32_t *>(base + l.blk_seg);
    t.seg_list = reinterpret_cast<int32_t *>(base + l.seg_list);
    t.tile_order = reinterpret_cast<int32_t *>(base + l.tile_order);
    return t;
}

PLORA_HD MetaView view_of(const Tables &t)
{
    MetaView v;
    v.hdr = t.hdr; v.seg = t.seg; v.ad = t.ad; v.tile = t.tile; v.blk_seg = t.blk_seg; v.seg_list = t.seg_list; v.tile_order = t.tile_order;
    return v;
}

// ---- derivation of the tables, in two phases ------------------------------------------------------
// Phase 1 runs on one thread (prefix sums over adapters and segments); phase 2 is loops
// "for (i = tid; i < n; i += nthreads)" over independent entries.  Phase 2 reads what phase 1 wrote, so
// the caller separates them with a barrier (device: one workgroup, __syncthreads; host: tid 0 of 1, nothing to do).

// scratch: 3 ints per adapter (tokens, non-empty segments, list cursor).  On the device it lies in LDS: the one
// thread that runs this phase then never waits for a load from memory - everything it reads comes from the
// description or from the scratch, everything it writes to the tables is a store it does not wait for.
// seg_copy / ad_copy (either may be null): a second place for the segment records and for what the tile records need
// of an adapter.  On the device they lie in LDS, so that the phases that follow read them from there and not from the
// tables in memory (every such read would be a trip to the L2, and the tile derivation chains several).
struct AdapterGemm {
    const void *ext_b;
    int64_t ap_off;
};

template <class Src> PLORA_HD void derive_phase1(const DescReader<Src> &in, const Tables &t, int32_t *scratch,
                                                 SegInfo *seg_copy, AdapterGemm *ad_copy, MetaHeader *hd_copy)
{
    const int n_seg = in.n_seg(), n_ad = in.n_adapters();
    const int64_t D = in.D();
    const int64_t ap_rows = in.w_out_in() ? in.K() : D;   // rows of the padded operand [rows][rp], see GemmSeg
    int32_t *tokens = scratch, *n_own = scratch + n_ad, *cursor = scratch + 2 * n_ad;
    for (int k = 0; k < n_ad; ++k) { tokens[k] = 0; n_own[k] = 0; }
    int64_t h = 0, hb = 0, zt = 0;
    int32_t blk = 0, max_r16 = 0, row0 = 0;
    for (int s = 0; s < n_seg; ++s) {
        SegInfo g;
        g.row0 = row0; g.row1 = in.seg_row1(s); row0 = g.row1;
        g.adapter = in.seg_adapter(s);
        const int32_t len = g.row1 - g.row0;
        const int32_t r = g.adapter >= 0 ? in.ad_rank(g.adapter) : 0;
        g.r = r;
        g.rp = pad_to(r, kRankPadGemm);
        g.r16 = pad_to(r, kRankPadMfma);
        g.lp = pad_to(len, kTokPad);
        g.blk0 = blk;
        g.h_off = h; g.hb_off = hb; g.zt_off = zt;
        if (g.adapter >= 0) {
            blk += (len + kSkinnyRows - 1) / kSkinnyRows;
            if (len > 0 && g.r16 > max_r16) max_r16 = g.r16;
            h += (int64_t)len * g.r;
            hb += (int64_t)len * g.rp;
            zt += (int64_t)g.r16 * g.lp;
            tokens[g.adapter] += len;
            n_own[g.adapter] += len > 0;
        }
        t.seg[s] = g;
        if (seg_copy) seg_copy[s] = g;
    }
    int64_t at = 0, ap = 0;
    int32_t r16_off = 0, list0 = 0;
    for (int k = 0; k < n_ad; ++k) {
        AdapterInfo a;
        a.A = in.ad_ptr(k, 0);
        a.B = in.ad_ptr(k, 1);
        a.dA = static_cast<float *>(const_cast<void *>(in.ad_ptr(k, 2)));
        a.dB = static_cast<float *>(const_cast<void *>(in.ad_ptr(k, 3)));
        a.r = in.ad_rank(k);
        a.rp = pad_to(a.r, kRankPadGemm);
        a.r16 = pad_to(a.r, kRankPadMfma);
        a.scale = in.ad_scale(k);
        a.at_off = at; at += (int64_t)a.r16 * D;
        // (integer arithmetic: the host derives the tables with a null base, and an offset from a null pointer is undefined)
        a.ext_b = in.w_out_in() ? reinterpret_cast<const void *>((uintptr_t)in.at_base() + 2 * (uintptr_t)a.at_off) : a.B;
        a.ap_off = ap; ap += (int64_t)a.rp * ap_rows;
        a.r16_off = r16_off; r16_off += a.r16;
        a.by_tokens = 0;                    // filled in by phase 2
        a.seg_list0 = list0; a.n_own = n_own[k]; a.tokens = tokens[k]; a.reserved = 0;
        cursor[k] = list0;
        list0 += n_own[k];
        t.ad[k] = a;
        if (ad_copy) { ad_copy[k].ext_b = a.ext_b; ad_copy[k].ap_off = a.ap_off; }
    }
    // per-adapter lists of non-empty segments, in segment order
    int32_t prev = 0;
    for (int s = 0; s < n_seg; ++s) {
        const int32_t row1 = in.seg_row1(s);
        const int a = in.seg_adapter(s);
        if (a >= 0 && row1 > prev) t.seg_list[cursor[a]++] = s;
        prev = row1;
    }
    MetaHeader hd;
    hd.T = in.T(); hd.D = D; hd.K = in.K();
    hd.n_seg = n_seg; hd.n_adapters = n_ad; hd.n_blocks = blk; hd.max_r16 = max_r16;
    hd.w_out_in = in.w_out_in(); hd.reserved = 0; hd.at_base = in.at_base();
    *t.hdr = hd;
    if (hd_copy) *hd_copy = hd;
}

PLORA_HD bool seg_has_lowrank(const SegInfo &g) { return g.adapter >= 0 && g.row1 > g.row0; }

// The segment that holds token block `blk` (only segments with an adapter and rows own blocks).
PLORA_HD int seg_of_block(const SegInfo *seg, int n_seg, int blk)
{
    int lo = 0, hi = n_seg - 1;                 // last segment with blk0 <= blk
    while (lo < hi) {
        const int mid = (lo + hi + 1) / 2;
        if (seg[mid].blk0 <= blk) lo = mid; else hi = mid - 1;
    }
    // blk < n_blocks lies in some owner o (o.blk0 <= blk < o.blk0 + blocks of o); every later segment starts at or
    // behind the end of o's blocks, so the last segment with blk0 <= blk is o itself
    return lo;
}

// Extension steps and the first segments of one GEMM row tile.  seg / ad: where to read the segment records and the
// adapters' GEMM operands from (the tables themselves, or the copies phase 1 made).
template <class AdSrc>
PLORA_HD void derive_tile(const Tables &t, const SegInfo *seg, const AdSrc *ad, int n_seg, int64_t T, int64_t tile)
{
    const int64_t m0 = tile * kGemmTileRows;
    const int64_t m1 = m0 + kGemmTileRows < T ? m0 + kGemmTileRows : T;
    int lo = 0, hi = n_seg;                     // first segment with row1 > m0
    while (lo < hi) {
        const int mid = (lo + hi) / 2;
        if (seg[mid].row1 > m0) hi = mid; else lo = mid + 1;
    }
    GemmTile gt;
    gt.n_ext = 0; gt.n_own = 0; gt.first_seg = n_seg; gt.third_seg = n_seg;
    for (int i = 0; i < 2; ++i) {
        gt.s[i].row0 = 0; gt.s[i].row1 = 0; gt.s[i].rp = 0; gt.s[i].r = 0;
        gt.s[i].hb_off = 0; gt.s[i].B = nullptr; gt.s[i].ap_off = 0;
    }
    for (int s = lo; s < n_seg && seg[s].row0 < m1; ++s) {
        const SegInfo g = seg[s];
        if (!seg_has_lowrank(g)) continue;
        if (gt.n_own < 2) {
            GemmSeg &q = gt.s[gt.n_own];
            q.row0 = g.row0; q.row1 = g.row1; q.rp = g.rp; q.r = g.r; q.hb_off = g.hb_off;
            q.B = ad[g.adapter].ext_b; q.ap_off = ad[g.adapter].ap_off;
            if (gt.n_own == 0) gt.first_seg = s;
        } else if (gt.n_own == 2) {
            gt.third_seg = s;
        }
        gt.n_own += 1;
        gt.n_ext += g.rp / kRankPadGemm;
    }
    t.tile[tile] = gt;
}

// hd: the header as phase 1 wrote it (passed by value so that nobody has to read it back); tokens: per-adapter token
// counts (phase 1's scratch).
template <class AdSrc>
PLORA_HD void derive_phase2(const Tables &t, const MetaHeader &hd, const SegInfo *seg, const AdSrc *ad, const int32_t *tokens,
                            int tid, int nthreads)
{
    const int n_seg = hd.n_seg, n_ad = hd.n_adapters, n_blocks = hd.n_blocks;
    const int64_t T = hd.T;
    const int64_t n_tiles = (T + kGemmTileRows - 1) / kGemmTileRows;
    for (int b = tid; b < n_blocks; b += nthreads) t.blk_seg[b] = seg_of_block(seg, n_seg, b);
    for (int64_t tile = tid; tile < n_tiles; tile += nthreads) derive_tile(t, seg, ad, n_seg, T, tile);
    // place of each adapter in the order by token count, longest first (the weight-gradient kernels hand out
    // adapters in that order, so the last workgroups are short)
    for (int k = tid; k < n_ad; k += nthreads) {
        const int32_t mine = tokens[k];
        int rank = 0;
        for (int j = 0; j < n_ad; ++j) {
            const int32_t theirs = tokens[j];
            if (theirs > mine || (theirs == mine && j < k)) ++rank;
        }
        t.ad[rank].by_tokens = k;
    }
}

// Phase 3 (after phase 2): the order in which the GEMMs walk their row tiles.  Workgroups that run side by side
// on one XCD work on a group of kGemmGroupRows consecutive entries of this order and share the columns of W they
// stream; they only stay in step if their tiles have the same number of contraction steps, so the row tiles are
// sorted by their extension steps, most first, tiles of equal length in row order (lengths of kSortKeys - 1 steps
// and more count as one class).  A counting sort in three steps with a barrier between them: every thread counts
// the classes in its own contiguous chunk of tiles, one thread per class turns the counts into start positions,
// every thread places its chunk.  counts: kSortKeys ints per thread (device: LDS; host: one thread).
constexpr int kSortKeys = 9;

PLORA_HD int sort_key(int32_t n_ext) { return n_ext < kSortKeys - 1 ? n_ext : kSortKeys - 1; }

PLORA_HD void tile_chunk(int64_t n_tiles, int tid, int nthreads, int64_t &lo, int64_t &hi)
{
    const int64_t per = (n_tiles + nthreads - 1) / nthreads;
    lo = per * tid < n_tiles ? per * tid : n_tiles;
    hi = lo + per < n_tiles ? lo + per : n_tiles;
}

PLORA_HD void derive_phase3_count(const Tables &t, int64_t n_tiles, int tid, int nthreads, int32_t *counts)
{
    int64_t lo, hi;
    tile_chunk(n_tiles, tid, nthreads, lo, hi);
    int32_t c[kSortKeys];
    for (int k = 0; k < kSortKeys; ++k) c[k] = 0;
    for (int64_t i = lo; i < hi; ++i) c[sort_key(t.tile[i].n_ext)] += 1;
    for (int k = 0; k < kSortKeys; ++k) counts[tid * kSortKeys + k] = c[k];
}

// counts[thread][class] -> starts[thread][class]: position of the first tile of that class in that thread's chunk
PLORA_HD void derive_phase3_scan(int tid, int nthreads, const int32_t *counts, int32_t *starts)
{
    for (int k = tid; k < kSortKeys; k += nthreads) {       // one thread per class
        int32_t base = 0;
        for (int kk = kSortKeys - 1; kk > k; --kk)          // all tiles of the longer classes come first
            for (int th = 0; th < nthreads; ++th) base += counts[th * kSortKeys + kk];
        for (int th = 0; th < nthreads; ++th) {
            starts[th * kSortKeys + k] = base;
            base += counts[th * kSortKeys + k];
        }
    }
}

PLORA_HD void derive_phase3_place(const Tables &t, int64_t n_tiles, int tid, int nthreads, const int32_t *starts)
{
    int64_t lo, hi;
    tile_chunk(n_tiles, tid, nthreads, lo, hi);
    int32_t pos[kSortKeys];
    for (int k = 0; k < kSortKeys; ++k) pos[k] = starts[tid * kSortKeys + k];
    for (int64_t i = lo; i < hi; ++i) t.tile_order[pos[sort_key(t.tile[i].n_ext)]++] = (int32_t)i;
}

// Byte offsets of the workspace regions, each 256-byte aligned.
struct WorkspaceLayout {
    size_t zero, meta, desc, at, ap, hb, zt_h, zt_g, hf, gf, part, wpart, total;
    size_t meta_bytes;
};

// ---- launch wrappers implemented in the kernel files; all enqueue on `st` and return the HIP status ----

// Compute units of the current device (thread-safe, looked up once per device); 0 with *err set on failure.
int device_cu_count(hipError_t *err);
// Lets `kernel` use up to the 160 KB of LDS of a compute unit; done once per device and kernel (slot: a small
// index that is unique per kernel), thread-safe.
hipError_t allow_full_lds(const void *kernel, int slot);
constexpr int kLdsSlots = 16;

// Metadata and the small jobs in front of the heavy kernels, in one launch when the compact description fits a
// kernel argument (otherwise it is first uploaded in chunks to desc_stage): derived tables and zero page into the
// workspace; packing of A_k (bf16 path: A_k^T [r16][d_in] with zero rows beyond r, and / or A_k padded to rp
// columns); transposed bf16 copy of a saved activation, zt[j][t] = bf16(h[t][j]) (bf16 backward).
// want_bp (instead of want_ap, W stored [d_out][d_in]): B_k^T [d_out][rp] with zero columns beyond r into `ap`.
hipError_t launch_prep(const uint32_t *desc_host, int n_words, const MetaHeader &h, char *meta_dev, uint32_t *desc_stage,
                       void *zero_dev, void *at, void *ap, bool want_at, bool want_ap, bool want_bp, const float *hf,
                       void *zt, hipStream_t st);

// bf16 path -------------------------------------------------------------------------------------
// Skinny product over token blocks: acc[t][j] = sum_c S[t][c] * Bm_k[j][c]  (c < C).
//   mode 0 (shrink): S = x (C = d_in), Bm_k = packed A_k^T;  mode 1 (dH): S = dy (C = d_out), Bm_k = B_k.
//   `part` receives the fp32 partial tiles of the contraction splits; a finishing kernel sums them and
//   writes (each optional): hf fp32 [len][r] (unscaled in mode 0); hb bf16 [len][rp] = scale_k*acc;
//   zt bf16 [r16][lp] transposed, = (zt_scaled ? scale_k : 1) * acc.
hipError_t launch_skinny_bf16(const MetaView &mv, const MetaHeader &h, int mode, const void *S, int64_t C,
                              const void *at, const void *zero, float *part, float *hf, void *hb, void *zt,
                              bool zt_scaled, hipStream_t st);
// C[T][N] = S[T][Kd] * Wop + side[T][rp] * ext_k, rounded to bf16.
//   w_rows_contract : Wop = W [Kd][N] (contraction index is the row index),  ext_k = GemmSeg::B   [r][N]
//   otherwise       : Wop = W [N][Kd] (contraction index is contiguous),     ext_k = ap + GemmSeg::ap_off [N][rp]
//   W[d_in][d_out]: forward (S = x, Kd = d_in, N = d_out) is the first form, backward (S = dy, Kd = d_out, N = d_in)
//   the second; W[d_out][d_in]: the other way round.
//   accumulate: C += the product (C is read in the epilogue and the sum rounded once more), otherwise C is overwritten
hipError_t launch_gemm_bf16(const MetaView &mv, const MetaHeader &h, bool w_rows_contract, int64_t Kd, int64_t N,
                            const void *S, const void *W, const void *side, const void *ap, const void *zero, void *C,
                            bool accumulate, hipStream_t st);
// Stand-alone low-rank update C[T][N] += side * op_k (bf16, one rounding): side = bf16 low-rank factor [len][rp] per
// segment, opT = padded small matrices [N][rp] (adapter k at N * (ap_off_k / table_rows)).
hipError_t launch_expand_bf16(const MetaView &mv, const MetaHeader &h, void *C, int64_t N, const void *side, const void *opT,
                              int64_t table_rows, const void *zero, hipStream_t st);
// Token contraction: out_k = mult * sum_t S[t][c] * zt[j][t] over all segments of adapter k.
//   want_dA: S = x, out = dA_k[c][j], mult = 1;  else S = dy, out = dB_k[j][c], mult = scale_k.
//   n_split > 1: the token walk is split, partial tiles go through `part` ([split][r16_total][C] fp32).
hipError_t launch_tokcontract_bf16(const MetaView &mv, const MetaHeader &h, bool want_dA, const void *S,
                                   int64_t C, const void *zt, const void *zero, float *part, int n_split,
                                   int r16_total, int n_active_adapters, hipStream_t st);
// The same two passes for several projections at once (see GroupView).  hv: projection 0's header with max_r16 replaced
// by the fused one.  Shrink: hf / hb / zt per projection as in launch_skinny_bf16 (mode 0).  dA: the results go to each
// projection's own dA_k; n_split must be tokc_splits(hv, C, n_active_adapters).
hipError_t launch_skinny_group(const GroupView &gv, const MetaHeader &hv, const void *x, int64_t C, const void *zero, float *part,
                               float *const *hf, void *const *hb, void *const *zt, hipStream_t st);
hipError_t launch_tokc_group_dA(const GroupView &gv, const MetaHeader &hv, const void *x, int64_t C, const void *zero,
                                float *part, int n_split, int n_active_adapters, hipStream_t st);
int tokc_splits(const MetaHeader &h, int64_t C, int n_active_adapters);
int tokc_tile_columns(const MetaHeader &h, int64_t C, int n_active_adapters);
int skinny_splits(const MetaHeader &h, int64_t C);

// fp32 path (fp64 accumulation) ---------------------------------------------------------------------
hipError_t launch_f32_lowrank(const MetaView &mv, const MetaHeader &h, int mode, const float *S, int64_t C,
                              float *out, hipStream_t st);
hipError_t launch_f32_gemm(const MetaView &mv, const MetaHeader &h, bool forward, const float *S, const float *W,
                           const float *side, float *C, bool accumulate, hipStream_t st);   // W's layout: h.w_out_in
// to_y: y += scale_k h B_k (side = h);  else dx += g A_k^T (side = g, which carries scale_k).
hipError_t launch_f32_expand(const MetaView &mv, const MetaHeader &h, bool to_y, float *C, const float *side, hipStream_t st);
hipError_t launch_f32_wgrad(const MetaView &mv, const MetaHeader &h, bool want_dA, const float *S, int64_t C,
                            const float *side, hipStream_t st);

// NF4 base weight: out[i] = level[index_i] * absmax[i / 64] for n_elems elements (a multiple of 64), bf16 or fp32.
hipError_t launch_nf4_dequant(const void *codes, const float *absmax, int64_t n_elems, bool bf16, void *out, hipStream_t st);

// optimizer ----------------------------------------------------------------------------------------
struct AdamwTensor {
    void *param; float *master; const float *grad; float *m, *v;
    uint64_t numel;
    float lr, beta1, beta2, eps, weight_decay;
    int32_t step;
    float grad_scale;
};
// AdamW step of n tensors (any sizes, each with its own hyperparameters); bf16 tells the type of `param`.
hipError_t launch_adamw(const AdamwTensor *t, int n, bool bf16, hipStream_t st);

}  // namespace plora
