// Weight gradients of the packed multi-LoRA layer on bf16 inputs (gfx950): the two products that
// contract over the token axis (appendix C.2),
//   case 3   dA_k[c][j] =           sum_t x_t[c]  g_t[j]      (g carries scale_k)
//   case 1   dB_k[j][c] = scale_k * sum_t dy_t[c] h_t[j]
// summed over every segment of adapter k.  Each streams a big [T][C] matrix once (bound by HBM)
// against the small transposed bf16 factor zt[j][t] written by the skinny kernel.
//
// The token index is the slow index of the big matrix, so its MFMA operand needs a transpose; it
// is staged HBM -> LDS as it lies in memory (direct loads into a ring of stages that fills the LDS)
// and read with the transposing LDS load (ds_read_b64_tr_b16).  The rank stays whole in every tile;
// tiles are cut along the hidden dimension (256 or 128 columns per workgroup, one wave per 32
// columns) and a workgroup walks the tokens of one adapter, longest adapters first.  The MFMA code
// is specialised per number of 16-wide rank blocks so that every LDS read of a stage is in flight
// before the first MFMA.  Nothing in the loop may spill: a scratch reload waits on the same counter
// as the direct loads and would drain the ring.
// When that gives too few workgroups to fill the chip the token walk is split as well and
// the fp32 partial tiles are summed, in a fixed order, by a small finishing kernel; otherwise the
// result is written directly.  No atomics anywhere: the summation order is fixed.
#include "plora_internal.h"
#include <type_traits>

namespace plora {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T *)(p))

constexpr int TC_BT = 64;                  // tokens per stage (TC_BT / 32 MFMA K steps)
constexpr int TC_MAX_NST = 8;              // LDS ring stages: as many as fit in the 160 KB of a compute unit, at most this
constexpr int TC_LDS_BYTES = 160 * 1024;
constexpr int TC_CB = 2;                                  // 16-column MFMA blocks per wave: a wave owns 32 columns
constexpr int TC_SL = TC_BT * 32 * 2 / 1024;              // big-matrix load instructions per wave per stage (4)
constexpr int TC_NB = PLORA_MAX_RANK / 16;
constexpr int TC_KS = TC_BT / 32;                         // MFMA K steps per stage
constexpr int TC_ZC = TC_BT / 8;                          // 16-byte chunks per small-factor row
constexpr int TC_ZR = 64 / TC_ZC;                         // small-factor rows per load instruction
constexpr int TC_ZSH = TC_ZC == 4 ? 2 : 1;                // rows that share a 256-byte LDS line: 4 or 2
static_assert(TC_BT == 32 || TC_BT == 64, "");

__device__ inline void tc_wait_vmcnt(int n)
{
#define W_(N) case N: __builtin_amdgcn_s_waitcnt(0x0f70 | (N & 15) | ((N >> 4) << 14)); break;
    switch (n) {
        W_(0) W_(1) W_(2) W_(3) W_(4) W_(5) W_(6) W_(7) W_(8) W_(9) W_(10) W_(11) W_(12) W_(13) W_(14) W_(15) W_(16)
        W_(17) W_(18) W_(19) W_(20) W_(21) W_(22) W_(23) W_(24) W_(25) W_(26) W_(27) W_(28) W_(29) W_(30) W_(31) W_(32)
        W_(33) W_(34) W_(35) W_(36) W_(37) W_(38) W_(39) W_(40) W_(41) W_(42) W_(43) W_(44) W_(45) W_(46) W_(47) W_(48)
    default: __builtin_amdgcn_s_waitcnt(0x0f70); break;    // never reached: at most (TC_MAX_NST - 2) * 6 loads stay in flight
    }
#undef W_
}

// grid (column tiles, adapters, token splits).  part != nullptr: write the fp32 partial tile
// [r16][C] of this split instead of the final result.
// GROUP (dA only): the small factor of adapter k is the transposed g of several projections that share x, one below
// the other (GroupView); mv is projection 0's view, `zt` is not used, every projection's dA_k gets its own columns.
template <bool WANT_DA, int BC, bool GROUP = false>
__global__ void __launch_bounds__(2 * BC) __attribute__((amdgpu_waves_per_eu(2, 2))) k_tokc(MetaView mv, const uint16_t *__restrict__ S, int C,
                                             const uint16_t *__restrict__ zt, const uint16_t *__restrict__ zero,
                                             float *__restrict__ part, int r16_total, int nst,
                                             std::conditional_t<GROUP, GroupView, NoGroup> gv)
{
    static_assert(!GROUP || WANT_DA, "");
    // BC columns of the big matrix per workgroup (256 or 128), one wave per 32 columns
    static_assert(BC == 256 || BC == 128, "");
    constexpr int TC_BC = BC, TC_NW = BC / 32, TC_S_BYTES = TC_BT * BC * 2;
    constexpr int CPRW = BC / 8;                                  // 16-byte chunks per row of the big-matrix tile
    constexpr int RPIW = 64 / CPRW;                               // rows per 1 KB load instruction
    // 16-byte chunk c of token row u is stored at slot c ^ swz(u); chosen so that the 8 rows (u..u+3 and
    // u+8..u+11) that one pass of a transposing read touches fall into 8 different 32-byte bank groups
    auto swz = [](int u) {
        return BC == 256 ? 4 * (u & 3) + 2 * ((u >> 3) & 1) : 2 * (u & 3) + 8 * ((u >> 3) & 1);
    };
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    const int k = mv.ad[blockIdx.y].by_tokens;       // longest adapters first
    const AdapterInfo a = mv.ad[k];
    const int c0 = blockIdx.x * TC_BC;
    int r16 = a.r16, max_r16;
    int p_r16[kMaxGroup];                            // GROUP: rank rows (padded to 16) of each projection
    if constexpr (GROUP) {
        r16 = 0;
#pragma unroll
        for (int p = 0; p < kMaxGroup; ++p) {
            p_r16[p] = p < gv.n_proj ? gv.mv[p].ad[k].r16 : 0;
            r16 += p_r16[p];
        }
        max_r16 = gv.max_r16;
    } else {
        max_r16 = mv.hdr->max_r16;
    }
    const int nb = r16 / 16;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t lds_base = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)LDS_PTR(char, lds));
    const int stage_bytes = TC_S_BYTES + max_r16 * TC_BT * 2;

    // steps (TC_BT tokens each) of this adapter over its own segments (list built on the host), and the
    // slice of them that belongs to this split
    const int32_t *own = mv.seg_list + a.seg_list0;
    const int n_own = a.n_own;
    int n_steps_all = 0;
    for (int li = 0; li < n_own; ++li) {
        const SegInfo g = mv.seg[own[li]];
        n_steps_all += (g.row1 - g.row0 + TC_BT - 1) / TC_BT;
    }
    const int per = (n_steps_all + gridDim.z - 1) / gridDim.z;
    const int step0 = blockIdx.z * per;
    int n_steps = n_steps_all - step0;
    n_steps = n_steps < per ? n_steps : per;
    if (n_steps < 0) n_steps = 0;

    // cursor of the next stage to fetch: index into the adapter's segment list, token offset inside that
    // segment, and the fields of the segment that the loader needs (kept in registers so that the load
    // issue right behind the barrier does not wait for a metadata fetch)
    int cur_li = 0, cur_t = 0;
    for (int skip = step0; skip > 0 && cur_li < n_own;) {
        const SegInfo g = mv.seg[own[cur_li]];
        const int st_here = (g.row1 - g.row0 + TC_BT - 1) / TC_BT;
        if (skip >= st_here) { skip -= st_here; ++cur_li; }
        else { cur_t = skip * TC_BT; skip = 0; }
    }
    // GROUP: the 8 rows that small-factor load instruction q = wave + TC_NW jj covers lie in one projection: zp[jj], and
    // zfirst[jj] is the first of that projection's rows in the fused factor
    constexpr int ZL = (PLORA_MAX_RANK / TC_ZR + TC_NW - 1) / TC_NW;
    int zp[ZL], zfirst[ZL];
    if constexpr (GROUP) {
#pragma unroll
        for (int jj = 0; jj < ZL; ++jj) {
            const int u = (wave + TC_NW * jj) * TC_ZR;
            int cum = 0;
            zp[jj] = 0; zfirst[jj] = 0;
#pragma unroll
            for (int p = 1; p < kMaxGroup; ++p) {
                cum += p_r16[p - 1];
                if (p < gv.n_proj && u >= cum) { zp[jj] = p; zfirst[jj] = cum; }
            }
        }
    }
    int seg_row0 = 0, seg_len = 0, seg_lp = 0;
    int64_t seg_zt = 0;
    const uint16_t *seg_zp[ZL];                      // GROUP: start of the current segment's rows in projection zp[jj]'s buffer
    auto load_desc = [&]() {
        if (cur_li < n_own) {
            const int sidx = own[cur_li];
            const SegInfo g = mv.seg[sidx];
            seg_row0 = g.row0; seg_len = g.row1 - g.row0; seg_lp = g.lp; seg_zt = g.zt_off;
            if constexpr (GROUP) {
#pragma unroll
                for (int jj = 0; jj < ZL; ++jj) seg_zp[jj] = gv.small[zp[jj]] + gv.mv[zp[jj]].seg[sidx].zt_off;
            }
        }
    };
    load_desc();

    // ---- loader.  Big-matrix tile [TC_BT t][CPRW chunks]: instruction q covers token rows RPIW q ..,
    // lane -> (row RPIW q + lane / CPRW, slot lane % CPRW); wave w issues q = w, w + TC_NW, ...
    // Small-factor tile [r16 j][TC_ZC chunks]:
    // instruction q covers rows TC_ZR q.., lane -> (row TC_ZR q + lane/TC_ZC, slot lane%TC_ZC), slot c' of
    // row u holds chunk c' ^ ((u >> TC_ZSH) & (TC_ZC-1)); wave w issues q = w, w + TC_NW, ... below r16/TC_ZR.
    const int nzi = r16 / TC_ZR;
    const int my_z = (nzi > wave) ? (nzi - wave + TC_NW - 1) / TC_NW : 0;
    const int lps = TC_SL + my_z;
    auto load16 = [&](const uint16_t *gp, uint32_t dst) {
        asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gp), "s"(dst));
    };
    auto issue = [&](int slot) {
        const uint32_t base = lds_base + slot * stage_bytes;
        const int tbase = __builtin_amdgcn_readfirstlane(cur_t);
#pragma unroll
        for (int jj = 0; jj < TC_SL; ++jj) {
            const int q = wave + TC_NW * jj;
            const int u = q * RPIW + lane / CPRW;
            const int chunk = (lane % CPRW) ^ swz(u);
            int c = c0 + chunk * 8;
            c = c < C ? c : C - 8;                                  // columns past the end only feed outputs that are not stored
            const int t = tbase + u;
            const uint16_t *p = (t < seg_len) ? S + (int64_t)(seg_row0 + t) * C + c : zero;
            load16(p, base + q * 1024);
        }
#pragma unroll
        for (int jj = 0; jj < (PLORA_MAX_RANK / TC_ZR + TC_NW - 1) / TC_NW; ++jj) {
            if (jj < my_z) {
                const int q = wave + TC_NW * jj;
                const int u = q * TC_ZR + lane / TC_ZC;
                const int chunk = (lane % TC_ZC) ^ ((u >> TC_ZSH) & (TC_ZC - 1));
                if constexpr (GROUP) load16(seg_zp[jj] + (int64_t)(u - zfirst[jj]) * seg_lp + tbase + chunk * 8, base + TC_S_BYTES + q * 1024);
                else load16(zt + seg_zt + (int64_t)u * seg_lp + tbase + chunk * 8, base + TC_S_BYTES + q * 1024);
            }
        }
        cur_t = tbase + TC_BT;
        if (cur_t >= seg_len) { ++cur_li; cur_t = 0; load_desc(); }
    };

    // ---- MFMA operands.  Wave w owns columns 32w..32w+31 (two 16-column blocks) and every rank block.
    // Transposing read of the big-matrix operand: the 16 lanes of group kg fetch the 4(t) x 16(c) block
    // at tokens 32*ks + 8*kg (+4 for the second read), 8 bytes each; lane i then holds column i.
    const int i16 = lane & 15, kg = lane >> 4;
    int soff[TC_CB];
#pragma unroll
    for (int cb = 0; cb < TC_CB; ++cb) {
        const int u = kg * 8 + (i16 >> 2);                            // token row fetched by this lane (first read)
        const int cl = wave * (TC_CB * 16) + cb * 16 + (i16 & 3) * 4; // first column fetched by this lane
        soff[cb] = u * (TC_BC * 2) + ((((cl >> 3) ^ swz(u)) * 16) + (cl & 7) * 2);
    }
    // second read (token row u+4) and later K steps (u+32): (u&3) and (u>>3)&1 unchanged, plain adds
    // small-factor operand: rank row j = 16b + i16, chunk 4*ks + kg; the swizzle term only depends on
    // i16, so block b sits 16 rows behind block b-1 and K step ks flips one offset bit
    const int zoff0 = TC_S_BYTES + i16 * (TC_BT * 2) + ((kg ^ ((i16 >> TC_ZSH) & (TC_ZC - 1))) * 16);

    f32x4 acc[TC_CB][TC_NB];
#pragma unroll
    for (int cb = 0; cb < TC_CB; ++cb)
#pragma unroll
        for (int b = 0; b < TC_NB; ++b) acc[cb][b] = f32x4{0.f, 0.f, 0.f, 0.f};

    auto compute = [&](auto nbc, const char *sb) {
        constexpr int NBC = decltype(nbc)::value;
#pragma unroll
        for (int ks = 0; ks < TC_KS; ++ks) {
            bf16x8 sf[TC_CB], zf[NBC];
#pragma unroll
            for (int cb = 0; cb < TC_CB; ++cb) {
                const char *p = sb + soff[cb] + ks * 32 * (TC_BC * 2);
                bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(LDS_PTR(bf16x4, p));
                bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(LDS_PTR(bf16x4, p + 4 * (TC_BC * 2)));
                sf[cb] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            }
#pragma unroll
            for (int b = 0; b < NBC; ++b) zf[b] = *LDS_PTR(const bf16x8, sb + (zoff0 ^ (ks * 64)) + b * 16 * (TC_BT * 2));
#pragma unroll
            for (int b = 0; b < NBC; ++b)
#pragma unroll
                for (int cb = 0; cb < TC_CB; ++cb)
                    acc[cb][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(sf[cb], zf[b], acc[cb][b], 0, 0, 0);
        }
    };

    // ring of nst stages: stage `it` lives in slot it % nst; nst - 1 stages are in flight ahead of the reader
    for (int p = 0; p < nst - 1; ++p)
        if (p < n_steps) issue(p);
    int rd_slot = 0, wr_slot = nst - 1;
    for (int it = 0; it < n_steps; ++it) {
        const int ahead = (n_steps - 1 - it < nst - 2) ? n_steps - 1 - it : nst - 2;
        tc_wait_vmcnt(ahead * lps);
        __builtin_amdgcn_s_waitcnt(0xc07f);      // this wave's LDS reads of the slot about to be refilled are done
        __builtin_amdgcn_sched_barrier(0);       // (nothing may be moved across the barrier)
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        if (it + nst - 1 < n_steps) issue(wr_slot);
        const char *sb = lds + rd_slot * stage_bytes;
        rd_slot = (rd_slot + 1 == nst) ? 0 : rd_slot + 1;
        wr_slot = (wr_slot + 1 == nst) ? 0 : wr_slot + 1;
        // straight-line code for each possible number of rank blocks: every LDS read of the stage is
        // issued before the first MFMA, so their latencies overlap instead of adding up per block
        switch (nb) {
        case 1: compute(std::integral_constant<int, 1>{}, sb); break;
        case 2: compute(std::integral_constant<int, 2>{}, sb); break;
        case 3: compute(std::integral_constant<int, 3>{}, sb); break;
        case 4: compute(std::integral_constant<int, 4>{}, sb); break;
        case 5: compute(std::integral_constant<int, 5>{}, sb); break;
        case 6: compute(std::integral_constant<int, 6>{}, sb); break;
        case 7: compute(std::integral_constant<int, 7>{}, sb); break;
        default: compute(std::integral_constant<int, 8>{}, sb); break;
        }
    }

    // ---- epilogue.  Lane holds rank column j = 16b + i16 and big-matrix columns c = cbase + 4*kg + i.
    const float mult = WANT_DA ? 1.f : a.scale;
    int r16_off = a.r16_off;
    if constexpr (GROUP) {
        r16_off = 0;                                  // rows of the fused factors of the adapters before this one
        for (int p = 0; p < gv.n_proj; ++p) r16_off += gv.mv[p].ad[k].r16_off;
    }
#pragma unroll
    for (int cb = 0; cb < TC_CB; ++cb) {
        const int c = c0 + wave * (TC_CB * 16) + cb * 16 + kg * 4;
#pragma unroll
        for (int b = 0; b < TC_NB; ++b) {
            const int j = b * 16 + i16;
            if (b < nb && c < C) {
                if (part) {
                    float4 v;
                    v.x = acc[cb][b][0]; v.y = acc[cb][b][1]; v.z = acc[cb][b][2]; v.w = acc[cb][b][3];
                    *reinterpret_cast<float4 *>(part + ((int64_t)blockIdx.z * r16_total + r16_off + j) * C + c) = v;
                } else if constexpr (GROUP) {
                    int pj = 0, first = 0, cum = 0;   // the projection that owns rank block b, and its first row
#pragma unroll
                    for (int p = 1; p < kMaxGroup; ++p) {
                        cum += p_r16[p - 1];
                        if (p < gv.n_proj && b * 16 >= cum) { pj = p; first = cum; }
                    }
                    const AdapterInfo ap = gv.mv[pj].ad[k];
                    const int jl = j - first;
                    if (jl < ap.r) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) ap.dA[(int64_t)(c + i) * ap.r + jl] = acc[cb][b][i];
                    }
                } else if (j < a.r) {
                    if (WANT_DA) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) a.dA[(int64_t)(c + i) * a.r + j] = acc[cb][b][i];
                    } else {
                        float4 v;
                        v.x = mult * acc[cb][b][0]; v.y = mult * acc[cb][b][1];
                        v.z = mult * acc[cb][b][2]; v.w = mult * acc[cb][b][3];
                        *reinterpret_cast<float4 *>(a.dB + (int64_t)j * C + c) = v;
                    }
                }
            }
        }
    }
}

// Sums the partial tiles [split][r16 rows][C] in split order and writes dA_k[c][j] or scale_k-scaled
// dB_k[j][c].  grid (C / 256, rank rows of all adapters); one output element per thread.
template <bool WANT_DA>
__global__ void __launch_bounds__(256) k_tokc_finish(MetaView mv, const float *__restrict__ part, int C, int n_split,
                                                    int r16_total)
{
    const int row = blockIdx.y;                      // row of the concatenated [r16_total][C] partial tile
    const int n_ad = mv.hdr->n_adapters;
    int k = 0;
    for (int q = 0; q < n_ad; ++q)
        if (row >= mv.ad[q].r16_off) k = q;
    const AdapterInfo a = mv.ad[k];
    const int j = row - a.r16_off;
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (j >= a.r || c >= C) return;
    float v[kTokMaxSplits];
#pragma unroll
    for (int sp = 0; sp < kTokMaxSplits; ++sp)
        v[sp] = (sp < n_split) ? part[((int64_t)sp * r16_total + row) * C + c] : 0.f;
    float sum = v[0];
#pragma unroll
    for (int sp = 1; sp < kTokMaxSplits; ++sp) sum += v[sp];
    if (WANT_DA) a.dA[(int64_t)c * a.r + j] = sum;
    else a.dB[(int64_t)j * C + c] = a.scale * sum;
}

// The same for the partial tiles of a fused dA pass: row -> adapter -> projection -> that projection's dA_k.
__global__ void __launch_bounds__(256) k_tokc_finish_group(GroupView gv, const float *__restrict__ part, int C, int n_split)
{
    const int row = blockIdx.y;                      // row of the concatenated [r16_total][C] partial tile
    const int n_ad = gv.mv[0].hdr->n_adapters;
    int k = 0, k_off = 0;
    for (int q = 0; q < n_ad; ++q) {
        int off = 0;
        for (int p = 0; p < gv.n_proj; ++p) off += gv.mv[p].ad[q].r16_off;
        if (row >= off) { k = q; k_off = off; }
    }
    int j = row - k_off, pj = 0;                     // row inside the fused factor of adapter k -> projection, local row
    for (; pj < gv.n_proj - 1; ++pj) {
        const int r16 = gv.mv[pj].ad[k].r16;
        if (j < r16) break;
        j -= r16;
    }
    const AdapterInfo a = gv.mv[pj].ad[k];
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (j >= a.r || c >= C) return;
    float sum = part[(int64_t)row * C + c];
    for (int sp = 1; sp < n_split; ++sp) sum += part[((int64_t)sp * gv.r16_total + row) * C + c];   // fixed order
    a.dA[(int64_t)c * a.r + j] = sum;
}

// Launch shape: column-tile width and number of token splits.  128-column tiles throughout: two workgroups then
// share a compute unit, which pays more than the wider rows of 256-column tiles (measured: dB 8-19 % faster at the
// wide layers, the rest within a few percent either way; the 256-column instantiation is kept for tuning).  When the
// tiles alone give fewer than about two workgroups per compute unit the token walk is split as well; the split is
// capped so that a split keeps about four stages, and so that the fp32 partial tiles (written once, read once) stay
// below half of the bytes of the big matrix.
static int tokc_plan(const MetaHeader &h, int64_t C, int n_active_adapters, int *bc_out)
{
    const int bc = 128;
    int splits = 1;
    if (n_active_adapters > 0) {
        const int64_t wgs = (C + 127) / 128 * n_active_adapters;
        int want = (int)((512 + wgs - 1) / wgs);
        int cap = (int)(h.T / TC_BT / n_active_adapters / 4);
        const int64_t r16_sum = (int64_t)h.n_adapters * (h.max_r16 > 0 ? h.max_r16 : 16);   // upper bound of the partial rows
        const int cap_bytes = (int)(h.T / (8 * r16_sum));
        if (cap > cap_bytes) cap = cap_bytes;
        if (cap < 1) cap = 1;
        if (want > cap) want = cap;
        if (want > kTokMaxSplits) want = kTokMaxSplits;
        splits = want < 1 ? 1 : want;
    }
    if (bc_out) *bc_out = bc;
    return splits;
}

int tokc_splits(const MetaHeader &h, int64_t C, int n_active_adapters)
{
    return tokc_plan(h, C, n_active_adapters, nullptr);
}

int tokc_tile_columns(const MetaHeader &h, int64_t C, int n_active_adapters)
{
    int bc = 256;
    (void)tokc_plan(h, C, n_active_adapters, &bc);
    return bc;
}

template <bool WANT_DA, int BC>
static hipError_t launch_tokc(const MetaView &mv, const MetaHeader &h, const uint16_t *S, int C, const uint16_t *zt,
                              const uint16_t *zero, float *part, int n_split, int r16_total, hipStream_t st)
{
    // ring depth: the share of the 160 KB of LDS that lets 256 / BC workgroups sit on a compute unit,
    // but two stages at least (a second workgroup on the compute unit pays more than a third stage: measured)
    const size_t stage = (size_t)TC_BT * BC * 2 + (size_t)(h.max_r16 > 0 ? h.max_r16 : 16) * TC_BT * 2;
    size_t budget = (size_t)TC_LDS_BYTES * BC / 256;
    if (budget < 2 * stage) budget = 2 * stage;
    int nst = (int)(budget / stage);
    nst = nst > TC_MAX_NST ? TC_MAX_NST : nst;
    const size_t lds = nst * stage;
    auto kern = k_tokc<WANT_DA, BC>;
    {
        hipError_t e = allow_full_lds(reinterpret_cast<const void *>(kern), 1 + (WANT_DA ? 2 : 0) + (BC == 256 ? 1 : 0));
        if (e != hipSuccess) return e;
    }
    const dim3 grid((unsigned)((C + BC - 1) / BC), (unsigned)h.n_adapters, (unsigned)n_split);
    hipLaunchKernelGGL(kern, grid, dim3(2 * BC), lds, st, mv, S, C, zt, zero, n_split > 1 ? part : nullptr, r16_total, nst, NoGroup{0});
    return hipGetLastError();
}

hipError_t launch_tokc_group_dA(const GroupView &gv, const MetaHeader &hv, const void *x, int64_t C, const void *zero,
                                float *part, int n_split, int n_active_adapters, hipStream_t st)
{
    if (hv.n_adapters == 0) return hipSuccess;
    if (gv.n_proj < 2 || gv.n_proj > kMaxGroup || gv.max_r16 > PLORA_MAX_RANK || hv.max_r16 != gv.max_r16) return hipErrorInvalidValue;
    int bc = 128;
    if (tokc_plan(hv, C, n_active_adapters, &bc) != n_split || bc != 128) return hipErrorInvalidValue;
    constexpr int BC = 128;
    const size_t stage = (size_t)TC_BT * BC * 2 + (size_t)(gv.max_r16 > 0 ? gv.max_r16 : 16) * TC_BT * 2;
    size_t budget = (size_t)TC_LDS_BYTES * BC / 256;
    if (budget < 2 * stage) budget = 2 * stage;
    int nst = (int)(budget / stage);
    nst = nst > TC_MAX_NST ? TC_MAX_NST : nst;
    auto kern = k_tokc<true, BC, true>;
    {
        hipError_t e = allow_full_lds(reinterpret_cast<const void *>(kern), 8);
        if (e != hipSuccess) return e;
    }
    const dim3 grid((unsigned)((C + BC - 1) / BC), (unsigned)hv.n_adapters, (unsigned)n_split);
    hipLaunchKernelGGL(kern, grid, dim3(2 * BC), nst * stage, st, gv.mv[0], static_cast<const uint16_t *>(x), (int)C,
                       static_cast<const uint16_t *>(nullptr), static_cast<const uint16_t *>(zero), n_split > 1 ? part : nullptr,
                       gv.r16_total, nst, gv);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || n_split <= 1) return e;
    hipLaunchKernelGGL(k_tokc_finish_group, dim3((unsigned)((C + 255) / 256), (unsigned)gv.r16_total), dim3(256), 0, st, gv, part,
                       (int)C, n_split);
    return hipGetLastError();
}

hipError_t launch_tokcontract_bf16(const MetaView &mv, const MetaHeader &h, bool want_dA, const void *S,
                                   int64_t C, const void *zt, const void *zero, float *part, int n_split,
                                   int r16_total, int n_active_adapters, hipStream_t st)
{
    if (h.n_adapters == 0) return hipSuccess;
    int bc = 256;
    if (tokc_plan(h, C, n_active_adapters, &bc) != n_split) return hipErrorInvalidValue;   // the caller sized `part` from the same plan
    const uint16_t *s16 = static_cast<const uint16_t *>(S), *z16 = static_cast<const uint16_t *>(zt);
    const uint16_t *zero16 = static_cast<const uint16_t *>(zero);
    hipError_t e;
#define PL_TOKC(DA_, BC_) launch_tokc<DA_, BC_>(mv, h, s16, (int)C, z16, zero16, part, n_split, r16_total, st)
    if (want_dA) e = bc == 256 ? PL_TOKC(true, 256) : PL_TOKC(true, 128);
    else e = bc == 256 ? PL_TOKC(false, 256) : PL_TOKC(false, 128);
#undef PL_TOKC
    if (e != hipSuccess || n_split <= 1) return e;
    const dim3 g2((unsigned)((C + 255) / 256), (unsigned)r16_total);
    if (want_dA) hipLaunchKernelGGL(k_tokc_finish<true>, g2, dim3(256), 0, st, mv, part, (int)C, n_split, r16_total);
    else hipLaunchKernelGGL(k_tokc_finish<false>, g2, dim3(256), 0, st, mv, part, (int)C, n_split, r16_total);
    return hipGetLastError();
}

}  // namespace plora
