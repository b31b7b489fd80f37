// Device-side core of the attention kernels (attn.hip).
//
// Bidirectional attention of a group of query rows against the K/V cache plus,
// in the decode step, the fresh K/V of the rows' own draft.
//
// Work is organised per "unit" (a draft in the step, a sequence in the prefill):
// the rows of a unit all see the same keys.  A workgroup takes QT 16-row tiles
// of one unit and one head; its NW waves split the 32-key tiles, keep a running
// (max, sum, O) per row and are merged through LDS in a fixed order.
// Scores are computed transposed, S^T = K Q^T, so that after the MFMA every
// lane holds scores of ONE query row (lane & 15): the softmax statistics are
// lane-local plus two cross-lane exchanges, and the probabilities are already
// in the register order the second MFMA (O^T = V^T P^T) wants, because V^T is
// stored with the 32 keys of a tile permuted to match (see gemm.hip, EpiQKV).
//
// Visibility (ODB-dLLM Sec. 4.2): cached keys of the block itself are skipped,
// a draft's rows see only that draft's fresh keys; there is no causal mask.
#pragma once
#include "model.h"

namespace odb {

template <int DH>
__device__ inline void store_out_tile(const AttnArgs &a, int mt, int hd, int dt16, int lane, f32x4 v) {
    const int mi = lane & 15, g = lane >> 4;
    const int kt = hd * (DH / 32) + (dt16 >> 1);
    u16 *dst = a.out + ((size_t)kt * a.mt_total + mt) * kTileElems + (((dt16 & 1) * 2 + (g >> 1)) * 16 + mi) * 8 +
               (g & 1) * 4;
    uint2 p;
    p.x = pack2(v[0], v[1]);
    p.y = pack2(v[2], v[3]);
    *reinterpret_cast<uint2 *>(dst) = p;
}

// Scores of one 32-key tile (K fragments kf) against QT row tiles, online-softmax update of the running
// (max, sum) and the rescaling of O that goes with it; returns the probabilities as operand fragments pf.
// MASK: some keys of the tile may be invisible, as KeyVis says.  kKeysCached: cache positions key0 .. key0+31,
// those past L or inside the block are masked; kKeysFresh: fresh keys of the rows' own unit, those from fresh_n
// on are masked; kKeysShared: fresh keys of block_0 of the sequence, visible where bit key of `visible` is set;
// kKeysPooled: the fresh keys of all speculative blocks of the sequence, m per block one after the other - a
// row sees those of its own block only (block of row r of the pooled unit = r / m), the block-diagonal mask of
// the decoded-share stage.
// The running references mrun are in log2 units (raw score * sc, sc = log2(e)/sqrt(dh) > 0).
constexpr float kAttnSlack = 8.0f;
constexpr int kKeysCached = 0, kKeysFresh = 1, kKeysShared = 2, kKeysPooled = 3;
// What attn_scores needs to know about key visibility (all wave-uniform):
//   mode; fresh_n: number of valid fresh keys (kKeysFresh, kKeysPooled); visible: kKeysShared;
//   m, row0 (kKeysPooled): keys per block, first row of the tile inside the pooled unit.
// POOL: the kKeysShared / kKeysPooled modes can occur (decoded-share step only; compiled out otherwise).
struct KeyVis {
    int fresh_n;
    unsigned long long visible;
    int m, row0;
};
template <int DH, int QT, bool MASK, bool POOL = false>
__device__ __forceinline__ void attn_scores(const AttnArgs &a, float sc, int key0, int mode, const KeyVis &kv,
                                            const frag_t (&kf)[2][DH / 32], const frag_t (&q)[QT][DH / 32],
                                            f32x4 (&o)[QT][DH / 16], float (&mrun)[QT], float (&lrun)[QT],
                                            frag_t (&pf)[QT], int lane) {
    constexpr int DT32 = DH / 32, DT16 = DH / 16;
    const int g = lane >> 4;
    bool ok[2][4];
    if (MASK) {
        if (POOL && mode == kKeysPooled) {
            // a row sees the keys [blk * m, blk * m + m) of its own block, blk = row / m (QT == 1 in this mode)
            const int lo = (kv.row0 + (lane & 15)) / kv.m * kv.m, hi = lo + kv.m < kv.fresh_n ? lo + kv.m : kv.fresh_n;
#pragma unroll
            for (int s = 0; s < 2; s++)
#pragma unroll
                for (int rr = 0; rr < 4; rr++) {
                    int key = key0 + s * 16 + 4 * g + rr;
                    ok[s][rr] = key >= lo && key < hi;
                }
        } else if (POOL && mode == kKeysShared) {
#pragma unroll
            for (int s = 0; s < 2; s++)
#pragma unroll
                for (int rr = 0; rr < 4; rr++) {
                    int key = key0 + s * 16 + 4 * g + rr;
                    ok[s][rr] = key < 64 && ((kv.visible >> key) & 1ull) != 0;
                }
        } else {
#pragma unroll
            for (int s = 0; s < 2; s++)
#pragma unroll
                for (int rr = 0; rr < 4; rr++) {
                    int key = key0 + s * 16 + 4 * g + rr;
                    ok[s][rr] = mode == kKeysCached ? (key < a.L && !(key >= a.blk_lo && key < a.blk_hi)) : key < kv.fresh_n;
                }
        }
    }
#pragma unroll
    for (int t = 0; t < QT; t++) {
        f32x4 st[2];
#pragma unroll
        for (int s = 0; s < 2; s++) {
            st[s] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int dt = 0; dt < DT32; dt++) st[s] = mfma16(kf[s][dt], q[t][dt], st[s]);
        }
        float tm = -INFINITY;
#pragma unroll
        for (int s = 0; s < 2; s++)
#pragma unroll
            for (int rr = 0; rr < 4; rr++) {
                if (MASK) st[s][rr] = ok[s][rr] ? st[s][rr] : -INFINITY;
                tm = fmaxf(tm, st[s][rr]);
            }
        // The reference mrun[t] of a row only has to be common to the four lanes that hold the row and to
        // keep exp2 in range; it need not be the exact running maximum.  It is raised (a cross-lane
        // maximum, a rescaling of O and of the running sum) only when some score of the wave exceeds its
        // row's reference by more than 2^kAttnSlack - after the first tiles that is rare, and then the
        // common path has no cross-lane exchange at all.  Probabilities stay below 2^kAttnSlack (binary16 holds them).
        if (__any(tm * sc > mrun[t] + kAttnSlack)) {
            tm = fmaxf(tm, __shfl_xor(tm, 16));
            tm = fmaxf(tm, __shfl_xor(tm, 32));
            const float mnew = fmaxf(mrun[t], tm * sc);
            const float alpha = __builtin_amdgcn_exp2f(mrun[t] - (mnew == -INFINITY ? 0.f : mnew));
            lrun[t] *= alpha;
#pragma unroll
            for (int dt = 0; dt < DT16; dt++) o[t][dt] *= alpha;
            mrun[t] = mnew;
        }
        const float mref = mrun[t] == -INFINITY ? 0.f : mrun[t];
        float p[2][4], ps = 0.f;
#pragma unroll
        for (int s = 0; s < 2; s++)
#pragma unroll
            for (int rr = 0; rr < 4; rr++) {
                p[s][rr] = __builtin_amdgcn_exp2f(__builtin_fmaf(st[s][rr], sc, -mref));
                ps += p[s][rr];
            }
        lrun[t] += ps;
        pf[t].w[0] = pack2_inrange(p[0][0], p[0][1]);
        pf[t].w[1] = pack2_inrange(p[0][2], p[0][3]);
        pf[t].w[2] = pack2_inrange(p[1][0], p[1][1]);
        pf[t].w[3] = pack2_inrange(p[1][2], p[1][3]);
    }
}

// Scores of one 32-key tile: st[t][s] = K_s Q_t^T (s: the two 16-key halves of the tile)
template <int DH, int QT>
__device__ __forceinline__ void attn_qk(const frag_t (&kf)[2][DH / 32], const frag_t (&q)[QT][DH / 32], f32x4 (&st)[QT][2]) {
#pragma unroll
    for (int t = 0; t < QT; t++)
#pragma unroll
        for (int s = 0; s < 2; s++) {
            st[t][s] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int dt = 0; dt < DH / 32; dt++) st[t][s] = mfma16(kf[s][dt], q[t][dt], st[t][s]);
        }
}

// The softmax half of attn_scores on scores st that are already there (cached keys only), followed by the score
// MFMAs of the NEXT tile (K fragments kf_next -> st_next).  masked (wave-uniform): some keys of the tile are
// invisible; their scores are set to -inf in a branch of its own, so that the common tile pays nothing for masks.
// The rare raise of a row's reference (see attn_scores) is taken for all row tiles in one branch.
template <int DH, int QT>
__device__ __forceinline__ void attn_softmax_qk(const AttnArgs &a, float sc, int key0, bool masked, f32x4 (&st)[QT][2],
                                                const frag_t (&kf_next)[2][DH / 32], const frag_t (&q)[QT][DH / 32],
                                                f32x4 (&st_next)[QT][2], f32x4 (&o)[QT][DH / 16], float (&mrun)[QT],
                                                float (&lrun)[QT], frag_t (&pf)[QT], int lane) {
    constexpr int DT16 = DH / 16;
    if (masked) {
        const int g = lane >> 4;
#pragma unroll
        for (int s = 0; s < 2; s++)
#pragma unroll
            for (int rr = 0; rr < 4; rr++) {
                const int key = key0 + s * 16 + 4 * g + rr;
                const bool ok = key < a.L && !(key >= a.blk_lo && key < a.blk_hi);
#pragma unroll
                for (int t = 0; t < QT; t++) st[t][s][rr] = ok ? st[t][s][rr] : -INFINITY;
            }
    }
    float tm[QT];
    bool raise = false;
#pragma unroll
    for (int t = 0; t < QT; t++) {
        tm[t] = fmaxf(fmaxf(fmaxf(st[t][0][0], st[t][0][1]), fmaxf(st[t][0][2], st[t][0][3])),
                      fmaxf(fmaxf(st[t][1][0], st[t][1][1]), fmaxf(st[t][1][2], st[t][1][3])));
        raise = raise || tm[t] * sc > mrun[t] + kAttnSlack;
    }
    if (__any(raise)) {
#pragma unroll
        for (int t = 0; t < QT; t++) {
            if (__any(tm[t] * sc > mrun[t] + kAttnSlack)) {
                float x = fmaxf(tm[t], __shfl_xor(tm[t], 16));
                x = fmaxf(x, __shfl_xor(x, 32));
                const float mnew = fmaxf(mrun[t], x * sc);
                const float alpha = __builtin_amdgcn_exp2f(mrun[t] - (mnew == -INFINITY ? 0.f : mnew));
                lrun[t] *= alpha;
#pragma unroll
                for (int dt = 0; dt < DT16; dt++) o[t][dt] *= alpha;
                mrun[t] = mnew;
            }
        }
    }
#pragma unroll
    for (int t = 0; t < QT; t++) {
        const float mref = mrun[t] == -INFINITY ? 0.f : mrun[t];
        float p[2][4], ps = 0.f;
#pragma unroll
        for (int s = 0; s < 2; s++)
#pragma unroll
            for (int rr = 0; rr < 4; rr++) {
                p[s][rr] = __builtin_amdgcn_exp2f(__builtin_fmaf(st[t][s][rr], sc, -mref));
                ps += p[s][rr];
            }
        lrun[t] += ps;
        pf[t].w[0] = pack2_inrange(p[0][0], p[0][1]);
        pf[t].w[1] = pack2_inrange(p[0][2], p[0][3]);
        pf[t].w[2] = pack2_inrange(p[1][0], p[1][1]);
        pf[t].w[3] = pack2_inrange(p[1][2], p[1][3]);
    }
    attn_qk<DH, QT>(kf_next, q, st_next);
}

// O^T += V^T P^T for QT row tiles
template <int DH, int QT>
__device__ __forceinline__ void attn_pv(const frag_t (&vf)[DH / 16], const frag_t (&pf)[QT], f32x4 (&o)[QT][DH / 16]) {
#pragma unroll
    for (int t = 0; t < QT; t++)
#pragma unroll
        for (int dt = 0; dt < DH / 16; dt++) o[t][dt] = mfma16(vf[dt], pf[t], o[t][dt]);
}

// true if some key of the 32-key tile at key0 may be invisible (see attn_scores)
__device__ __forceinline__ bool attn_tile_masked(const AttnArgs &a, int key0, int mode, int fresh_n) {
    return mode == kKeysCached ? (key0 + 32 > a.L || (key0 < a.blk_hi && key0 + 32 > a.blk_lo))
         : mode == kKeysFresh ? key0 + 32 > fresh_n : true;
}

// One 32-key tile (K fragments kf, V^T fragments vf) against QT row tiles: scores, online softmax, O update.
template <int DH, int QT, bool POOL = false>
__device__ __forceinline__ void attn_tile_update(const AttnArgs &a, float sc, int key0, int mode, const KeyVis &kv,
                                                 const frag_t (&kf)[2][DH / 32], const frag_t (&vf)[DH / 16],
                                                 const frag_t (&q)[QT][DH / 32], f32x4 (&o)[QT][DH / 16],
                                                 float (&mrun)[QT], float (&lrun)[QT], int lane) {
    frag_t pf[QT];
    if (attn_tile_masked(a, key0, mode, kv.fresh_n)) attn_scores<DH, QT, true, POOL>(a, sc, key0, mode, kv, kf, q, o, mrun, lrun, pf, lane);
    else attn_scores<DH, QT, false, POOL>(a, sc, key0, mode, kv, kf, q, o, mrun, lrun, pf, lane);
    attn_pv<DH, QT>(vf, pf, o);
}

template <int QT, int NW>
constexpr int attn_smem_bytes() { return NW * 4 * 1024 + 2 * NW * QT * 16 * 4; }

// One work item: QT row tiles (chunk `item` of the units' tiles) of head hd.  sc = log2(e)/sqrt(dh).
// SHARED (decoded-share step, QT = 1): item is the m-tile; tiles from a.split_tile on belong to the pooled
// speculative unit of a sequence (the rows of its speculative blocks one after the other), whose rows see the
// cache, the pooled fresh keys of their own block and block_0's fresh keys at the decoded positions.
template <int DH, int QT, int NW, bool SHARED = false>
__device__ __forceinline__ void attn_wg(const AttnArgs &a, float sc, int item, int hd, char *smem) {
    constexpr int DT32 = DH / 32, DT16 = DH / 16;
    constexpr int DC = DT16 < 4 ? DT16 : 4;          // channel tiles merged per pass through LDS
    static_assert(!SHARED || QT == 1, "the decoded-share step works on single row tiles");
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, mi = lane & 15, g = lane >> 4;
    const bool spec = SHARED && item >= a.split_tile;                     // a speculative unit's tile
    const int tpu = spec ? a.tiles_per_unit_b : a.tiles_per_unit;
    const int chunks = (tpu + QT - 1) / QT;
    const int item_u = spec ? item - a.split_tile : item;
    const int unit = item_u / chunks, tu0 = (item_u % chunks) * QT;
    const int seq = spec ? unit : unit / a.units_per_seq;              // one pooled speculative unit per sequence
    const int mt_base = (spec ? a.split_tile : 0) + unit * tpu;           // first m-tile of the unit
    f32x4 (*s_o)[DC][64] = reinterpret_cast<f32x4 (*)[DC][64]>(smem);
    float (*s_m)[QT][16] = reinterpret_cast<float (*)[QT][16]>(smem + NW * 4 * 1024);
    float (*s_l)[QT][16] = s_m + NW;

    frag_t q[QT][DT32];
#pragma unroll
    for (int t = 0; t < QT; t++) {
        int tu = tu0 + t < tpu ? tu0 + t : tpu - 1;
        int mt = mt_base + tu;
#pragma unroll
        for (int dt = 0; dt < DT32; dt++)
            q[t][dt] = ld_frag(a.q + (((size_t)hd * a.mt_total + mt) * DT32 + dt) * kTileElems + lane * 8);
    }
    f32x4 o[QT][DT16];
    float mrun[QT], lrun[QT];
#pragma unroll
    for (int t = 0; t < QT; t++) {
        mrun[t] = -INFINITY;
        lrun[t] = 0.f;
#pragma unroll
        for (int dt = 0; dt < DT16; dt++) o[t][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // visibility of the unit's own fresh keys and (speculative unit) of block_0's
    const int m_seq = spec ? (a.mcount[seq] > 0 ? a.mcount[seq] : 1) : 1;
    const int fresh_n = spec ? a.spec_blocks * a.mcount[seq] : a.fresh;
    const KeyVis kv{fresh_n, spec ? a.dmask[seq] : 0ull, m_seq, tu0 * 16};
    struct TileRef { const u16 *kp, *vp; int key0, mode; bool live; };
    auto load_tile = [&](const TileRef &r, frag_t (&kf)[2][DT32], frag_t (&vf)[DT16]) __attribute__((always_inline)) {
#pragma unroll
        for (int s = 0; s < 2; s++)
#pragma unroll
            for (int dt = 0; dt < DT32; dt++)
                kf[s][dt] = ld_frag(r.kp + (size_t)(s * DT32 + dt) * kTileElems + lane * 8);
#pragma unroll
        for (int dt = 0; dt < DT16; dt++) vf[dt] = ld_frag(r.vp + (size_t)dt * kTileElems + lane * 8);
    };
    auto compute_tile = [&](const TileRef &r, const frag_t (&kf)[2][DT32], const frag_t (&vf)[DT16])
                            __attribute__((always_inline)) {
        attn_tile_update<DH, QT, SHARED>(a, sc, r.key0, r.mode, kv, kf, vf, q, o, mrun, lrun, lane);
    };

    // This wave's tiles: the 32-key tiles of the cache (those wholly inside the block are dead), then the
    // unit's own fresh tiles, then (speculative units of the decoded-share step) block_0's fresh tiles, dealt
    // to the waves round-robin as one sequence.  The loads of tile i+1 are issued before tile i is computed.
    const int n32 = (a.L + 31) / 32;
    const u16 *kc = a.kc + seq * a.kc_seq_stride + hd * a.kc_head_stride;
    const u16 *vc = a.vc + seq * a.vc_seq_stride + hd * a.vc_head_stride;
    const u16 *kfr = spec ? a.kf_b + unit * a.kf_b_unit_stride + hd * a.kf_b_head_stride
                          : a.kf + unit * a.kf_unit_stride + hd * a.kf_head_stride;
    const u16 *vfr = spec ? a.vf_b + unit * a.vf_b_unit_stride + hd * a.vf_b_head_stride
                          : a.vf + unit * a.vf_unit_stride + hd * a.vf_head_stride;
    const u16 *ksh = a.kf + seq * a.kf_unit_stride + hd * a.kf_head_stride;      // block_0 of this sequence (spec only)
    const u16 *vsh = a.vf + seq * a.vf_unit_stride + hd * a.vf_head_stride;
    const int nf32 = fresh_n > 0 ? (fresh_n + 31) / 32 : 0;
    const int ns32 = spec ? (a.fresh + 31) / 32 : 0;
    const int n_all = n32 + nf32 + ns32;
    const int total = w < n_all ? (n_all - w + NW - 1) / NW : 0;
    auto get = [&](int i) __attribute__((always_inline)) {
        TileRef r;
        const int gi = w + i * NW;
        if (gi < n32) {
            r.kp = kc + (size_t)gi * 2 * DT32 * kTileElems;
            r.vp = vc + (size_t)gi * DT16 * kTileElems;
            r.key0 = gi * 32;
            r.mode = kKeysCached;
            r.live = !(gi * 32 >= a.blk_lo && gi * 32 + 32 <= a.blk_hi);
        } else if (gi < n32 + nf32) {
            const int T = gi - n32;
            r.kp = kfr + (size_t)T * 2 * DT32 * kTileElems;
            r.vp = vfr + (size_t)T * DT16 * kTileElems;
            r.key0 = T * 32;
            r.mode = spec ? kKeysPooled : kKeysFresh;
            r.live = true;
        } else {
            const int T = gi - n32 - nf32;
            r.kp = ksh + (size_t)T * 2 * DT32 * kTileElems;
            r.vp = vsh + (size_t)T * DT16 * kTileElems;
            r.key0 = T * 32;
            r.mode = kKeysShared;
            r.live = true;
        }
        return r;
    };
    if (total > 0) {
        frag_t kf_c[2][DT32], vf_c[DT16], kf_n[2][DT32], vf_n[DT16];
        TileRef cur = get(0);
        if (cur.live) load_tile(cur, kf_c, vf_c);
        for (int i = 0; i < total; i++) {
            TileRef nxt = cur;
            const bool more = i + 1 < total;
            if (more) {
                nxt = get(i + 1);
                if (nxt.live) load_tile(nxt, kf_n, vf_n);
            }
            if (cur.live) compute_tile(cur, kf_c, vf_c);
            if (more) {
                cur = nxt;
#pragma unroll
                for (int s = 0; s < 2; s++)
#pragma unroll
                    for (int dt = 0; dt < DT32; dt++) kf_c[s][dt] = kf_n[s][dt];
#pragma unroll
                for (int dt = 0; dt < DT16; dt++) vf_c[dt] = vf_n[dt];
            }
        }
    }

    // merge the waves
#pragma unroll
    for (int t = 0; t < QT; t++) {
        float l = lrun[t];
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        lrun[t] = l;
        if (g == 0) {
            s_m[w][t][mi] = mrun[t];
            s_l[w][t][mi] = l;
        }
    }
    __syncthreads();
#pragma unroll
    for (int t = 0; t < QT; t++) {
        float mall = -INFINITY;
#pragma unroll
        for (int x = 0; x < NW; x++) mall = fmaxf(mall, s_m[x][t][mi]);
        float ltot = 0.f, fown = 0.f;
#pragma unroll
        for (int x = 0; x < NW; x++) {
            float mx = s_m[x][t][mi];
            float f = mx == -INFINITY ? 0.f : exp2f(mx - mall);
            ltot += s_l[x][t][mi] * f;
            if (x == w) fown = f;
        }
        const int tu = tu0 + t;
        const int mt = mt_base + tu;
#pragma unroll
        for (int d0 = 0; d0 < DT16; d0 += DC) {
#pragma unroll
            for (int dt = 0; dt < DC; dt++) s_o[w][dt][lane] = o[t][d0 + dt] * fown;
            __syncthreads();
            if (tu < tpu) {
                for (int dt = w; dt < DC; dt += NW) {
                    f32x4 v = s_o[0][dt][lane];
#pragma unroll
                    for (int x = 1; x < NW; x++) v += s_o[x][dt][lane];
                    store_out_tile<DH>(a, mt, hd, d0 + dt, lane, v * (1.0f / ltot));
                }
            }
            __syncthreads();
        }
    }
}

}  // namespace odb
