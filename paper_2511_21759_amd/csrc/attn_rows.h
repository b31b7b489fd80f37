// Attention for many query rows per (sequence, head): the prefill and the long-block,
// many-draft decode step (see attn_core.h for the tile arithmetic and the layouts).
//
// A workgroup takes NW * QTW consecutive 16-row tiles of ONE sequence and one head; every wave owns
// QTW of them from start to finish, so nothing is merged across waves.  All waves walk over the
// same cached 32-key tiles, which are copied from global memory straight into an LDS ring
// (global_load ... lds, NS stages, NS - 1 tiles ahead) once per workgroup and read from there by
// every wave: a K/V tile fetched from L2 serves NW * QTW * 16 rows.  The ring is deep because a
// workgroup is usually the first on its XCD to touch its K/V: with 16 KiB per tile and a few
// microseconds of HBM latency, two tiles in flight bound the kernel at 1.7 us per tile (measured).  The fresh keys of a draft
// (decode step) are private to that draft's rows; each wave reads its own from global memory
// after the shared loop.  Visibility is as in attn_core.h.
#pragma once
#include <type_traits>
#include "attn_core.h"

namespace odb {

template <int DH, int NS>
constexpr int attn_rows_smem_bytes() { return NS * (2 * (DH / 32) + DH / 16) * 1024; }

// Requires tiles_per_unit % QTW == 0 when there are fresh keys (a wave's tiles then belong to one draft).
template <int DH, int NW, int QTW, int NS>
__global__ __launch_bounds__(64 * NW) void attn_rows_kernel(AttnArgs a, float sc) {
    constexpr int DT32 = DH / 32, DT16 = DH / 16;
    constexpr int FR = 2 * DT32 + DT16;              // 1 KiB fragments per 32-key tile: K then V^T
    constexpr int PER = (FR + NW - 1) / NW;          // fragments each wave copies per stage
    static_assert(FR % NW == 0, "every wave copies the same number of fragments");
    extern __shared__ __attribute__((aligned(16))) char smem[];
    typedef frag_t stage_t[FR][64];
    stage_t *ring = reinterpret_cast<stage_t *>(smem);

    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int tiles_per_seq = a.units_per_seq * a.tiles_per_unit;
    const int chunks = (tiles_per_seq + NW * QTW - 1) / (NW * QTW);
    // One-dimensional grid (gridDim.y == 1 although the heads are a multiple of 8): workgroup ids go round-robin over the XCDs, and
    // id = xcd + 8 * (item + items * (head / 8)) with head = xcd + 8 * (head / 8) keeps all row chunks of a head
    // (they read the same K/V) on one XCD, whose L2 then holds the K/V of its own heads only.
    int hd = blockIdx.y, item = blockIdx.x;
    if (gridDim.y == 1 && (a.H & 7) == 0) {
        const int items = gridDim.x / a.H, j = blockIdx.x >> 3;
        hd = (blockIdx.x & 7) + 8 * (j / items);
        item = j % items;
    }
    const int seq = item / chunks;
    const int ts0 = (item % chunks) * (NW * QTW) + w * QTW;      // this wave's first tile within the sequence
    const bool wave_live = ts0 < tiles_per_seq;
    const int unit = seq * a.units_per_seq + (wave_live ? ts0 : tiles_per_seq - 1) / a.tiles_per_unit;

    frag_t q[QTW][DT32];
#pragma unroll
    for (int t = 0; t < QTW; t++) {
        const int ts = ts0 + t < tiles_per_seq ? ts0 + t : tiles_per_seq - 1;
        const int mt = seq * tiles_per_seq + ts;
#pragma unroll
        for (int dt = 0; dt < DT32; dt++)
            q[t][dt] = ld_frag(a.q + (((size_t)hd * a.mt_total + mt) * DT32 + dt) * kTileElems + lane * 8);
    }
    f32x4 o[QTW][DT16];
    float mrun[QTW], lrun[QTW];
#pragma unroll
    for (int t = 0; t < QTW; t++) {
        mrun[t] = -INFINITY;
        lrun[t] = 0.f;
#pragma unroll
        for (int dt = 0; dt < DT16; dt++) o[t][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // live cached tiles: all 32-key tiles of the sequence but those wholly inside the block
    const int n32 = (a.L + 31) / 32;
    const int d_lo = (a.blk_lo + 31) / 32, d_hi = a.blk_hi / 32;
    const int dead = d_hi > d_lo ? d_hi - d_lo : 0;
    const int n_live = n32 - dead;
    auto tile_of = [&](int i) { return dead > 0 && i >= d_lo ? i + dead : i; };
    const u16 *kc = a.kc + seq * a.kc_seq_stride + hd * a.kc_head_stride + lane * 8;
    const u16 *vc = a.vc + seq * a.vc_seq_stride + hd * a.vc_head_stride + lane * 8;
    auto issue = [&](int slot, int i) __attribute__((always_inline)) {
        const int T = tile_of(i);
#pragma unroll
        for (int u = 0; u < PER; u++) {
            const int f = w + u * NW;
            const u16 *src = f < 2 * DT32 ? kc + ((size_t)T * 2 * DT32 + f) * kTileElems
                                          : vc + ((size_t)T * DT16 + (f - 2 * DT32)) * kTileElems;
            __builtin_amdgcn_global_load_lds(reinterpret_cast<const void *>(src),
                                             (__attribute__((address_space(3))) void *)(&ring[slot][f][0]), 16, 0, 0);
        }
    };

    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");        // q has arrived: the counted waits below see only the ring
    static_assert(PER * (NS - 2) <= 28 && (PER * (NS - 2) <= 16 || PER % 2 == 0), "wait_vmcnt covers these counts");
    static_assert(NS >= 4, "tiles being read while the next is requested");
    // Copies of tiles 0 .. NS-2 are requested up front; in iteration i tile i+NS-1 follows, into the slot of
    // tile i-1.  A wave enters iteration i with the scores of tile i in registers and the K fragments of
    // tile i+1 read; it fetches V of tile i, runs the softmax of tile i and the score MFMAs of tile i+1,
    // fetches K of tile i+2 and issues P*V of tile i (the reads complete under it).  Past the last tile the
    // "next" tiles are the last one again; what is computed from them is never used.
    // (MFMAs and vector instructions hardly overlap on this chip - a wave that interleaves 16 MFMAs with 48
    // independent fmas takes 85 % of the sum of the two alone, two waves of a SIMD that run one kind each take
    // 80 % - so what the softmax costs is its instruction count: masks are applied on masked tiles only.)
    frag_t kf[2][DT32], vf[DT16], pf[QTW];
    const KeyVis kv{a.fresh, 0ull, 1, 0};
    auto read_k = [&](int i) __attribute__((always_inline)) {
        const stage_t &st = ring[i % NS];
#pragma unroll
        for (int s = 0; s < 2; s++)
#pragma unroll
            for (int dt = 0; dt < DT32; dt++) kf[s][dt] = st[s * DT32 + dt][lane];
    };
    // waits until this wave's copies of tiles 0 .. upto have landed (later requests may still be in flight)
    auto landed = [&](int upto, int requested) __attribute__((always_inline)) {
        const int last = requested < n_live - 1 ? requested : n_live - 1;
        wait_vmcnt(last > upto ? PER * (last - upto) : 0);
    };
#pragma unroll
    for (int j = 0; j < NS - 1; j++)
        if (j < n_live) issue(j, j);
    f32x4 sc_t[2][QTW][2];
    if (n_live > 0) {
        landed(n_live > 1 ? 1 : 0, NS - 2);
        __builtin_amdgcn_s_barrier();
        if (wave_live) {
            read_k(0);
            attn_qk<DH, QTW>(kf, q, sc_t[0]);
            read_k(n_live > 1 ? 1 : 0);
        }
    }
    auto iter = [&](auto P, int i) __attribute__((always_inline)) {
        constexpr int p = decltype(P)::value;
        const int i2 = i + 2 < n_live ? i + 2 : n_live - 1;
        landed(i2, i + NS - 2);
        __builtin_amdgcn_s_barrier();
        // tile i+2 is visible to every wave, and every wave is done with the slot of tile i-1
        if (i + NS - 1 < n_live) issue((i + NS - 1) % NS, i + NS - 1);
        if (wave_live) {
            const stage_t &st = ring[i % NS];
#pragma unroll
            for (int dt = 0; dt < DT16; dt++) vf[dt] = st[2 * DT32 + dt][lane];
            const int key0 = tile_of(i) * 32;
            attn_softmax_qk<DH, QTW>(a, sc, key0, attn_tile_masked(a, key0, kKeysCached, 0), sc_t[p], kf, q, sc_t[1 - p], o,
                                     mrun, lrun, pf, lane);
            read_k(i2);
            attn_pv<DH, QTW>(vf, pf, o);
        }
    };
    {
        int i = 0;
        for (; i + 1 < n_live; i += 2) {
            iter(std::integral_constant<int, 0>{}, i);
            iter(std::integral_constant<int, 1>{}, i + 1);
        }
        if (i < n_live) iter(std::integral_constant<int, 0>{}, i);
    }
    if (!wave_live) return;

    // fresh keys of this wave's draft
    const int nf32 = a.fresh > 0 ? (a.fresh + 31) / 32 : 0;
    const u16 *kfr = a.kf + unit * a.kf_unit_stride + hd * a.kf_head_stride + lane * 8;
    const u16 *vfr = a.vf + unit * a.vf_unit_stride + hd * a.vf_head_stride + lane * 8;
    for (int T = 0; T < nf32; T++) {
#pragma unroll
        for (int s = 0; s < 2; s++)
#pragma unroll
            for (int dt = 0; dt < DT32; dt++) kf[s][dt] = ld_frag(kfr + ((size_t)T * 2 * DT32 + s * DT32 + dt) * kTileElems);
#pragma unroll
        for (int dt = 0; dt < DT16; dt++) vf[dt] = ld_frag(vfr + ((size_t)T * DT16 + dt) * kTileElems);
        attn_scores<DH, QTW, true>(a, sc, T * 32, kKeysFresh, kv, kf, q, o, mrun, lrun, pf, lane);
        attn_pv<DH, QTW>(vf, pf, o);
    }

#pragma unroll
    for (int t = 0; t < QTW; t++) {
        if (ts0 + t < tiles_per_seq) {
            float l = lrun[t];
            l += __shfl_xor(l, 16);
            l += __shfl_xor(l, 32);
            const float inv = 1.0f / l;
            const int mt = seq * tiles_per_seq + ts0 + t;
#pragma unroll
            for (int dt = 0; dt < DT16; dt++) store_out_tile<DH>(a, mt, hd, dt, lane, o[t][dt] * inv);
        }
    }
}

}  // namespace odb
