// binary16 MFMA GEMM  C[M,N] = A[M,K] * W[N,K]^T  for 33 rows and more (the multi-draft step,
// the prefill, the long-context step).  Same operand layouts and epilogues as gemm_core.h.
//
// A workgroup computes a 128-row block x (8*NGW n-tiles) x one slice of K.  Its eight waves split
// the n-tiles; the 128 x 32 slab of A that a k-step needs is shared through LDS: every wave fetches
// one of the slab's eight 16-row tiles PF steps ahead into registers and drops it into a ring of LDS
// slots when its turn comes, so A is read from L2 once per workgroup while every wave streams its
// own weight tiles from HBM straight into MFMA operand registers.  With a K split (grid.x =
// n-blocks x KS) the partial sums go to an fp32 workspace in MFMA fragment order and
// tile_epilogue_kernel adds them in a fixed order and runs the epilogue.
#pragma once
#include <type_traits>
#include "gemm_core.h"

namespace odb {

struct TileArgs {
    const u16 *A, *W;
    int KT, MT_total, NT;
    int n_blocks, KS;          // grid.x = n_blocks * KS, blockIdx.x = n-block * KS + k-slice
    float *partial;            // [KS][MT_total][NT][256] fp32 (KS > 1)
    const float *ssq;          // fused RMSNorm of the input rows (see GemmArgs)
    int n_ssq;
    float eps, inv_d;
};

// LM-head statistics for the tile kernel: one partial (max, sum exp, argmax) per row and n-block
struct TileLMStats {
    static constexpr bool kRowStats = true;
    float *stats;
    int n_part;
};

template <class Epi> struct is_row_stats { static constexpr bool value = false; };
template <> struct is_row_stats<TileLMStats> { static constexpr bool value = true; };


__device__ __forceinline__ void merge_stat(float &m, float &s, int &a, float om, float os, int oa) {
    float nm = fmaxf(m, om);
    s = s * (m == nm ? 1.f : __expf(m - nm)) + os * (om == nm ? 1.f : __expf(om - nm));
    a = m > om ? a : (om > m ? oa : (a < oa ? a : oa));
    m = nm;
}

// NW waves per workgroup, each NGW n-tiles wide: the workgroup covers NW*NGW n-tiles.  One k-tile per barrier; every
// wave keeps PF k-tiles (its share of the A slab and its own weight tiles) in flight.  The A slab goes through a ring
// of kTileSlots LDS slots (a slot is rewritten four barriers after its last reader asked for it).
constexpr int kTileSlots = 4;
constexpr int tile_smem_bytes() { return kTileSlots * 8 * 1024 + 8 * 1024 + 128 * 4; }

// SW: the weight tiles are read by one workgroup only (a single block of rows), so they are loaded non-temporally.
template <int NW, int NGW, int PF, class Epi, bool SW = false>
__global__ __launch_bounds__(64 * NW) void gemm_tile_kernel(TileArgs g, Epi epi) {
    constexpr int AW = 8 / NW;                 // A tiles (per k-tile) of the slab each wave fetches
    static_assert(NW == 4 || NW == 8, "waves per workgroup");
    static_assert(PF % kTileSlots == 0, "ring slots and register buffers are indexed by the unrolled step");
    __shared__ __attribute__((aligned(16))) char smem[tile_smem_bytes()];
    frag_t (*a_lds)[8][64] = reinterpret_cast<frag_t (*)[8][64]>(smem);                    // [slots][8 m-tiles][64 lanes]
    f32x4 (*scr)[64] = reinterpret_cast<f32x4 (*)[64]>(smem + kTileSlots * 8 * 1024);      // [8 waves][64]
    float *s_rstd = reinterpret_cast<float *>(smem + kTileSlots * 8 * 1024 + 8 * 1024);

    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    // (k-slice in the low bits of the id: workgroup ids go round-robin over the XCDs, so an XCD's workgroups then share
    // one or two k-slices of A instead of reading all of it into every L2; 22.0 -> 21.6 us at 128 rows)
    const int nb = blockIdx.x / g.KS, ks = blockIdx.x % g.KS;
    const int mt0 = blockIdx.y * 8;
    const int k_lo = (int)((unsigned)ks * (unsigned)g.KT / (unsigned)g.KS), k_hi = (int)((unsigned)(ks + 1) * (unsigned)g.KT / (unsigned)g.KS);
    const int nk = k_hi - k_lo;                 // k-tiles of this slice
    const int nt0 = (nb * NW + w) * NGW;

    const u16 *wp[NGW];
#pragma unroll
    for (int j = 0; j < NGW; j++) {
        int nt = nt0 + j < g.NT ? nt0 + j : g.NT - 1;
        wp[j] = g.W + ((size_t)nt * g.KT + k_lo) * kTileElems + lane * 8;
    }
    const u16 *ap[AW];                                                             // the A tiles this wave fetches
#pragma unroll
    for (int i = 0; i < AW; i++) {
        int mt = mt0 + w * AW + i < g.MT_total ? mt0 + w * AW + i : g.MT_total - 1;
        ap[i] = g.A + ((size_t)k_lo * g.MT_total + mt) * kTileElems + lane * 8;
    }
    const size_t a_step = (size_t)g.MT_total * kTileElems;

    // row scales of the fused RMSNorm: 128 / NW rows per wave; a row's partial sums (up to 256) are one
    // 16-byte load per lane, and the loads of 16 rows are issued back to back
    if (g.ssq) {
        const int si = 4 * lane;
#pragma unroll
        for (int r0 = 0; r0 < 16 * AW; r0 += 16) {
            f32x4 sv[16];
            float q[16];
#pragma unroll
            for (int r = 0; r < 16; r++) {
                int row = (mt0 + w * AW) * 16 + r0 + r;
                row = row < g.MT_total * 16 ? row : g.MT_total * 16 - 1;
                const float *p = g.ssq + (size_t)row * g.n_ssq;
                q[r] = 0.f;
                for (int i0 = 256; i0 < g.n_ssq; i0 += 256) {       // rows wider than 4096 only
                    const int i = i0 + si, ic = i < g.n_ssq - 4 ? i : g.n_ssq - 4;
                    f32x4 v = *reinterpret_cast<const f32x4 *>(p + ic);
                    q[r] += i < g.n_ssq ? (v[0] + v[1]) + (v[2] + v[3]) : 0.f;
                }
                sv[r] = *reinterpret_cast<const f32x4 *>(p + (si < g.n_ssq - 4 ? si : g.n_ssq - 4));
            }
#pragma unroll
            for (int r = 0; r < 16; r++) {
                float t = q[r] + (si < g.n_ssq ? (sv[r][0] + sv[r][1]) + (sv[r][2] + sv[r][3]) : 0.f);
#pragma unroll
                for (int o = 32; o > 0; o >>= 1) t += __shfl_xor(t, o);
                if (lane == 0) s_rstd[w * 16 * AW + r0 + r] = 1.0f / sqrtf(t * g.inv_d + g.eps);
            }
        }
    } else if (lane < 16 * AW) {
        s_rstd[w * 16 * AW + lane] = 1.0f;
    }

    f32x4 acc[8][NGW];
#pragma unroll
    for (int m = 0; m < 8; m++)
#pragma unroll
        for (int j = 0; j < NGW; j++) acc[m][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Loads past the end of the slice fetch its last tile again and are never used: the refills of the main loop
    // are unconditional, so the order of the outstanding loads is fixed and every wait counts exactly.
    frag_t wr[PF][NGW], ar[PF][AW];
    auto load_step = [&](int slot, int c) __attribute__((always_inline)) {
        const int k = c < nk ? c : nk - 1;
#pragma unroll
        for (int i = 0; i < AW; i++) ar[slot][i] = ld_frag(ap[i] + k * a_step);
#pragma unroll
        for (int j = 0; j < NGW; j++)
            wr[slot][j] = SW ? ld_frag_stream(wp[j] + (size_t)k * kTileElems) : ld_frag(wp[j] + (size_t)k * kTileElems);
    };
#pragma unroll
    for (int s = 0; s < PF; s++) load_step(s, s);

    // PIPE (up to two n-tiles per wave): step c stores the slab of step c+1, and after the barrier reads it into a second
    // set of registers while the MFMAs of step c run on the set read one step earlier.  Wider waves have no registers
    // for the second set: they store, wait and read the slab of step c itself.
    constexpr bool PIPE = NGW <= 2;
    frag_t a[PIPE ? 2 : 1][8];
    if constexpr (PIPE) {
#pragma unroll
        for (int i = 0; i < AW; i++) a_lds[0][w * AW + i][lane] = ar[0][i];
        __syncthreads();
#pragma unroll
        for (int m = 0; m < 8; m++) a[0][m] = a_lds[0][m][lane];
    }
    auto step = [&](int s, int c) __attribute__((always_inline)) {
        constexpr int nxt = PIPE ? 1 : 0;
#pragma unroll
        for (int i = 0; i < AW; i++) a_lds[(s + nxt) % kTileSlots][w * AW + i][lane] = ar[(s + nxt) % PF][i];
        __syncthreads();
#pragma unroll
        for (int m = 0; m < 8; m++) a[(s + nxt) & nxt][m] = a_lds[(s + nxt) % kTileSlots][m][lane];
#pragma unroll
        for (int m = 0; m < 8; m++)
#pragma unroll
            for (int j = 0; j < NGW; j++) acc[m][j] = mfma16(wr[s][j], a[s & nxt][m], acc[m][j]);
        load_step(s, c + PF);
    };
    int cb = 0;
    for (; cb + PF <= nk; cb += PF) {
#pragma unroll
        for (int s = 0; s < PF; s++) step(s, cb + s);
    }
    {
        const int rest = nk - cb;                // uniform over the workgroup
#pragma unroll
        for (int s = 0; s < PF - 1; s++)
            if (s < rest) step(s, cb + s);
    }
    __syncthreads();

    if (g.KS > 1) {
        // partial sums in fragment order; tile_epilogue_kernel finishes the job
#pragma unroll
        for (int m = 0; m < 8; m++)
#pragma unroll
            for (int j = 0; j < NGW; j++) {
                const int mt = mt0 + m, nt = nt0 + j;
                if (mt < g.MT_total && nt < g.NT) {
                    size_t tile = ((size_t)ks * g.MT_total + mt) * g.NT + nt;
                    *reinterpret_cast<f32x4 *>(g.partial + tile * 256 + lane * 4) = acc[m][j];
                }
            }
        return;
    }

    if constexpr (is_row_stats<Epi>::value) {
        // softmax statistics per row over this workgroup's n-tiles: lane-local, across the four lane
        // groups, across the wave's NGW tiles, then across the eight waves through LDS
        float *st_m = reinterpret_cast<float *>(smem);               // the A slots are free now: [NW waves][128 rows]
        float *st_s = st_m + NW * 128;
        int *st_a = reinterpret_cast<int *>(st_s + NW * 128);
        const int mi = lane & 15, gq = lane >> 4;
#pragma unroll
        for (int m = 0; m < 8; m++) {
            float rm = -INFINITY, rs = 0.f;
            int ra = 0x7fffffff;
#pragma unroll
            for (int j = 0; j < NGW; j++) {
                if (nt0 + j < g.NT) {
                    f32x4 c = acc[m][j] * s_rstd[m * 16 + mi];
                    float cm = c[0];
                    int ca = (nt0 + j) * 16 + 4 * gq;
#pragma unroll
                    for (int r = 1; r < 4; r++)
                        if (c[r] > cm) { cm = c[r]; ca = (nt0 + j) * 16 + 4 * gq + r; }
                    float cs = 0.f;
#pragma unroll
                    for (int r = 0; r < 4; r++) cs += __expf(c[r] - cm);
                    merge_stat(rm, rs, ra, cm, cs, ca);
                }
            }
#pragma unroll
            for (int o = 16; o <= 32; o <<= 1) {
                float om = __shfl_xor(rm, o), os = __shfl_xor(rs, o);
                int oa = __shfl_xor(ra, o);
                merge_stat(rm, rs, ra, om, os, oa);
            }
            if (gq == 0) {
                st_m[w * 128 + m * 16 + mi] = rm;
                st_s[w * 128 + m * 16 + mi] = rs;
                st_a[w * 128 + m * 16 + mi] = ra;
            }
        }
        __syncthreads();
        if (threadIdx.x < 128) {
            const int r = threadIdx.x, row = mt0 * 16 + r;
            float rm = st_m[r], rs = st_s[r];
            int ra = st_a[r];
#pragma unroll
            for (int x = 1; x < NW; x++) merge_stat(rm, rs, ra, st_m[x * 128 + r], st_s[x * 128 + r], st_a[x * 128 + r]);
            if (row < g.MT_total * 16) {
                float *p = epi.stats + ((size_t)row * epi.n_part + nb) * 3;
                p[0] = rm;
                p[1] = rs;
                p[2] = __int_as_float(ra);
            }
        }
    } else {
#pragma unroll
        for (int m = 0; m < 8; m++)
#pragma unroll
            for (int j = 0; j < NGW; j++) {
                const int mt = mt0 + m, nt = nt0 + j;
                if (mt < g.MT_total && nt < g.NT) {
                    f32x4 c;
                    if (!epi.transposed(nt)) {
                        c = acc[m][j] * s_rstd[m * 16 + (lane & 15)];
                    } else {
                        // lane (g, ni) gets rows 4g..4g+3 of column ni: through this wave's LDS scratch
                        const int ni = lane & 15, gq = lane >> 4;
                        scr[w][lane] = acc[m][j];
                        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");      // store before the transposed reads
                        const float *base = reinterpret_cast<const float *>(&scr[w][0]);
#pragma unroll
                        for (int r = 0; r < 4; r++)
                            c[r] = base[((ni >> 2) * 16 + 4 * gq + r) * 4 + (ni & 3)] * s_rstd[m * 16 + 4 * gq + r];
                        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");      // reads before the next tile's store
                    }
                    epi(mt, nt, c, lane, 0);
                }
            }
    }
}

// Adds the KS partial sums of every output tile in a fixed order and runs the epilogue.
template <class Epi>
__global__ __launch_bounds__(512) void tile_epilogue_kernel(TileArgs g, Epi epi) {
    __shared__ float s_rstd[16];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int mt = blockIdx.y, nt = blockIdx.x * 8 + w;
    if (g.ssq) {
        // 16 rows of this m-tile: two per wave
        for (int r = w * 2; r < w * 2 + 2; r++) {
            const float *p = g.ssq + (size_t)(mt * 16 + r) * g.n_ssq;
            float q = 0.f;
            for (int i0 = 0; i0 < g.n_ssq; i0 += 256) {
                const int i = i0 + 4 * lane, ic = i < g.n_ssq - 4 ? i : g.n_ssq - 4;
                f32x4 v = *reinterpret_cast<const f32x4 *>(p + ic);
                q += i < g.n_ssq ? (v[0] + v[1]) + (v[2] + v[3]) : 0.f;
            }
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) q += __shfl_xor(q, o);
            if (lane == 0) s_rstd[r] = 1.0f / sqrtf(q * g.inv_d + g.eps);
        }
    } else if (threadIdx.x < 16) {
        s_rstd[threadIdx.x] = 1.0f;
    }
    __syncthreads();
    if (nt >= g.NT) return;
    const auto pre = epi_preload(epi, mt, nt, lane);       // (the residual tile: requested with the partial sums, not after them)
    // The KS partial sums of a tile are requested together and added in slice order: a loop that loads and adds one
    // slice at a time is a chain of KS memory latencies (5.6 of the 6.4 us this kernel took at eight slices).
    f32x4 c = f32x4{0.f, 0.f, 0.f, 0.f};
    const size_t slice = (size_t)g.MT_total * g.NT * 256;
    const float *base = g.partial + ((size_t)mt * g.NT + nt) * 256;
    if (!epi.transposed(nt)) {
        const float *p = base + lane * 4;
        auto sum = [&](auto N) __attribute__((always_inline)) {
            constexpr int n = decltype(N)::value;
            f32x4 v[n];
#pragma unroll
            for (int s = 0; s < n; s++) v[s] = *reinterpret_cast<const f32x4 *>(p + s * slice);
#pragma unroll
            for (int s = 0; s < n; s++) c += v[s];
        };
        switch (g.KS) {
            case 2: sum(std::integral_constant<int, 2>{}); break;
            case 4: sum(std::integral_constant<int, 4>{}); break;
            case 8: sum(std::integral_constant<int, 8>{}); break;
            case 16: sum(std::integral_constant<int, 16>{}); break;
            default:
                for (int s = 0; s < g.KS; s++) c += *reinterpret_cast<const f32x4 *>(p + s * slice);
        }
        c *= s_rstd[lane & 15];
    } else {
        const int ni = lane & 15, gq = lane >> 4;
        const float *p = base + ((ni >> 2) * 16 + 4 * gq) * 4 + (ni & 3);
        auto sum = [&](auto N) __attribute__((always_inline)) {
            constexpr int n = decltype(N)::value;
            float v[n][4];
#pragma unroll
            for (int s = 0; s < n; s++)
#pragma unroll
                for (int r = 0; r < 4; r++) v[s][r] = p[s * slice + r * 4];
#pragma unroll
            for (int s = 0; s < n; s++)
#pragma unroll
                for (int r = 0; r < 4; r++) c[r] += v[s][r];
        };
        switch (g.KS) {
            case 2: sum(std::integral_constant<int, 2>{}); break;
            case 4: sum(std::integral_constant<int, 4>{}); break;
            case 8: sum(std::integral_constant<int, 8>{}); break;
            default:
                for (int s = 0; s < g.KS; s++)
#pragma unroll
                    for (int r = 0; r < 4; r++) c[r] += p[s * slice + r * 4];
        }
#pragma unroll
        for (int r = 0; r < 4; r++) c[r] *= s_rstd[4 * gq + r];
    }
    epi_apply(epi, mt, nt, c, lane, 0, pre);
}

}  // namespace odb
