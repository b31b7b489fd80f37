// Stand-alone launches of the weight-streaming GEMM (see gemm_core.h).
#include <mutex>

#include "gemm_big.h"

namespace odb {

template <int MT, int NG, int PF, class Epi, int WKT = WK, bool IL = false>
__global__ __launch_bounds__(64 * WKT) void gemm_stream_kernel(GemmArgs g, Epi epi) {
    __shared__ __attribute__((aligned(16))) char smem[kGemmSmemBytes];
    frag_t wb[PF][NG];
    gemm_wg<MT, NG, PF, Epi, WKT, IL>(g, epi, blockIdx.x, gridDim.x, blockIdx.y * MT, wb, smem);
}

constexpr int kStreamWGs = 256;      // one workgroup per compute unit
// Every workgroup of the streaming kernels reads the same activation tiles; started at the same k-tile they ask the
// same L2 channels for them at the same time.  Workgroup wg starts kKRot * wg k-tiles further on and wraps round
// (7 is coprime to the 12 and 16 k-tiles per wave of the 8B shape; of 1, 3, 5 and 7 the multipliers 3 and 7 leave the
// 32-row gate/up kernel at its 33.0 us, 1 and 5 cost it 0.6 us): the down projection 22.5 -> 20.7 us at 32 rows,
// gate/up 49.0 -> 47.4 us at 128 rows; the order of a workgroup's fp32 sums depends on its index, not on the run.
constexpr int kKRot = 7;

// The streaming kernel with K split over KS workgroups per block of n-tiles, for projections whose activations
// are long (the down projection: every workgroup of the plain kernel reads all 32 x 12288 of them through L2,
// which costs as much as a third of its weight stream).  Workgroup (n-block, ks) adds k-slice ks for NG n-tiles
// and leaves its sums in partial[ks]; each workgroup then bumps the block's arrival counter, and the one that
// arrives last adds the KS partial sums in slice order (so the result does not depend on who was last) and runs
// the epilogue.  Nobody waits: the other workgroups simply exit.  Partial sums and counter travel as
// device-coherent accesses, ordered by a wait for the stores' completion before the counter is touched; cache-wide
// fences (a release / acquire pair) were measured to stall the weight streams of every workgroup on the chip
// (108 us instead of 20 us in a traffic model of this kernel).  The counter is back at zero when the kernel ends.
template <int MT, int NG, int PF, int KS, class Epi>
__global__ __launch_bounds__(64 * WK) void gemm_stream_ksplit_kernel(GemmArgs g, Epi epi, float *partial, unsigned *arrive) {
    __shared__ __attribute__((aligned(16))) char smem[kGemmSmemBytes];
    __shared__ unsigned s_old;
    const int ks = blockIdx.x % KS, nb = blockIdx.x / KS, nblocks = gridDim.x / KS;
    const int kl = g.KT / KS;
    GemmArgs gs = g;
    gs.k_len = kl;
    gs.A += (size_t)ks * kl * g.MT_total * kTileElems;
    gs.W += (size_t)ks * kl * kTileElems;
    const size_t slice = (size_t)g.MT_total * g.NT * 256;
    frag_t wb[PF][NG];
    gemm_wg<MT, NG, PF, EpiPartial, WK, false>(gs, EpiPartial{partial + ks * slice, g.NT}, nb, nblocks, 0, wb, smem);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");         // this wave's partial sums have been written
    __syncthreads();
    if (threadIdx.x == 0) s_old = __hip_atomic_fetch_add(arrive + nb, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (s_old != KS - 1) return;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int n_lo = (int)((unsigned)nb * (unsigned)g.NT / (unsigned)nblocks), n_hi = (int)((unsigned)(nb + 1) * (unsigned)g.NT / (unsigned)nblocks);
    const int nn = n_hi - n_lo;
    for (int t = wv; t < g.MT_total * nn; t += WK) {
        const int mt = t / nn, nt = n_lo + t % nn;
        const float *q = partial + ((size_t)mt * g.NT + nt) * 256 + lane;
        const auto pre = epi_preload(epi, mt, nt, lane);
        f32x4 c = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int s = 0; s < KS; s++)
#pragma unroll
            for (int r = 0; r < 4; r++)
                c[r] += __hip_atomic_load(q + s * slice + r * 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        epi_apply(epi, mt, nt, c, lane, 0, pre);
    }
    if (threadIdx.x == 0) __hip_atomic_store(arrive + nb, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

constexpr int kSplitKS = 4, kSplitNG = 4, kSplitPF = 4;      // (2 x 2 n-tiles, rings of 2, 6 and 8 measured slower)
// shapes the K-split kernel takes: up to 96 rows without a fused norm, n-blocks x KS workgroups within the chip,
// k-slices that the waves and the ring divide, room for the partial sums
static bool ksplit_ok(GemmShape sh, Workspace ws) {
    const int nblocks = (sh.N_tiles + kSplitNG - 1) / kSplitNG;
    return sh.M_tiles <= 6 && ws.arrive && nblocks * kSplitKS <= kStreamWGs && nblocks <= 1024 &&
           sh.K_tiles % (kSplitKS * WK * kSplitPF) == 0 &&
           (size_t)kSplitKS * sh.M_tiles * sh.N_tiles * 1024 <= ws.partial_bytes;
}
template <class Epi>
static void launch_stream_ksplit(const u16 *a, const u16 *w, GemmShape sh, Epi e, Workspace ws, hipStream_t s) {
    GemmArgs g;
    g.A = a; g.W = w; g.KT = sh.K_tiles; g.MT_total = sh.M_tiles; g.NT = sh.N_tiles;
    g.ssq = nullptr; g.n_ssq = 0; g.eps = 0.f; g.inv_d = 0.f; g.k_len = 0; g.k_rot = kKRot;
    const int nblocks = (sh.N_tiles + kSplitNG - 1) / kSplitNG;
    const dim3 grid(nblocks * kSplitKS);
    if (sh.M_tiles <= 2) gemm_stream_ksplit_kernel<2, kSplitNG, kSplitPF, kSplitKS, Epi><<<grid, 64 * WK, 0, s>>>(g, e, ws.partial, ws.arrive);
    else if (sh.M_tiles <= 4) gemm_stream_ksplit_kernel<4, kSplitNG, 4, kSplitKS, Epi><<<grid, 64 * WK, 0, s>>>(g, e, ws.partial, ws.arrive);
    else gemm_stream_ksplit_kernel<6, kSplitNG, 2, kSplitKS, Epi><<<grid, 64 * WK, 0, s>>>(g, e, ws.partial, ws.arrive);
}

// The persistent streaming kernel for up to 128 rows: MT row tiles per wave (2, 4, 6 or 8: 32-row steps),
// NG n-tiles per group, a PF-deep ring, WKT waves (four when the accumulators need the 512-register budget).
// The per-projection choices below are the fastest measured on MI355X; K_tiles that the ring depth does not
// divide fall back to a ring of one.
template <int MT, int NG, int PF, int WKT, bool IL, class Epi>
static void launch_stream(const u16 *a, const u16 *w, GemmShape sh, NormIn ni, Epi e, hipStream_t s) {
    GemmArgs g;
    g.A = a; g.W = w; g.KT = sh.K_tiles; g.MT_total = sh.M_tiles; g.NT = sh.N_tiles;
    g.ssq = ni.ssq; g.n_ssq = ni.n_ssq; g.eps = ni.eps; g.inv_d = 1.0f / (float)(sh.K_tiles * 32);
    g.k_len = 0; g.k_rot = kKRot;
    const int kw = sh.K_tiles / WKT;                // K_tiles is a multiple of 8 (checked at model creation)
    const int groups = (sh.N_tiles + NG - 1) / NG;
    dim3 grid(groups < kStreamWGs ? groups : kStreamWGs, 1);
    if (kw % PF == 0) gemm_stream_kernel<MT, NG, PF, Epi, WKT, IL><<<grid, 64 * WKT, 0, s>>>(g, e);
    else gemm_stream_kernel<MT, NG, 1, Epi, WKT, IL><<<grid, 64 * WKT, 0, s>>>(g, e);
}

// workgroup shapes of the tile kernel: (waves, n-tiles per wave, ring depth)
struct TileCfg { int nw, ngw, max_wgs; };
static TileCfg tile_cfg(int m_tiles) { return m_tiles > 8 ? TileCfg{8, 2, 256} : TileCfg{8, 1, 256}; }

template <class Epi>
static void launch_tile(const u16 *a, const u16 *w, GemmShape sh, NormIn ni, Epi e, Workspace ws, bool may_split,
                        hipStream_t s) {
    TileArgs g;
    g.A = a; g.W = w; g.KT = sh.K_tiles; g.MT_total = sh.M_tiles; g.NT = sh.N_tiles;
    g.ssq = ni.ssq; g.n_ssq = ni.n_ssq; g.eps = ni.eps; g.inv_d = 1.0f / (float)(sh.K_tiles * 32);
    g.partial = ws.partial;
    const int m_blocks = (sh.M_tiles + 7) / 8;
    const TileCfg c = tile_cfg(sh.M_tiles);
    const int per_wg = c.nw * c.ngw;
    g.n_blocks = (sh.N_tiles + per_wg - 1) / per_wg;
    int ks = 1;
    while (may_split && g.n_blocks * m_blocks * ks * 2 <= c.max_wgs && sh.K_tiles % (ks * 2) == 0 &&
           sh.K_tiles / (ks * 2) >= 8 && (size_t)(ks * 2) * sh.M_tiles * sh.N_tiles * 1024 <= ws.partial_bytes)
        ks *= 2;
    g.KS = ks;
    dim3 grid(g.n_blocks * ks, m_blocks);
    // (8 waves x 1 n-tile, ring of 8) for the multi-draft step, (8 x 2, ring of 4) for compute-bound shapes:
    // the best of the shapes tried on MI355X (4-wave workgroups of 1, 2 or 4 n-tiles per wave, 8 x 2 with a ring of 8
    // and 2 or 4 k-tiles per barrier were all slower or equal - occupancy beats wider tiles here; 8 x 4 spills)
    // (a single block of rows: every weight tile is read once, non-temporally)
    if (c.ngw == 1 && m_blocks == 1) gemm_tile_kernel<8, 1, 8, Epi, true><<<grid, 512, 0, s>>>(g, e);
    else if (c.ngw == 1) gemm_tile_kernel<8, 1, 8, Epi><<<grid, 512, 0, s>>>(g, e);
    else gemm_tile_kernel<8, 2, 4, Epi><<<grid, 512, 0, s>>>(g, e);
    if (ks > 1) {
        if constexpr (!is_row_stats<Epi>::value)
            tile_epilogue_kernel<Epi><<<dim3((sh.N_tiles + 7) / 8, sh.M_tiles), 512, 0, s>>>(g, e);
    }
}

// 256 rows and more: blocks of MBT x 16 rows through LDS (gemm_big.h), 64 * WN columns wide
template <int WN, class Epi, int MBT = 16>
static void launch_big_wn(const u16 *a, const u16 *w, GemmShape sh, NormIn ni, Epi e, hipStream_t s) {
    BigArgs g;
    g.A = a; g.W = w; g.KT = sh.K_tiles; g.MT_total = sh.M_tiles; g.NT = sh.N_tiles;
    g.ssq = ni.ssq; g.n_ssq = ni.n_ssq; g.eps = ni.eps; g.inv_d = 1.0f / (float)(sh.K_tiles * 32);
    g.m_blocks = (sh.M_tiles + MBT - 1) / MBT;
    g.n_blocks = (sh.N_tiles + 4 * WN - 1) / (4 * WN);
    static std::once_flag attr_once;        // once per instantiation: the ring needs more than the default 64 KiB
    std::call_once(attr_once, [] {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_big_kernel<WN, Epi, 8, MBT>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, big_smem_bytes(WN));
    });
    dim3 grid(8 * g.m_blocks * ((g.n_blocks + 7) / 8));
    gemm_big_kernel<WN, Epi, 8, MBT><<<grid, 64 * 8, big_smem_bytes(WN), s>>>(g, e);
}

// Block shape for the LDS-ring kernel - MBT 16-row tiles by 64 * WN columns - or wn = 0 when the tile kernel
// should run instead.  With T blocks on 256 compute units a launch takes ceil(T / 256) block-times, and a
// block-time shrinks more slowly than the block (the k-step is bound by its barrier and operand delivery as
// much as by its MFMAs).  Measured on one GPU at K = 4096, in units of the 256 x 256 block (110 us): 256-row
// blocks of 192 / 128 columns 0.87 / 0.68; 128-row blocks of 256 / 192 / 128 columns 0.66 / 0.60 / 0.46.  The
// shape with the smallest rounds x block-time wins among those whose block slots are at least 70 % useful (a
// ragged last block counts by its real rows); below 70 % for every shape the 128-row tile kernel wins
// (measured at 640 rows).  The 128-row blocks serve shapes that would leave compute units idle: QKV at 512 rows
// (256 blocks of 128 x 192 instead of 192 of 256 x 128: 83 -> 69 us), every wide projection at 640 rows (five row
// blocks that fit exactly: refresh 14.7 -> 13.0 ms), the 256-row step (7.6 -> 7.2 ms).
struct BigChoice { int mbt, wn; };
static BigChoice big_choice(GemmShape sh) {
    BigChoice best{16, 0};
    if (sh.M_tiles < 12 || sh.N_tiles < 32) return best;     // (192 rows fill three quarters of a 256-row block)
    const double rel16[5] = {0, 0, 0.68, 0.87, 1.0}, rel8[5] = {0, 0, 0.46, 0.60, 0.66};
    double best_cost = 0;
    for (int mbt = 16; mbt >= 8; mbt -= 8)
        for (int wn = 4; wn >= 2; wn--) {
            const int blocks = ((sh.M_tiles + mbt - 1) / mbt) * ((sh.N_tiles + 4 * wn - 1) / (4 * wn));
            const int rounds = (blocks + kStreamWGs - 1) / kStreamWGs;
            const double useful = (sh.M_tiles / (double)mbt) * (sh.N_tiles / (4.0 * wn)) / ((double)rounds * kStreamWGs);
            const double cost = rounds * (mbt == 16 ? rel16[wn] : rel8[wn]);
            // (a 128-row shape has to promise 5 % over the best 256-row one: the unit times are measurements)
            if (useful >= 0.7 && (best.wn == 0 || cost < best_cost * (mbt == 8 && best.mbt == 16 ? 0.95 : 1.0) - 1e-9)) {
                best = BigChoice{mbt, wn};
                best_cost = cost;
            }
        }
    return best;
}
static int big_width(GemmShape sh) { return big_choice(sh).wn; }
static bool use_big(GemmShape sh) { return big_width(sh) != 0; }

template <class Epi>
static void launch_big(const u16 *a, const u16 *w, GemmShape sh, NormIn ni, Epi e, hipStream_t s) {
    const BigChoice c = big_choice(sh);
    if (c.mbt == 8) {
        switch (c.wn) {
            case 2: launch_big_wn<2, Epi, 8>(a, w, sh, ni, e, s); break;
            case 3: launch_big_wn<3, Epi, 8>(a, w, sh, ni, e, s); break;
            default: launch_big_wn<4, Epi, 8>(a, w, sh, ni, e, s); break;
        }
        return;
    }
    switch (c.wn) {
        case 2: launch_big_wn<2>(a, w, sh, ni, e, s); break;
        case 3: launch_big_wn<3>(a, w, sh, ni, e, s); break;
        default: launch_big_wn<4>(a, w, sh, ni, e, s); break;
    }
}

void launch_gemm_qkv(const u16 *xa, const u16 *w, GemmShape sh, NormIn ni, QkvOut out, Workspace ws, hipStream_t s) {
    EpiQKV e{out, sh.M_tiles};
    // (Up to 96 rows a ring of ONE stage is the fastest since the weight tiles are loaded non-temporally - 2048 waves
    // with one group of tiles each in flight keep the HBM stream full, and fewer outstanding weight loads per
    // compute unit leave the activation loads less to queue behind: 1.9 % per step at 32 rows for this and the
    // gate/up projection together, 1.5 % at 64 rows, 0.5 % at 96; the 128-row gate/up keeps its four waves and deeper ring.)
    if (sh.M_tiles <= 2) launch_stream<2, 3, 1, 8, true>(xa, w, sh, ni, e, s);
    else if (sh.M_tiles <= 4) launch_stream<4, 3, 1, 8, true>(xa, w, sh, ni, e, s);          // 33..64 rows: still eight waves
    else if (sh.M_tiles <= 6) launch_stream<6, 3, 1, 8, true>(xa, w, sh, ni, e, s);          // 65..96 rows
    // (128 rows: eight waves and a ring of one fit 256 registers - 36.5 -> 35.3 us against four waves with a ring of four)
    else if (sh.M_tiles <= 8) launch_stream<8, 3, 1, 8, false>(xa, w, sh, ni, e, s);
    else if (use_big(sh)) launch_big(xa, w, sh, ni, e, s);
    else launch_tile(xa, w, sh, ni, e, ws, true, s);
}
void launch_gemm_resid(const u16 *a, const u16 *w, GemmShape sh, float *h, int ldh, NormOut no, Workspace ws,
                       hipStream_t s) {
    EpiResid e{h, ldh, no, sh.M_tiles};
    // K split over four workgroups with the in-kernel reduction (gemm_stream_ksplit_kernel) where it measured
    // faster at the 8B shape: the down projection (more input than output channels) up to 96 rows and the O
    // projection from 33 to 96 rows.  Per step: 3.55 -> 3.47 ms at 32 rows, 4.25 -> 4.03 at 64, 4.77 -> 4.71 at 96.
    // (At 32 rows the O projection is 0.6 % slower that way than with the plain streaming kernel; at 96 rows either
    // projection alone measured 1 % slower and only both together faster; at 128 rows, where the ring is down to
    // two stages, every combination loses 1-1.5 % to the tile kernel, and a four-wave variant with a ring of
    // four loses 4 %.)
    // Otherwise, more than 32 rows: the tile kernel, whose K split over workgroups also splits the activation
    // reads, with a separate pass that adds the partial sums.  From 2048 rows the 256 x 128 blocks of the 256-row
    // kernel fill the chip (8 x 32 blocks for N = 4096).
    const bool long_k = sh.K_tiles > sh.N_tiles;
    if (sh.M_tiles <= 6 && (long_k || sh.M_tiles > 2) && ksplit_ok(sh, ws)) launch_stream_ksplit(a, w, sh, e, ws, s);
    else if (sh.M_tiles <= 2) launch_stream<2, 1, 8, 8, false>(a, w, sh, NormIn{nullptr, 0, 0.f}, e, s);
    // (128-row blocks only for the O projection: at 1024 rows 256 blocks of 128 x 128 take 57 us against 64 us for the
    // tile kernel and its reduction pass; the down projection, three times as long in K, measured 4 % slower that way)
    else if (use_big(sh) && (big_choice(sh).mbt == 16 || sh.K_tiles <= sh.N_tiles))
        launch_big(a, w, sh, NormIn{nullptr, 0, 0.f}, e, s);
    else launch_tile(a, w, sh, NormIn{nullptr, 0, 0.f}, e, ws, true, s);
}
void launch_gemm_swiglu(const u16 *xa, const u16 *w, GemmShape sh, NormIn ni, u16 *act, unsigned *status, Workspace ws,
                        hipStream_t s) {
    EpiSwiGLU e{act, sh.M_tiles, status};
    if (sh.M_tiles <= 2) launch_stream<2, 6, 1, 8, true>(xa, w, sh, ni, e, s);
    else if (sh.M_tiles <= 4) launch_stream<4, 6, 1, 8, true>(xa, w, sh, ni, e, s);
    else if (sh.M_tiles <= 6) launch_stream<6, 6, 1, 8, true>(xa, w, sh, ni, e, s);
    else if (sh.M_tiles <= 8) launch_stream<8, 6, 2, 4, true>(xa, w, sh, ni, e, s);
    else if (use_big(sh)) launch_big(xa, w, sh, ni, e, s);
    else launch_tile(xa, w, sh, ni, e, ws, true, s);
}

constexpr int kLmNG = 6;      // n-tiles per group of the LM head at up to 32 rows

// partials per row that launch_gemm_lmstats writes
// Up to 32 rows the group is four n-tiles wide where that leaves fewer padded slots in a workgroup's last group
// (126464 columns: 31 n-tiles per workgroup = eight groups of four with one slot idle, against six groups of six
// with five; measured 166 -> 159 us).
static int lm_ng(int n_tiles, int m_tiles) {
    if (m_tiles > 2) return kLmNG;
    const int per = (n_tiles + kStreamWGs - 1) / kStreamWGs;
    return (per + 3) / 4 * 4 < (per + kLmNG - 1) / kLmNG * kLmNG ? 4 : kLmNG;
}
// Beyond 128 rows the LM head of a long vocabulary always runs on the LDS-ring kernel, 256 columns wide where no other width is chosen
// (129..191 rows leave part of a 256-row block empty, and still measure 283 us against 427 us on the tile kernel:
// the vocabulary is long enough to be bound by the weight stream either way)
static int lm_big_width(GemmShape sh) { const int wn = big_width(sh); return wn || sh.N_tiles < 32 ? wn : 4; }
// From 33 to 128 rows the LM head runs on the tile kernel with four n-tiles per wave (see launch_gemm_lmstats)
constexpr int kLmTileNGW = 4;
static bool lm_tile(int m_tiles) { return m_tiles > 2 && m_tiles <= 8; }
int lm_stats_parts(int n_tiles, int m_tiles) {
    if (lm_tile(m_tiles)) return (n_tiles + 8 * kLmTileNGW - 1) / (8 * kLmTileNGW);
    if (m_tiles <= 8) {
        const int ng = lm_ng(n_tiles, m_tiles);
        const int groups = (n_tiles + ng - 1) / ng;
        return (groups < kStreamWGs ? groups : kStreamWGs) * ng;
    }
    if (const int wn = lm_big_width(GemmShape{m_tiles, n_tiles, 0})) return (n_tiles + 4 * wn - 1) / (4 * wn);
    const TileCfg c = tile_cfg(m_tiles);
    return (n_tiles + c.nw * c.ngw - 1) / (c.nw * c.ngw);
}

void launch_gemm_lmstats(const u16 *xa, const u16 *w, GemmShape sh, NormIn ni, float *stats, Workspace ws,
                         hipStream_t s) {
    const int parts = lm_stats_parts(sh.N_tiles, sh.M_tiles);
    if (sh.M_tiles <= 2 && lm_ng(sh.N_tiles, sh.M_tiles) == 4) launch_stream<2, 4, 4, 8, true>(xa, w, sh, ni, EpiLMStats<2>(stats, parts), s);
    else if (sh.M_tiles <= 2) launch_stream<2, kLmNG, 4, 8, true>(xa, w, sh, ni, EpiLMStats<2>(stats, parts), s);
    else if (lm_tile(sh.M_tiles)) {
        // 33..128 rows.  A streaming workgroup reads all activation rows once per group of six n-tiles, and with 31
        // n-tiles per workgroup that is five to six times [rows x d] through each compute unit's vector-memory path,
        // more than its weights: at 128 rows the kernel was bound by that path (244 us, 4.2 TB/s).  The tile kernel
        // shares the activation slab between eight waves through LDS, so with four n-tiles per wave a workgroup reads
        // the activations once for 32 n-tiles; the vocabulary gives 247 such workgroups, one round on the chip:
        // 167 us at 128 rows (6.2 TB/s), and the finishing kernel merges 247 partials per row instead of 1536.
        TileArgs g;
        g.A = xa; g.W = w; g.KT = sh.K_tiles; g.MT_total = sh.M_tiles; g.NT = sh.N_tiles;
        g.ssq = ni.ssq; g.n_ssq = ni.n_ssq; g.eps = ni.eps; g.inv_d = 1.0f / (float)(sh.K_tiles * 32);
        g.partial = nullptr; g.KS = 1;
        g.n_blocks = parts;
        gemm_tile_kernel<8, kLmTileNGW, 4, TileLMStats, true><<<dim3(g.n_blocks, 1), 512, 0, s>>>(g, TileLMStats{stats, parts});
    }
    else if (use_big(sh)) launch_big(xa, w, sh, ni, TileLMStats{stats, parts}, s);
    else if (lm_big_width(sh)) launch_big_wn<4>(xa, w, sh, ni, TileLMStats{stats, parts}, s);
    else launch_tile(xa, w, sh, ni, TileLMStats{stats, parts}, ws, false, s);
}
void launch_gemm_store(const u16 *xa, const u16 *w, GemmShape sh, NormIn ni, float *out, int units, int rpu_pad,
                       int valid, int ld, Workspace ws, hipStream_t s) {
    EpiStore e{out, units, rpu_pad, valid, ld};
    if (sh.M_tiles <= 2) launch_stream<2, 3, 8, 8, true>(xa, w, sh, ni, e, s);
    else if (sh.M_tiles <= 4) launch_stream<4, 3, 4, 8, true>(xa, w, sh, ni, e, s);
    else if (sh.M_tiles <= 8) launch_stream<8, 3, 2, 8, false>(xa, w, sh, ni, e, s);
    else if (use_big(sh)) launch_big(xa, w, sh, ni, e, s);
    else launch_tile(xa, w, sh, ni, e, ws, false, s);
}

}  // namespace odb
