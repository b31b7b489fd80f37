// binary16 MFMA GEMM  C[M,N] = A[M,K] * W[N,K]^T  for the compute-bound shapes (256 rows and more:
// the cache-refresh prefill, the batched long-context step).  Same operand layouts and epilogues
// as gemm_core.h / gemm_tile.h.
//
// A workgroup of eight waves computes a 256 x (64 WN) block of C over all of K, WN = 4, 3 or 2 (256, 192 or
// 128 columns: the narrower blocks exist for shapes whose count of 256-wide blocks fills the compute units
// badly), or with MBT = 8 a 128 x (64 WN) block (each wave half as many row tiles; the description below is
// for 256 rows).  Per k-tile it needs sixteen 1 KiB tiles of A and 4 WN of W; they are copied from global memory straight into LDS
// (global_load ... lds, no registers in between) into a ring of four stages, three k-tiles ahead of
// the MFMAs, so one barrier per k-tile is the only synchronisation.  The waves form a 2 x 4 grid,
// each owning 8 x WN output tiles: per k-tile a wave reads 8 + WN operand tiles from LDS for 8 WN MFMAs,
// one k-tile ahead into a second register set, so LDS traffic and MFMAs overlap within a wave.
// Operand bytes per flop are half those of the 128-row tile kernel, which is what matters here:
// a re-read that misses the 4 MiB L2 of an XCD is served at HBM-like bandwidth (about 7 TB/s measured
// on MI355X, against 22 TB/s for L2 hits), so the ids of the workgroups are also mapped to blocks
// such that the workgroups resident on one XCD share their weight panels and rows of A.
#pragma once
#include <type_traits>
#include "gemm_tile.h"

namespace odb {

// ring stages for a block 64 * WN columns wide (16 + 4 WN KiB of a 32 KiB slot per stage).  Four for every
// width: three and five measured within 3 % of it on the same GPU (differences between GPUs of the pool are larger).
constexpr int big_stages(int) { return 4; }
constexpr int big_stage_bytes(int) { return 32 * 1024; }       // every width uses 32 KiB slots (narrower slots measured slower)
constexpr int big_smem_bytes(int wn) { return big_stages(wn) * big_stage_bytes(wn) + 8 * 1024 + 256 * 4; }   // ring, per-wave scratch, row scales

struct BigArgs {
    const u16 *A, *W;
    int KT, MT_total, NT;
    int m_blocks, n_blocks;
    const float *ssq;          // fused RMSNorm of the input rows (see GemmArgs)
    int n_ssq;
    float eps, inv_d;
};

// NWV = 4 (four waves of 128 x 32 WN columns each, accumulators in the AGPR half of the register file) halves the
// LDS reads per MFMA but measured 20 % slower than eight waves on MI355X; only NWV = 8 is instantiated.
// MBT: 16-row tiles per block, 16 (256 rows) or 8 (128 rows: twice the blocks for shapes that leave compute
// units idle otherwise; per flop it needs 1.4 x the operand bytes of the 256-row block).
template <int WN, class Epi, int NWV = 8, int MBT = 16>
__global__ __launch_bounds__(64 * NWV) void gemm_big_kernel(BigArgs g, Epi epi) {
    static_assert(WN >= 2 && WN <= 4, "block width in units of 64 columns");
    static_assert(NWV == 8 || NWV == 4, "waves per workgroup");
    static_assert(MBT == 16 || MBT == 8, "rows per block");
    constexpr int CW = NWV / 2;                 // waves side by side; two rows of them
    constexpr int WT = 4 * WN / CW;             // 16-column tiles per wave
    constexpr int MW = MBT / 2;                 // 16-row tiles per wave
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr int NS = big_stages(WN);
    typedef frag_t stage_t[32][64];                                          // tiles 0..15: A, 16..16+4*WN-1: W
    stage_t *ring = reinterpret_cast<stage_t *>(smem);
    f32x4 (*scr)[64] = reinterpret_cast<f32x4 (*)[64]>(smem + NS * big_stage_bytes(WN));   // [waves][64]
    float *s_rstd = reinterpret_cast<float *>(smem + NS * big_stage_bytes(WN) + 8 * 1024);

    const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave index, scalar
    const int wm = w / CW, wn = w % CW;                  // position of the wave in the 2 x CW grid
    // Workgroup ids go round-robin over the 8 XCDs.  The ids that land on one XCD walk down the row
    // blocks of a column of blocks before they move to that XCD's next column, so concurrently
    // resident workgroups of an XCD share weight panels (and all of them the rows of A) in its L2.
    const int xcd = blockIdx.x % 8, jx = blockIdx.x / 8;
    const int nb = (jx / g.m_blocks) * 8 + xcd, mb = jx % g.m_blocks;
    if (nb >= g.n_blocks) return;
    const int mt0 = mb * MBT, nt0 = nb * 4 * WN;

    // the first half of the waves copies the MBT tiles of A into every stage, the second half the 4 WN of W
    constexpr int PA = MBT / CW, PW = 4 * WN / CW, PMAX = PA > PW ? PA : PW;
    const u16 *src[PMAX];
    size_t kstride;
    const int per = w < CW ? PA : PW, slot0 = w < CW ? PA * w : 16 + (w - CW) * PW;
    if (w < CW) {
#pragma unroll
        for (int i = 0; i < PMAX; i++) {
            int mt = mt0 + PA * w + (i < PA ? i : PA - 1);
            mt = mt < g.MT_total ? mt : g.MT_total - 1;
            src[i] = g.A + (size_t)mt * kTileElems;
        }
        kstride = (size_t)g.MT_total * kTileElems;
    } else {
#pragma unroll
        for (int i = 0; i < PMAX; i++) {
            int nt = nt0 + PW * (w - CW) + (i < PW ? i : PW - 1);
            nt = nt < g.NT ? nt : g.NT - 1;
            src[i] = g.W + (size_t)nt * g.KT * kTileElems;
        }
        kstride = kTileElems;
    }
    // (the tile addresses are wave-uniform, so they live in scalar registers; a lane adds its 16 bytes)
    const unsigned lane_off = lane * 16;
    auto issue = [&](int slot, int k) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < PMAX; i++)
            if (i < per)
                __builtin_amdgcn_global_load_lds(reinterpret_cast<const void *>(
                                                     reinterpret_cast<const char *>(src[i] + (size_t)k * kstride) + lane_off),
                                                 (__attribute__((address_space(3))) void *)(&ring[slot][slot0 + i][0]),
                                                 16, 0, 0);
    };

    const int nk = g.KT;
#pragma unroll
    for (int j = 0; j < NS - 1; j++)
        if (j < nk) issue(j, j);

    // Row scales of the fused RMSNorm, 256 / NWV rows per wave in rounds of 16.  A row's partial sums (up to 256)
    // are one 16-byte load per lane, the loads of 16 rows are in flight together (behind the ring's first
    // stages), and the 64 lane-sums of each row are added through the still unused last slot of the
    // ring: written rotated by the row number, so that the transposed gather is free of bank conflicts.
    if (g.ssq) {
        // (32 KiB from the start of the last slot: for the narrower blocks this runs on into the per-wave
        // scratch behind the ring, which is not in use yet, and ends before the row scales)
        static_assert(big_stage_bytes(WN) + 8 * 1024 >= NWV * 16 * 64 * 4, "room for the row-scale scratch");
        constexpr int RW = MBT * 16 / NWV;      // rows per wave
        float *tmp = reinterpret_cast<float *>(&ring[NS - 1][0][0]) + w * (16 * 64);
        const int si = 4 * lane, sic = si < g.n_ssq - 4 ? si : g.n_ssq - 4;
#pragma unroll
        for (int half = 0; half < RW / 16; half++) {
            f32x4 sv[16];
            const float *rp[16];
#pragma unroll
            for (int r = 0; r < 16; r++) {
                int row = mt0 * 16 + w * RW + half * 16 + r;
                row = row < g.MT_total * 16 ? row : g.MT_total * 16 - 1;
                rp[r] = g.ssq + (size_t)row * g.n_ssq;
                sv[r] = *reinterpret_cast<const f32x4 *>(rp[r] + sic);
            }
#pragma unroll
            for (int r = 0; r < 16; r++) {
                float part = si < g.n_ssq ? (sv[r][0] + sv[r][1]) + (sv[r][2] + sv[r][3]) : 0.f;
                for (int i0 = 256; i0 < g.n_ssq; i0 += 256) {       // rows wider than 4096 only
                    const int i = i0 + si, ic = i < g.n_ssq - 4 ? i : g.n_ssq - 4;
                    f32x4 v = *reinterpret_cast<const f32x4 *>(rp[r] + ic);
                    part += i < g.n_ssq ? (v[0] + v[1]) + (v[2] + v[3]) : 0.f;
                }
                tmp[r * 64 + ((lane + r) & 63)] = part;
            }
            const int rr = lane & 15, p0 = (lane >> 4) * 16;
            float t = 0.f;
#pragma unroll
            for (int u = 0; u < 16; u++) t += tmp[rr * 64 + ((p0 + u + rr) & 63)];
            t += __shfl_xor(t, 16);
            t += __shfl_xor(t, 32);
            if (lane < 16) s_rstd[w * RW + half * 16 + lane] = 1.0f / sqrtf(t * g.inv_d + g.eps);
        }
    } else {
        for (int r = lane; r < MBT * 16 / NWV; r += 64) s_rstd[w * (MBT * 16 / NWV) + r] = 1.0f;
    }

    f32x4 acc[MW][WT];
#pragma unroll
    for (int m = 0; m < MW; m++)
#pragma unroll
        for (int j = 0; j < WT; j++) acc[m][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Software pipeline over the k-tiles.  In iteration k a wave first fetches the operand tiles of stage
    // k+1 from LDS into the second register set and then issues the MFMAs of stage k, so the LDS reads of
    // all waves run under the MFMAs instead of in a phase of their own after each barrier.  Stage k+NS-1
    // is requested from global memory in iteration k, into the slot whose tiles fed the MFMAs of k-1.
    static_assert(NS >= 3 && (NS - 2) * PMAX <= 16, "slot arithmetic and counted waits below");
    frag_t a[2][MW], b[2][WT];
    auto fetch = [&](auto P, int k) __attribute__((always_inline)) {
        constexpr int p = decltype(P)::value;
        const stage_t &st = ring[k % NS];
#pragma unroll
        for (int j = 0; j < WT; j++) b[p][j] = st[16 + wn * WT + j][lane];
#pragma unroll
        for (int m = 0; m < MW; m++) a[p][m] = st[wm * MW + m][lane];
    };
    auto mfmas = [&](auto P) __attribute__((always_inline)) {
        constexpr int p = decltype(P)::value;
#pragma unroll
        for (int m = 0; m < MW; m++)
#pragma unroll
            for (int j = 0; j < WT; j++) acc[m][j] = mfma16(b[p][j], a[p][m], acc[m][j]);
    };
    // a k-tile that has a successor
    auto step = [&](auto P, int k) __attribute__((always_inline)) {
        constexpr int p = decltype(P)::value;
        // stage k+1 has landed once every wave's copies of it are done (those of stages k+2 .. k+NS-2 may be in flight)
        if (k + NS - 2 <= nk - 1) {          // steady state: the copies of NS - 3 later stages stay in flight
            if (PA == PW || w < CW) wait_vmcnt(PA * (NS - 3));
            else wait_vmcnt(PW * (NS - 3));
        } else {
            wait_vmcnt(per * (nk - 1 - (k + 1)));
        }
        __builtin_amdgcn_s_barrier();
        if (k + NS - 1 < nk) issue((k + NS - 1) % NS, k + NS - 1);
        if constexpr (WN == 4 && NWV == 8 && MBT == 16) {
            // widest block: every register is taken, the reads of stage k+1 go ahead of the MFMAs of stage k
            // (measured 5 % faster than the interleaved order, which needs more live registers)
            fetch(std::integral_constant<int, 1 - p>{}, k + 1);
            mfmas(P);
        } else {
            // The MFMAs of stage k come first in program order and the LDS reads of stage k+1 are spread
            // between them: the wait for this stage's operands (read during the previous k-tile) then sits
            // in front of the first MFMA, before any new read is issued, and the new reads complete under
            // the MFMAs instead of being waited for ahead of them (2 % faster at 192 columns).
            mfmas(P);
            fetch(std::integral_constant<int, 1 - p>{}, k + 1);
            constexpr int NR = MW + WT, NM = MW * WT, MPR = NM / NR;
#pragma unroll
            for (int i = 0; i < NR; i++) {
                __builtin_amdgcn_sched_group_barrier(0x008, MPR, 0);       // MPR MFMAs
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);         // one LDS read
            }
            __builtin_amdgcn_sched_group_barrier(0x008, NM - NR * MPR, 0);
        }
    };
    // stage 0 has landed (everything issued so far has: the row-scale loads came after the ring's)
    wait_vmcnt(g.ssq ? 0 : per * ((nk < NS - 1 ? nk : NS - 1) - 1));
    __syncthreads();            // also orders the row-scale scratch before stage 3 reuses its slot
    fetch(std::integral_constant<int, 0>{}, 0);
    int k = 0;
    for (; k + 2 <= nk - 1; k += 2) {      // (no branch around a step's MFMAs: the accumulators keep their registers)
        step(std::integral_constant<int, 0>{}, k);
        step(std::integral_constant<int, 1>{}, k + 1);
    }
    if (k < nk - 1) {
        step(std::integral_constant<int, 0>{}, k);
        mfmas(std::integral_constant<int, 1>{});
    } else {
        mfmas(std::integral_constant<int, 0>{});
    }
    __syncthreads();            // the ring is reused below; also publishes s_rstd

    if constexpr (is_row_stats<Epi>::value) {
        // softmax statistics per row over this workgroup's columns: lane-local, across the four lane
        // groups, across the wave's four tiles, then across the four waves of a row half through LDS
        float *st_m = reinterpret_cast<float *>(smem);               // [CW column waves][256 rows]
        float *st_s = st_m + CW * 256;
        int *st_a = reinterpret_cast<int *>(st_s + CW * 256);
        const int mi = lane & 15, gq = lane >> 4;
#pragma unroll
        for (int m = 0; m < MW; m++) {
            const int r = wm * MW * 16 + m * 16 + mi;
            float rm = -INFINITY, rs = 0.f;
            int ra = 0x7fffffff;
#pragma unroll
            for (int j = 0; j < WT; j++) {
                const int nt = nt0 + wn * WT + j;
                if (nt < g.NT) {
                    f32x4 c = acc[m][j] * s_rstd[r];
                    float cm = c[0];
                    int ca = nt * 16 + 4 * gq;
#pragma unroll
                    for (int x = 1; x < 4; x++)
                        if (c[x] > cm) { cm = c[x]; ca = nt * 16 + 4 * gq + x; }
                    float cs = 0.f;
#pragma unroll
                    for (int x = 0; x < 4; x++) cs += __expf(c[x] - cm);
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
                st_m[wn * 256 + r] = rm;
                st_s[wn * 256 + r] = rs;
                st_a[wn * 256 + r] = ra;
            }
        }
        __syncthreads();
        for (int r = threadIdx.x; r < MBT * 16; r += 64 * NWV) {
            const int row = mt0 * 16 + r;
            float rm = st_m[r], rs = st_s[r];
            int ra = st_a[r];
#pragma unroll
            for (int x = 1; x < CW; x++) merge_stat(rm, rs, ra, st_m[x * 256 + r], st_s[x * 256 + r], st_a[x * 256 + r]);
            if (row < g.MT_total * 16) {
                float *p = epi.stats + ((size_t)row * epi.n_part + nb) * 3;
                p[0] = rm;
                p[1] = rs;
                p[2] = __int_as_float(ra);
            }
        }
    } else {
#pragma unroll
        for (int m = 0; m < MW; m++)
#pragma unroll
            for (int j = 0; j < WT; j++) {
                const int mt = mt0 + wm * MW + m, nt = nt0 + wn * WT + j;
                if (mt < g.MT_total && nt < g.NT) {
                    const float *rsd = s_rstd + (wm * MW + m) * 16;
                    f32x4 c;
                    if (!epi.transposed(nt)) {
                        c = acc[m][j] * rsd[lane & 15];
                    } else {
                        // lane (g, ni) gets rows 4g..4g+3 of column ni: through this wave's LDS scratch
                        const int ni = lane & 15, gq = lane >> 4;
                        scr[w][lane] = acc[m][j];
                        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");      // store before the transposed reads
                        const float *base = reinterpret_cast<const float *>(&scr[w][0]);
#pragma unroll
                        for (int r = 0; r < 4; r++)
                            c[r] = base[((ni >> 2) * 16 + 4 * gq + r) * 4 + (ni & 3)] * rsd[4 * gq + r];
                        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");      // reads before the next tile's store
                    }
                    epi(mt, nt, c, lane, 0);
                }
            }
    }
}

}  // namespace odb
