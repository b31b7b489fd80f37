// Device-side core of the weight-streaming binary16 MFMA GEMM  C[M,N] = A[M,K] * W[N,K]^T
// for few rows (launched from gemm.hip).
//
// A (activations) is tile-major [k_tile][m_tile][512], W is [n_tile][k_tile][512]
// (see common.h for the tile).  The work is persistent in spirit: nwg workgroups
// (one per compute unit) split the n-tiles into equal contiguous ranges, and the
// eight waves of a workgroup split K into eight slices.  Each wave therefore
// walks, NG n-tiles at a time, along contiguous runs of 1 KiB weight tiles,
// loading them straight into MFMA operand registers through a ring of PF stages
// that keeps running across the boundary between one group of n-tiles and the
// next, so the HBM stream never drains.  The eight K-slices of an output tile
// are added through LDS in a fixed order, so results do not depend on scheduling.
//
// Variants (template parameters of gemm_wg): WKT waves per workgroup (8, or 4 when 48
// accumulator tiles per wave need the 512-register budget of one wave per SIMD), and
// IL, which hands the k-tiles to the waves round-robin instead of in contiguous
// slices, so that the workgroup as a whole reads WKT KiB of contiguous weights per step
// (measured 5 % faster on the wide gate/up stream, slightly slower on the down projection).
//
// The epilogues fuse what follows each projection in the transformer block:
// RoPE + scatter of Q/K/V into the attention layouts, the residual add (plus the
// input of the next RMSNorm), SiLU(gate)*up, and the per-row softmax statistics
// of the LM head (logits are never stored).
#pragma once
#include "model.h"


namespace odb {

constexpr int WK = 8;    // waves per workgroup = K slices

struct GemmArgs {
    const u16 *A, *W;
    int KT, MT_total, NT;
    // fused RMSNorm of the input rows: A holds binary16(x * gain) and ssq[row][0..n_ssq) partial sums
    // of x^2; the result rows are scaled by 1/sqrt(sum/d + eps).  ssq == nullptr: A is used as is.
    const float *ssq;
    int n_ssq;
    float eps, inv_d;
    // k-tiles this call covers (0: all KT).  A and W then point at the first k-tile of the slice; KT stays the
    // distance between the n-tiles of W.
    int k_len;
    // > 0: workgroup wg walks its k-tiles starting at (wg * k_rot) % (k-tiles per wave) and wraps round, so that the
    // workgroups, which all read the same activation tiles, do not ask the same L2 channels for them at the same time
    int k_rot;
};

// m-tiles per reduction pass: at most six 1 KiB tiles per wave go through LDS at a time
// (with four waves twice as many: the buffer holds WK * 6 tiles)
constexpr int gemm_mc(int mt, int ng, int wkt = WK) {
    return wkt == 4 && mt == 8 ? (ng >= 6 ? 2 : (ng >= 3 ? 4 : 8))
                               : (ng >= 4 ? 1 : (ng >= 3 ? 2 : (mt < 4 ? mt : (mt % 4 == 0 ? 4 : 3))));
}

constexpr int kGemmSmemBytes = WK * 6 * 1024 + 8 * 16 * 4;    // LDS one workgroup needs (red + row scales)

// Hooks for epilogues that read global memory (the residual tile, the RoPE table): epi_preload issues those loads
// before the partial sums go through LDS, epi_apply hands their result to the epilogue, so that their latency runs
// under the reduction instead of in the tail of the kernel.  Default: nothing to preload.
struct NoPre {};
template <class Epi>
__device__ __forceinline__ NoPre epi_preload(const Epi &, int, int, int) { return NoPre{}; }
template <class Epi>
__device__ __forceinline__ void epi_apply(Epi &epi, int mt, int nt, f32x4 c, int lane, int slot, NoPre) { epi(mt, nt, c, lane, slot); }

// One workgroup's share of the GEMM: n-tiles [wg*NT/nwg, (wg+1)*NT/nwg), m-tiles mt0 .. mt0+MT-1.
// The epilogue is called as epi(mt, nt, c, lane, slot): slot numbers the (m-chunk, tile) pairs that
// this wave serves, the same in every group of n-tiles, so a stateful epilogue can keep one
// accumulator per slot; epi.finish(mt, part, lane, slot) follows once per slot at the end.
template <int MT, int NG, int PF, class Epi, int WKT = WK, bool IL = false>
__device__ __forceinline__ void gemm_wg(const GemmArgs &g, Epi epi, int wg, int nwg, int mt0,
                                        frag_t (&wb)[PF][NG], char *smem) {
    constexpr int MC = gemm_mc(MT, NG, WKT);                // m-tiles reduced per pass through LDS (<= 48 KiB)
    constexpr int SPW = (MC * NG + WKT - 1) / WKT;          // reduced tiles a wave serves per m-chunk
    static_assert(MT % MC == 0 && MC * NG * WKT <= 6 * WK && MT <= 8 && WKT <= WK, "m chunking");
    f32x4 (*red)[MC * NG][64] = reinterpret_cast<f32x4 (*)[MC * NG][64]>(smem);
    float *s_rstd = reinterpret_cast<float *>(smem + WK * 6 * 1024);

    const int lane = threadIdx.x & 63, wk = threadIdx.x >> 6;
    const int n_lo = (int)((unsigned)wg * (unsigned)g.NT / (unsigned)nwg);      // (32-bit: wg * NT stays far below 2^32)
    const int n_hi = (int)((unsigned)(wg + 1) * (unsigned)g.NT / (unsigned)nwg);
    if (n_lo >= n_hi) return;
    const int KW = (g.k_len ? g.k_len : g.KT) / WKT;
    const int ngroups = (n_hi - n_lo + NG - 1) / NG;
    const int k0 = IL ? wk : wk * KW, kst = IL ? WKT : 1;      // first k-tile of this wave and its stride

    const u16 *wbase = g.W + (size_t)k0 * kTileElems + lane * 8;
    const u16 *ap[MT];
#pragma unroll
    for (int m = 0; m < MT; m++) {
        int mt = mt0 + m < g.MT_total ? mt0 + m : g.MT_total - 1;
        ap[m] = g.A + ((size_t)k0 * g.MT_total + mt) * kTileElems + lane * 8;
    }
    const size_t a_step = (size_t)g.MT_total * kTileElems * kst;

    frag_t ab[PF][MT];
    const int rot = g.k_rot > 0 ? (int)(((unsigned)wg * (unsigned)g.k_rot) % (unsigned)KW) : 0;
    auto load_stage = [&](int slot, int grp, int k_seq) __attribute__((always_inline)) {
        int kk = k_seq + rot;
        kk = kk >= KW ? kk - KW : kk;
#pragma unroll
        for (int n = 0; n < NG; n++) {
            int nt = n_lo + grp * NG + n;
            nt = nt < n_hi ? nt : n_hi - 1;
            wb[slot][n] = ld_frag_stream(wbase + ((size_t)nt * g.KT + kk * kst) * kTileElems);
        }
#pragma unroll
        for (int m = 0; m < MT; m++) ab[slot][m] = ld_frag(ap[m] + kk * a_step);
    };

    // Row scales of the fused RMSNorm.  A row's partial sums (up to 256 of them) are one 16-byte
    // load per lane; the loads of all RPW rows of this wave are issued back to back and BEFORE the
    // first stage, so that waiting for them does not wait for the weight stream (loads return in
    // order), and they are only reduced after the ring has been filled.
    constexpr int RPW = MT * 16 / WKT;                      // rows per wave
    float q[RPW];
    f32x4 sv[RPW];
    const int si = 4 * lane, sic = si < g.n_ssq - 4 ? si : g.n_ssq - 4;     // n_ssq is a multiple of 16
#pragma unroll
    for (int j = 0; j < RPW; j++) {
        q[j] = 0.f;
        sv[j] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (g.ssq) {
            int row = mt0 * 16 + wk + j * WKT;
            row = row < g.MT_total * 16 ? row : g.MT_total * 16 - 1;
            const float *p = g.ssq + (size_t)row * g.n_ssq;
            for (int i0 = 256; i0 < g.n_ssq; i0 += 256) {   // rows wider than 4096 only
                const int i = i0 + si, ic = i < g.n_ssq - 4 ? i : g.n_ssq - 4;
                f32x4 v = *reinterpret_cast<const f32x4 *>(p + ic);
                q[j] += i < g.n_ssq ? (v[0] + v[1]) + (v[2] + v[3]) : 0.f;
            }
            sv[j] = *reinterpret_cast<const f32x4 *>(p + sic);
        }
    }
#pragma unroll
    for (int s = 0; s < PF; s++) load_stage(s, 0, s);
    if (g.ssq) {
        // 64 lane-partials per row -> one sum per row: transposed through LDS (row stride 65 floats keeps
        // the gather conflict-free), then lane l adds RPW of the partials of row l % RPW and the 64 / RPW
        // lanes of a row finish with shuffles.  A wave only touches its own part of the buffer.
        // (RP: RPW rounded up to a power of two - six row tiles over eight waves give twelve rows per wave;
        // the lanes of the rows beyond RPW add stale scratch and are dropped)
        constexpr int RP = RPW <= 1 ? 1 : RPW <= 2 ? 2 : RPW <= 4 ? 4 : RPW <= 8 ? 8 : RPW <= 16 ? 16 : RPW <= 32 ? 32 : 64;
        static_assert(RPW <= 64 && WKT * RP * 65 * 4 <= WK * 6 * 1024, "rows per wave");
        float *tmp = reinterpret_cast<float *>(smem) + wk * (RP * 65);
#pragma unroll
        for (int j = 0; j < RPW; j++)
            tmp[j * 65 + lane] = q[j] + (si < g.n_ssq ? (sv[j][0] + sv[j][1]) + (sv[j][2] + sv[j][3]) : 0.f);
        const int row = lane % RP, part = lane / RP;
        float t = 0.f;
#pragma unroll
        for (int i = 0; i < RP; i++) t += tmp[row * 65 + part * RP + i];
#pragma unroll
        for (int o = RP; o < 64; o <<= 1) t += __shfl_xor(t, o);
        if (lane < RPW) s_rstd[wk + lane * WKT] = 1.0f / sqrtf(t * g.inv_d + g.eps);
        __syncthreads();                        // the buffer is reused by the K reduction below
    } else if (lane < RPW) {
        s_rstd[wk + lane * WKT] = 1.0f;
    }

    for (int grp = 0; grp < ngroups; grp++) {
        f32x4 acc[MT][NG];
#pragma unroll
        for (int m = 0; m < MT; m++)
#pragma unroll
            for (int n = 0; n < NG; n++) acc[m][n] = f32x4{0.f, 0.f, 0.f, 0.f};

        for (int kb = 0; kb < KW; kb += PF) {
#pragma unroll
            for (int s = 0; s < PF; s++) {
#pragma unroll
                for (int m = 0; m < MT; m++)
#pragma unroll
                    for (int n = 0; n < NG; n++) acc[m][n] = mfma16(wb[s][n], ab[s][m], acc[m][n]);
                // refill this slot with the step PF ahead, which may belong to the next group
                int kn = kb + s + PF, gn = grp;
                if (kn >= KW) { kn -= KW; gn++; }
                if (gn < ngroups) load_stage(s, gn, kn);
            }
        }

        // add the eight K-slices through LDS, MC m-tiles at a time; the wave that owns a tile runs its epilogue
#pragma unroll
        for (int mc = 0; mc < MT; mc += MC) {
            decltype(epi_preload(epi, 0, 0, 0)) pre[SPW];
#pragma unroll
            for (int u = 0; u < SPW; u++) {
                const int t = wk + u * WKT, m = t / NG, n = t % NG;
                const int mt = mt0 + mc + m, nt = n_lo + grp * NG + n;
                if (t < MC * NG && mt < g.MT_total && nt < n_hi) pre[u] = epi_preload(epi, mt, nt, lane);
            }
#pragma unroll
            for (int m = 0; m < MC; m++)
#pragma unroll
                for (int n = 0; n < NG; n++) red[wk][m * NG + n][lane] = acc[mc + m][n];
            __syncthreads();
#pragma unroll
            for (int u = 0; u < SPW; u++) {
                const int t = wk + u * WKT;
                if (t >= MC * NG) break;
                const int m = t / NG, n = t % NG;
                const int mt = mt0 + mc + m, nt = n_lo + grp * NG + n;
                if (mt < g.MT_total && nt < n_hi) {
                    f32x4 c;
                    if (!epi.transposed(nt)) {
                        c = red[0][t][lane];
#pragma unroll
                        for (int w = 1; w < WKT; w++) c += red[w][t][lane];
                        c *= s_rstd[(mc + m) * 16 + (lane & 15)];
                    } else {
                        // hand lane (g, ni) the four rows 4g..4g+3 of column ni instead of four columns of one row
                        const int ni = lane & 15, gq = lane >> 4;
                        const float *base = reinterpret_cast<const float *>(&red[0][t][0]);
                        const int stride = MC * NG * 64 * 4;        // floats between the waves' copies
#pragma unroll
                        for (int r = 0; r < 4; r++) {
                            const int src = ((ni >> 2) * 16 + 4 * gq + r) * 4 + (ni & 3);
                            float v = base[src];
#pragma unroll
                            for (int w = 1; w < WKT; w++) v += base[w * stride + src];
                            c[r] = v * s_rstd[(mc + m) * 16 + 4 * gq + r];
                        }
                    }
                    epi_apply(epi, mt, nt, c, lane, (mc / MC) * SPW + u, pre[u]);
                }
            }
            __syncthreads();
        }
    }
    // epilogues that accumulate over the n-tiles of the workgroup write their result now
#pragma unroll
    for (int mc = 0; mc < MT; mc += MC)
#pragma unroll
        for (int u = 0; u < SPW; u++) {
            const int t = wk + u * WKT;         // a tile this wave served in every group
            if (t < MC * NG && mt0 + mc + t / NG < g.MT_total)
                epi.finish(mt0 + mc + t / NG, wg * NG + t % NG, lane, (mc / MC) * SPW + u);
        }
}

// ---- epilogues ------------------------------------------------------------------
// Default:    lane l holds C[row = 16*mt + (l&15)][col = 16*nt + 4*(l>>4) + r], r = 0..3.
// Transposed: lane l holds C[row = 16*mt + 4*(l>>4) + r][col = 16*nt + (l&15)].

__device__ inline void st_f16x4(u16 *p, float a, float b, float c, float d) {
    uint2 v;
    v.x = pack2(a, b);
    v.y = pack2(c, d);
    *reinterpret_cast<uint2 *>(p) = v;
}

// (by-value pick: `c ? x : y` on two struct members is an lvalue conditional, which the compiler turns into a
// select of addresses and then parks the members on the stack)
template <class T>
__device__ __forceinline__ T pick(bool c, T a, T b) { return c ? a : b; }

struct EpiQKV {
    QkvOut o;
    int mt_total;
    __device__ bool transposed(int nt) const { return nt * 16 >= 2 * o.d; }
    __device__ void finish(int, int, int, int) const {}
    __device__ void operator()(int mt, int nt, f32x4 c, int lane, int) const {
        const int mi = lane & 15, g = lane >> 4;
        // unit and tile inside the unit; in the decoded-share step the speculative units have their own size and K/V area
        const bool spec = o.split_tile > 0 && mt >= o.split_tile;
        const int tpu = pick(spec, o.tiles_per_unit_b, o.tiles_per_unit), mtu = pick(spec, mt - o.split_tile, mt);
        const int unit = pick(spec, o.fd_tpu_b, o.fd_tpu).quot(mtu), tu = mtu - unit * tpu;
        u16 *kdst = pick(spec, o.k_b, o.k) + unit * pick(spec, o.k_b_unit_stride, o.k_unit_stride);
        u16 *vdst = pick(spec, o.v_b, o.v) + unit * pick(spec, o.v_b_unit_stride, o.v_unit_stride);
        const size_t khs = pick(spec, o.k_b_head_stride, o.k_head_stride), vhs = pick(spec, o.v_b_head_stride, o.v_head_stride);
        // (index arithmetic on tiles with precomputed multipliers: it sits in the serial tail of the kernel)
        const int sec = o.fd_d.quot(nt), rt = nt - sec * (o.d >> 4);
        const int hd = o.fd_dh.quot(rt), p0 = (rt - hd * (o.dh >> 4)) * 16;            // p0 is a multiple of 16
        if (sec < 2) {
            // physical channel 2j is logical j, 2j+1 is j + dh/2: each adjacent pair is a RoPE pair
            const int pos = o.rowpos ? o.rowpos[mt * 16 + mi] : o.pos_off + tu * 16 + mi;
            const float2 *tab = reinterpret_cast<const float2 *>(o.rope) + (size_t)pos * (o.dh / 2);
            u16 *dst = sec == 0
                ? o.q + (((size_t)hd * mt_total + mt) * (o.dh / 32) + p0 / 32) * kTileElems
                : kdst + hd * khs + ((size_t)tu * (o.dh / 32) + p0 / 32) * kTileElems;
            const int j = (p0 + 4 * g) >> 1;
            float2 cs0 = tab[j], cs1 = tab[j + 1];
            float y0 = c[0] * cs0.x - c[1] * cs0.y;
            float y1 = c[1] * cs0.x + c[0] * cs0.y;
            float y2 = c[2] * cs1.x - c[3] * cs1.y;
            float y3 = c[3] * cs1.x + c[2] * cs1.y;
            const int kk = (p0 & 16) + 4 * g;                 // k-element of y0 inside the 32-wide tile
            note_saturation(o.status, y0, y1, y2, y3);
            st_f16x4(dst + ((kk >> 3) * 16 + mi) * 8 + (kk & 7), y0, y1, y2, y3);
        } else {
            // V^T tile: row = channel, the 32 keys of a tile sit in k-slot 8*g + 4*half + r
            u16 *dst = vdst + hd * vhs + ((size_t)(tu >> 1) * (o.dh / 16) + p0 / 16) * kTileElems + lane * 8 + 4 * (tu & 1);
            note_saturation(o.status, c[0], c[1], c[2], c[3]);
            st_f16x4(dst, c[0], c[1], c[2], c[3]);
        }
    }
};

// h += C.  With a NormOut it also prepares the next RMSNorm: hb = binary16(h * gain) in the
// operand layout and the sum of squares of this tile's 16 columns per row.
// What EpiResid reads from global memory for one output tile: the residual values and (when the tile also feeds the
// next RMSNorm) the norm's gain - both requested before the sums are there, not in a chain behind them.
struct ResidPre { f32x4 hv, gn; };
struct EpiResid {
    float *h;
    int ld;
    NormOut no;
    int mt_total;
    __device__ bool transposed(int) const { return false; }
    __device__ void finish(int, int, int, int) const {}
    __device__ ResidPre preload(int mt, int nt, int lane) const {
        const int mi = lane & 15, g = lane >> 4, row = mt * 16 + mi, col = nt * 16 + 4 * g;
        ResidPre p;
        p.hv = *reinterpret_cast<const f32x4 *>(h + (size_t)row * ld + col);
        p.gn = no.hb ? *reinterpret_cast<const f32x4 *>(no.gain + col) : f32x4{0.f, 0.f, 0.f, 0.f};
        return p;
    }
    __device__ void operator()(int mt, int nt, f32x4 c, int lane, int) const { apply(mt, nt, c, lane, preload(mt, nt, lane)); }
    __device__ void apply(int mt, int nt, f32x4 c, int lane, const ResidPre &pre) const {
        const int mi = lane & 15, g = lane >> 4, row = mt * 16 + mi, col = nt * 16 + 4 * g;
        float *p = h + (size_t)row * ld + col;
        f32x4 v = pre.hv + c;
        *reinterpret_cast<f32x4 *>(p) = v;
        if (no.hb) {
            const int kk = (nt & 1) * 16 + 4 * g;
            const f32x4 y = v * pre.gn;
            note_saturation(no.status, y[0], y[1], y[2], y[3]);
            st_f16x4(no.hb + ((size_t)(nt >> 1) * mt_total + mt) * kTileElems + ((kk >> 3) * 16 + mi) * 8 + (kk & 7),
                     y[0], y[1], y[2], y[3]);
            float q = v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
            q += __shfl_xor(q, 16);
            q += __shfl_xor(q, 32);
            if (g == 0) no.ssq[(size_t)row * no.n_ssq + nt] = q;
        }
    }
};

__device__ __forceinline__ ResidPre epi_preload(const EpiResid &e, int mt, int nt, int lane) { return e.preload(mt, nt, lane); }
__device__ __forceinline__ void epi_apply(EpiResid &e, int mt, int nt, f32x4 c, int lane, int, const ResidPre &pre) { e.apply(mt, nt, c, lane, pre); }

// W_gu interleaves the rows of W_gate and W_up (physical row 2j = gate j, 2j+1 = up j)
struct EpiSwiGLU {
    u16 *act;
    int mt_total;
    unsigned *status;
    __device__ bool transposed(int) const { return false; }
    __device__ void finish(int, int, int, int) const {}
    __device__ void operator()(int mt, int nt, f32x4 c, int lane, int) const {
        const int mi = lane & 15, g = lane >> 4;
        const int j = nt * 8 + 2 * g;                         // channel of the first (gate, up) pair
        // silu(gate) * up with the hardware exponential and reciprocal (each good to 1 ulp; the result is rounded to
        // binary16 next): the exact division and exponential are some forty instructions per pair in the kernel's tail
        float y0 = c[0] * __builtin_amdgcn_rcpf(1.0f + __expf(-c[0])) * c[1];
        float y1 = c[2] * __builtin_amdgcn_rcpf(1.0f + __expf(-c[2])) * c[3];
        const int kk = j & 31;
        note_saturation(status, y0, y1, 0.f, 0.f);
        u16 *dst = act + ((size_t)(j >> 5) * mt_total + mt) * kTileElems + ((kk >> 3) * 16 + mi) * 8 + (kk & 7);
        *reinterpret_cast<uint32_t *>(dst) = pack2(y0, y1);
    }
};

// Softmax statistics of the LM head without ever storing logits.  A wave serves the same
// (m-tile, n-slot) pairs in every group of n-tiles of its workgroup, so it keeps a running
// (max, sum exp(z - max), argmax) per row and slot in registers and writes ONE partial per row and
// slot at the end: stats[row][part], part = workgroup * NG + n-slot.  Ties keep the lowest token id.
// PASSES = slots per wave (see gemm_wg).
// (Exponentials are the hardware instruction, relative error about 1e-6 at the arguments that matter: they sit between
// the groups of the weight stream, and the error of a confidence is dominated by that of the logits, about 1e-3.)
template <int PASSES>
struct EpiLMStats {
    float *stats;
    int n_part;
    float rm[PASSES], rs[PASSES];
    int ra[PASSES];
    __host__ __device__ EpiLMStats(float *st, int np) : stats(st), n_part(np) {
#pragma unroll
        for (int p = 0; p < PASSES; p++) { rm[p] = -INFINITY; rs[p] = 0.f; ra[p] = 0x7fffffff; }
    }
    __device__ bool transposed(int) const { return false; }
    __device__ void operator()(int mt, int nt, f32x4 c, int lane, int pass) {
        const int g = lane >> 4;
        float m = c[0];
        int a = nt * 16 + 4 * g;
#pragma unroll
        for (int r = 1; r < 4; r++)
            if (c[r] > m) { m = c[r]; a = nt * 16 + 4 * g + r; }
        float s = 0.f;
#pragma unroll
        for (int r = 0; r < 4; r++) s += __expf(c[r] - m);
#pragma unroll
        for (int p = 0; p < PASSES; p++)
            if (p == pass) {
                float nm = fmaxf(rm[p], m);
                rs[p] = rs[p] * (rm[p] == nm ? 1.f : __expf(rm[p] - nm)) + s * (m == nm ? 1.f : __expf(m - nm));
                ra[p] = rm[p] > m ? ra[p] : (m > rm[p] ? a : (ra[p] < a ? ra[p] : a));
                rm[p] = nm;
            }
    }
    __device__ void finish(int mt, int part, int lane, int pass) const {
        const int mi = lane & 15, g = lane >> 4;
        float m = -INFINITY, s = 0.f;
        int a = 0x7fffffff;
#pragma unroll
        for (int p = 0; p < PASSES; p++)
            if (p == pass) { m = rm[p]; s = rs[p]; a = ra[p]; }
#pragma unroll
        for (int o = 16; o <= 32; o <<= 1) {
            float om = __shfl_xor(m, o), os = __shfl_xor(s, o);
            int oa = __shfl_xor(a, o);
            float nm = fmaxf(m, om);
            s = s * (m == nm ? 1.f : __expf(m - nm)) + os * (om == nm ? 1.f : __expf(om - nm));
            a = m > om ? a : (om > m ? oa : (a < oa ? a : oa));
            m = nm;
        }
        if (g == 0) {
            float *p = stats + ((size_t)(mt * 16 + mi) * n_part + part) * 3;
            p[0] = m;
            p[1] = s;
            p[2] = __int_as_float(a);
        }
    }
};

// plain fp32 store of the valid rows (unit u, i < valid) to a compact row-major matrix
struct EpiStore {
    float *out;
    int units, rpu_pad, valid, ld;
    __device__ bool transposed(int) const { return false; }
    __device__ void finish(int, int, int, int) const {}
    __device__ void operator()(int mt, int nt, f32x4 c, int lane, int) const {
        int row = mt * 16 + (lane & 15);
        int u = row / rpu_pad, i = row % rpu_pad;
        if (u < units && i < valid)
            *reinterpret_cast<f32x4 *>(out + ((size_t)u * valid + i) * ld + nt * 16 + 4 * (lane >> 4)) = c;
    }
};

// One K slice's sums, left for the workgroup that finishes the tile (gemm.hip: gemm_stream_ksplit_kernel):
// p[m_tile][n_tile][r][lane] holds element r of the lane's fragment.  Written with device-coherent stores so
// that a workgroup on another XCD reads them without any cache-wide fence.
struct EpiPartial {
    float *p;
    int nt_total;
    __device__ bool transposed(int) const { return false; }
    __device__ void finish(int, int, int, int) const {}
    __device__ void operator()(int mt, int nt, f32x4 c, int lane, int) const {
        float *q = p + ((size_t)mt * nt_total + nt) * 256 + lane;
#pragma unroll
        for (int r = 0; r < 4; r++) __hip_atomic_store(q + r * 64, c[r], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
};

}  // namespace odb
