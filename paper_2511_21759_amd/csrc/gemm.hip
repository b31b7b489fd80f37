// Weight-streaming bf16 MFMA GEMM  C[M,N] = A[M,K] * W[N,K]^T  for few rows.
//
// A (activations) is tile-major [k_tile][m_tile][512], W is [n_tile][k_tile][512]
// (see common.h for the tile).  A workgroup owns NG n-tiles x MT m-tiles and a
// slice of K (grid.y = split-K factor); its WK waves split that slice again, so
// every wave streams a contiguous run of 1 KiB weight tiles straight from HBM
// into MFMA operand registers, PF tiles ahead.  Partial sums of the waves are
// added through LDS in a fixed order; partial sums of different workgroups go
// through an fp32 workspace and are added, again in a fixed order, by the last
// workgroup to arrive - results do not depend on scheduling.
//
// The epilogues fuse what follows each projection in the transformer block:
// RoPE + scatter of Q/K/V into attention layouts, residual add, SiLU(gate)*up,
// and the per-row softmax statistics of the LM head (logits are never stored).
#include "model.h"

namespace odb {

struct GemmArgs {
    const u16 *A, *W;
    int KT, MT_total, NT, ksplit;
    float *partial;
    unsigned *counters;
};

template <int MT, int NG, int PF, bool SWAP>
__device__ inline void mainloop(const GemmArgs &g, int nt0, int mt0, int k0, int k1, int lane, f32x4 (&acc)[MT][NG]) {
    const u16 *wp[NG];
    const u16 *ap[MT];
#pragma unroll
    for (int n = 0; n < NG; n++) wp[n] = g.W + ((size_t)(nt0 + n) * g.KT) * kTileElems + lane * 8;
#pragma unroll
    for (int m = 0; m < MT; m++) {
        int mt = mt0 + m < g.MT_total ? mt0 + m : g.MT_total - 1;
        ap[m] = g.A + (size_t)mt * kTileElems + lane * 8;
    }
    const size_t a_step = (size_t)g.MT_total * kTileElems;
    frag_t wb[PF][NG], ab[PF][MT];
#pragma unroll
    for (int s = 0; s < PF - 1; s++) {
        int kt = k0 + s;
        if (kt < k1) {
#pragma unroll
            for (int n = 0; n < NG; n++) wb[s][n] = ld_frag(wp[n] + (size_t)kt * kTileElems);
#pragma unroll
            for (int m = 0; m < MT; m++) ab[s][m] = ld_frag(ap[m] + kt * a_step);
        }
    }
    for (int kb = k0; kb < k1; kb += PF) {
#pragma unroll
        for (int s = 0; s < PF; s++) {
            const int ls = (s + PF - 1) % PF;
            int kl = kb + s + PF - 1;
            if (kl < k1) {
#pragma unroll
                for (int n = 0; n < NG; n++) wb[ls][n] = ld_frag(wp[n] + (size_t)kl * kTileElems);
#pragma unroll
                for (int m = 0; m < MT; m++) ab[ls][m] = ld_frag(ap[m] + kl * a_step);
            }
            if (kb + s < k1) {
#pragma unroll
                for (int m = 0; m < MT; m++)
#pragma unroll
                    for (int n = 0; n < NG; n++)
                        acc[m][n] = SWAP ? mfma16(ab[s][m], wb[s][n], acc[m][n]) : mfma16(wb[s][n], ab[s][m], acc[m][n]);
            }
        }
    }
}

template <int MT, int NG, int WK, int PF, class Epi>
__global__ __launch_bounds__(64 * WK) void gemm_skinny_kernel(GemmArgs g, Epi epi) {
    constexpr int TP = Epi::kTP;
    constexpr int GP = NG / TP;               // epilogue groups per m-tile
    static_assert(NG % TP == 0 && GP <= WK, "tile grouping");
    const int lane = threadIdx.x & 63, wk = threadIdx.x >> 6;
    const int nt0 = blockIdx.x * NG, ks = blockIdx.y, mt0 = blockIdx.z * MT;
    const int kt_split = g.KT / g.ksplit;
    const int per_wave = (kt_split + WK - 1) / WK;
    const int k0 = ks * kt_split + wk * per_wave;
    const int k1 = min(k0 + per_wave, (ks + 1) * kt_split);

    f32x4 acc[MT][NG];
#pragma unroll
    for (int m = 0; m < MT; m++)
#pragma unroll
        for (int n = 0; n < NG; n++) acc[m][n] = f32x4{0.f, 0.f, 0.f, 0.f};

    if (epi.swapped(nt0)) mainloop<MT, NG, PF, true>(g, nt0, mt0, k0, k1, lane, acc);
    else mainloop<MT, NG, PF, false>(g, nt0, mt0, k0, k1, lane, acc);

    __shared__ f32x4 red[WK > 1 ? WK : 1][NG][64];
    __shared__ unsigned s_last;
    const bool split = g.ksplit > 1;

#pragma unroll
    for (int m = 0; m < MT; m++) {
        const int mt = mt0 + m;
        f32x4 c[TP];
        bool mine;
        int grp;
        if (WK > 1) {
#pragma unroll
            for (int n = 0; n < NG; n++) red[wk][n][lane] = acc[m][n];
            __syncthreads();
            mine = wk < GP;
            grp = wk;
            if (mine) {
#pragma unroll
                for (int t = 0; t < TP; t++) {
                    f32x4 sum = red[0][grp * TP + t][lane];
#pragma unroll
                    for (int w = 1; w < WK; w++) sum += red[w][grp * TP + t][lane];
                    c[t] = sum;
                }
            }
        }
#pragma unroll
        for (int gp = 0; gp < (WK > 1 ? 1 : GP); gp++) {
            if (WK == 1) {
                mine = true;
                grp = gp;
#pragma unroll
                for (int t = 0; t < TP; t++) c[t] = acc[m][gp * TP + t];
            }
            if (mine && mt < g.MT_total) {
                if (!split) {
                    epi(mt, nt0 + grp * TP, c, lane);
                } else {
#pragma unroll
                    for (int t = 0; t < TP; t++) {
                        size_t tile = ((size_t)ks * g.MT_total + mt) * g.NT + nt0 + grp * TP + t;
                        *reinterpret_cast<f32x4 *>(g.partial + tile * 256 + lane * 4) = c[t];
                    }
                }
            }
        }
        if (WK > 1) __syncthreads();
    }
    if (!split) return;

    // split-K: the last workgroup to arrive for this (m-block, n-group) adds the partials
    const unsigned cidx = blockIdx.z * gridDim.x + blockIdx.x;
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned old = atomicAdd(&g.counters[cidx], 1u);
        s_last = (old == (unsigned)g.ksplit - 1) ? 1u : 0u;
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();
    for (int tp = wk; tp < MT * GP; tp += WK) {
        const int m = tp / GP, grp = tp % GP, mt = mt0 + m;
        if (mt >= g.MT_total) continue;
        f32x4 c[TP];
#pragma unroll
        for (int t = 0; t < TP; t++) {
            f32x4 sum = f32x4{0.f, 0.f, 0.f, 0.f};
            for (int s = 0; s < g.ksplit; s++) {
                size_t tile = ((size_t)s * g.MT_total + mt) * g.NT + nt0 + grp * TP + t;
                sum += *reinterpret_cast<const f32x4 *>(g.partial + tile * 256 + lane * 4);
            }
            c[t] = sum;
        }
        epi(mt, nt0 + grp * TP, c, lane);
    }
    if (threadIdx.x == 0) g.counters[cidx] = 0;
}

// ---- epilogues ------------------------------------------------------------------
// Not swapped: lane l holds C[row = 16*mt + (l&15)][col = 16*nt + 4*(l>>4) + r], r = 0..3.
// Swapped:     lane l holds C[row = 16*mt + 4*(l>>4) + r][col = 16*nt + (l&15)].

__device__ inline void st_bf16x4(u16 *p, float a, float b, float c, float d) {
    uint2 v;
    v.x = pack2bf(a, b);
    v.y = pack2bf(c, d);
    *reinterpret_cast<uint2 *>(p) = v;
}

struct EpiQKV {
    static constexpr int kTP = 2;
    QkvOut o;
    int mt_total;
    __device__ bool swapped(int nt) const { return nt * 16 >= 2 * o.d; }
    __device__ void operator()(int mt, int nt, const f32x4 *c, int lane) const {
        const int mi = lane & 15, g = lane >> 4;
        const int unit = mt / o.tiles_per_unit, tu = mt % o.tiles_per_unit;
        const int n = nt * 16, sec = n / o.d, rr = n % o.d;
        const int hd = rr / o.dh, p0 = rr % o.dh;            // p0 is a multiple of 32
        if (sec < 2) {
            // physical channel 2j is logical j, 2j+1 is j + dh/2: each adjacent pair is a RoPE pair
            const int pos = o.pos_off + tu * 16 + mi;
            const float2 *tab = reinterpret_cast<const float2 *>(o.rope) + (size_t)pos * (o.dh / 2);
            u16 *dst = sec == 0
                ? o.q + (((size_t)hd * mt_total + mt) * (o.dh / 32) + p0 / 32) * kTileElems
                : o.k + unit * o.k_unit_stride + hd * o.k_head_stride + ((size_t)tu * (o.dh / 32) + p0 / 32) * kTileElems;
#pragma unroll
            for (int t = 0; t < 2; t++) {
                const int j = (p0 + t * 16 + 4 * g) >> 1;
                float2 cs0 = tab[j], cs1 = tab[j + 1];
                float y0 = c[t][0] * cs0.x - c[t][1] * cs0.y;
                float y1 = c[t][1] * cs0.x + c[t][0] * cs0.y;
                float y2 = c[t][2] * cs1.x - c[t][3] * cs1.y;
                float y3 = c[t][3] * cs1.x + c[t][2] * cs1.y;
                st_bf16x4(dst + ((t * 2 + (g >> 1)) * 16 + mi) * 8 + (g & 1) * 4, y0, y1, y2, y3);
            }
        } else {
            // V^T tile: row = channel, the 32 keys of a tile sit in k-slot 8*g + 4*half + r
#pragma unroll
            for (int t = 0; t < 2; t++) {
                const int dt16 = p0 / 16 + t;
                u16 *dst = o.v + unit * o.v_unit_stride + hd * o.v_head_stride +
                           ((size_t)(tu >> 1) * (o.dh / 16) + dt16) * kTileElems + lane * 8 + 4 * (tu & 1);
                st_bf16x4(dst, c[t][0], c[t][1], c[t][2], c[t][3]);
            }
        }
    }
};

struct EpiResid {
    static constexpr int kTP = 1;
    float *h;
    int ld;
    __device__ bool swapped(int) const { return false; }
    __device__ void operator()(int mt, int nt, const f32x4 *c, int lane) const {
        float *p = h + (size_t)(mt * 16 + (lane & 15)) * ld + nt * 16 + 4 * (lane >> 4);
        f32x4 v = *reinterpret_cast<f32x4 *>(p);
        *reinterpret_cast<f32x4 *>(p) = v + c[0];
    }
};

struct EpiSwiGLU {
    static constexpr int kTP = 2;
    u16 *act;
    int mt_total;
    __device__ bool swapped(int) const { return false; }
    __device__ void operator()(int mt, int nt, const f32x4 *c, int lane) const {
        const int mi = lane & 15, g = lane >> 4, t = nt >> 1;
        float y[4];
#pragma unroll
        for (int r = 0; r < 4; r++) {
            float x = c[0][r];
            y[r] = x / (1.0f + expf(-x)) * c[1][r];
        }
        u16 *dst = act + ((size_t)(t >> 1) * mt_total + mt) * kTileElems + (((t & 1) * 2 + (g >> 1)) * 16 + mi) * 8 +
                   (g & 1) * 4;
        st_bf16x4(dst, y[0], y[1], y[2], y[3]);
    }
};

struct EpiLMStats {
    static constexpr int kTP = 2;
    float *stats;
    int n_part;
    __device__ bool swapped(int) const { return false; }
    __device__ void operator()(int mt, int nt, const f32x4 *c, int lane) const {
        const int mi = lane & 15, g = lane >> 4;
        float m = -INFINITY;
        int a = 0;
#pragma unroll
        for (int t = 0; t < 2; t++)
#pragma unroll
            for (int r = 0; r < 4; r++) {
                float z = c[t][r];
                if (z > m) { m = z; a = nt * 16 + t * 16 + 4 * g + r; }
            }
        float s = 0.f;
#pragma unroll
        for (int t = 0; t < 2; t++)
#pragma unroll
            for (int r = 0; r < 4; r++) s += expf(c[t][r] - m);
#pragma unroll
        for (int o = 16; o <= 32; o <<= 1) {
            float om = __shfl_xor(m, o), os = __shfl_xor(s, o);
            int oa = __shfl_xor(a, o);
            float nm = fmaxf(m, om);
            s = s * (m == nm ? 1.f : expf(m - nm)) + os * (om == nm ? 1.f : expf(om - nm));
            a = m > om ? a : (om > m ? oa : (a < oa ? a : oa));
            m = nm;
        }
        if (g == 0) {
            float *p = stats + ((size_t)(mt * 16 + mi) * n_part + (nt >> 1)) * 3;
            p[0] = m;
            p[1] = s;
            p[2] = __int_as_float(a);
        }
    }
};

struct EpiStore {
    static constexpr int kTP = 1;
    float *out;
    int rows, ld;
    __device__ bool swapped(int) const { return false; }
    __device__ void operator()(int mt, int nt, const f32x4 *c, int lane) const {
        int row = mt * 16 + (lane & 15);
        if (row < rows) *reinterpret_cast<f32x4 *>(out + (size_t)row * ld + nt * 16 + 4 * (lane >> 4)) = c[0];
    }
};

// ---- launch ---------------------------------------------------------------------
template <class Epi>
static void launch(const u16 *a, const u16 *w, GemmShape sh, Epi epi, Workspace ws, hipStream_t s) {
    GemmArgs g;
    g.A = a; g.W = w; g.KT = sh.K_tiles; g.MT_total = sh.M_tiles; g.NT = sh.N_tiles;
    g.partial = ws.partial; g.counters = ws.counters;
    const int mt_blk = sh.M_tiles <= 2 ? 2 : (sh.M_tiles <= 4 ? 4 : 8);
    const int ng = (mt_blk == 8 && sh.N_tiles % 4 == 0) ? 4 : 2;
    const int wk = mt_blk == 8 ? 4 : 8;
    const int mblocks = (sh.M_tiles + mt_blk - 1) / mt_blk;
    const int wgs = (sh.N_tiles / ng) * mblocks;
    int ksplit = 1;
    while (wgs * ksplit < 256 && sh.K_tiles % (ksplit * 2) == 0 && sh.K_tiles / (ksplit * 2) >= wk &&
           (size_t)(ksplit * 2) * sh.M_tiles * sh.N_tiles * 1024 <= ws.partial_bytes)
        ksplit *= 2;
    g.ksplit = ksplit;
    dim3 grid(sh.N_tiles / ng, ksplit, mblocks);
    if (mt_blk == 2) gemm_skinny_kernel<2, 2, 8, 4, Epi><<<grid, 512, 0, s>>>(g, epi);
    else if (mt_blk == 4) gemm_skinny_kernel<4, 2, 8, 3, Epi><<<grid, 512, 0, s>>>(g, epi);
    else if (ng == 4) gemm_skinny_kernel<8, 4, 4, 2, Epi><<<grid, 256, 0, s>>>(g, epi);
    else gemm_skinny_kernel<8, 2, 4, 2, Epi><<<grid, 256, 0, s>>>(g, epi);
}

void launch_gemm_qkv(const u16 *xa, const u16 *w, GemmShape sh, QkvOut out, Workspace ws, hipStream_t s) {
    EpiQKV e{out, sh.M_tiles};
    launch(xa, w, sh, e, ws, s);
}
void launch_gemm_resid(const u16 *a, const u16 *w, GemmShape sh, float *h, int ldh, Workspace ws, hipStream_t s) {
    EpiResid e{h, ldh};
    launch(a, w, sh, e, ws, s);
}
void launch_gemm_swiglu(const u16 *xa, const u16 *w, GemmShape sh, u16 *act, Workspace ws, hipStream_t s) {
    EpiSwiGLU e{act, sh.M_tiles};
    launch(xa, w, sh, e, ws, s);
}
void launch_gemm_lmstats(const u16 *xa, const u16 *w, GemmShape sh, float *stats, Workspace ws, hipStream_t s) {
    EpiLMStats e{stats, sh.N_tiles / 2};
    launch(xa, w, sh, e, ws, s);
}
void launch_gemm_store(const u16 *xa, const u16 *w, GemmShape sh, float *out, int rows, int ld, Workspace ws,
                       hipStream_t s) {
    EpiStore e{out, rows, ld};
    launch(xa, w, sh, e, ws, s);
}

}  // namespace odb
