// Row-wise device functions shared by rows.hip and the fused step kernel (step.hip):
// embedding gather and the final reduction of the LM-head statistics with the
// threshold unmask.
#pragma once
#include "model.h"

namespace odb {

// h[r, :] = E[token(r), :] as fp32 (the residual stream stays in fp32).  One thread per 16 columns.
__device__ __forceinline__ void embed_row(int r, const u16 *embed, const int32_t *tokens, RowMap rm, int d, int vocab,
                                          float *h, NormOut no, int mt_total) {
    int u = r / rm.rpu_pad, i = r % rm.rpu_pad;
    int tok = 0;
    if (i < rm.valid) tok = tokens[(size_t)u * rm.valid + i];
    tok = tok < 0 ? 0 : (tok >= vocab ? vocab - 1 : tok);
    const u16 *src = embed + (size_t)tok * d;
    float *dst = h + (size_t)r * d;
    for (int nt = threadIdx.x; nt < d / 16; nt += blockDim.x) {
        float x[16];
#pragma unroll
        for (int half = 0; half < 2; half++) {
            frag_t f = ld_frag(src + nt * 16 + half * 8);
#pragma unroll
            for (int j = 0; j < 4; j++) {
                x[half * 8 + 2 * j] = bf2f(f.w[j] & 0xffff);
                x[half * 8 + 2 * j + 1] = bf2f(f.w[j] >> 16);
            }
        }
#pragma unroll
        for (int j = 0; j < 16; j += 4)
            *reinterpret_cast<float4 *>(dst + nt * 16 + j) = make_float4(x[j], x[j + 1], x[j + 2], x[j + 3]);
        if (no.hb) {
            float q = 0.f;
#pragma unroll
            for (int j = 0; j < 16; j++) q += x[j] * x[j];
            no.ssq[(size_t)r * no.n_ssq + nt] = q;
            const float *gn = no.gain + nt * 16;
#pragma unroll
            for (int half = 0; half < 2; half++) {
                frag_t f;
#pragma unroll
                for (int j = 0; j < 4; j++)
                    f.w[j] = pack2(x[half * 8 + 2 * j] * gn[half * 8 + 2 * j],
                                     x[half * 8 + 2 * j + 1] * gn[half * 8 + 2 * j + 1]);
                const int chunk = (nt & 1) * 2 + half;
                *reinterpret_cast<frag_t *>(no.hb + ((size_t)(nt >> 1) * mt_total + (r >> 4)) * kTileElems +
                                            (chunk * 16 + (r & 15)) * 8) = f;
            }
        }
    }
}

// ---- LM-head statistics -> confidence, argmax, unmask ------------------------
// stats[row][part] = (max logit, sum exp(logit - max), argmax as int bits) over
// the 16 vocabulary columns of part.  Merging keeps the lowest id on equal maxima.
struct Stat { float m, s; int a; };

__device__ inline Stat merge(Stat x, Stat y) {
    Stat o;
    o.m = fmaxf(x.m, y.m);
    // equal maxima (including two empty -inf partials) must not evaluate inf - inf
    float ex = x.m == o.m ? 1.f : expf(x.m - o.m);
    float ey = y.m == o.m ? 1.f : expf(y.m - o.m);
    o.s = x.s * ex + y.s * ey;
    o.a = x.m > y.m ? x.a : (y.m > x.m ? y.a : (x.a < y.a ? x.a : y.a));
    return o;
}

// the whole wave merges the n_part partials of one row (p = first partial of the row); every lane gets the result
__device__ __forceinline__ Stat merge_row_partials(const float *p, int n_part, int lane) {
    Stat acc = {-INFINITY, 0.f, 0x7fffffff};
    for (int q0 = 0; q0 < n_part; q0 += 64 * 8) {            // eight independent partials per lane and pass
        Stat t[8];
#pragma unroll
        for (int j = 0; j < 8; j++) {
            int q = q0 + lane + 64 * j;
            if (q < n_part) t[j] = Stat{p[q * 3], p[q * 3 + 1], __float_as_int(p[q * 3 + 2])};
            else t[j] = Stat{-INFINITY, 0.f, 0x7fffffff};
        }
#pragma unroll
        for (int j = 0; j < 8; j++) acc = merge(acc, t[j]);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        Stat t = {__shfl_xor(acc.m, o), __shfl_xor(acc.s, o), __shfl_xor(acc.a, o)};
        acc = merge(acc, t);
    }
    return acc;
}

// One workgroup finishes unit u: merges the partial statistics of its rpu rows, then applies the
// acceptance rule (ODB-dLLM Sec. 3, Observation 3, plus the forced most-confident pick).
__device__ __forceinline__ void lm_finish_wg(int u, const float *stats, int n_part, int rows, int rpu, int rpu_pad,
                                             const int32_t *tokens, int mask_id, float tau, float *conf,
                                             int32_t *argmax, uint8_t *unmask, float *s_conf) {
    int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nw = blockDim.x >> 6;
    for (int i = wave; i < rpu; i += nw) {
        int row = u * rpu + i;                                  // compact output row
        if (row >= rows) break;
        const float *p = stats + ((size_t)u * rpu_pad + i) * n_part * 3;
        const Stat acc = merge_row_partials(p, n_part, lane);
        if (lane == 0) {
            float c = 1.0f / acc.s;
            if (conf) conf[row] = c;
            if (argmax) argmax[row] = acc.a;
            s_conf[i & 255] = c;
        }
    }
    if (unmask) {
        __syncthreads();
        if (wave == 0) {
            // most confident masked position of this draft, lowest index on ties
            float best = -1.f;
            int best_i = 0x7fffffff;
            for (int i = lane; i < rpu; i += 64) {
                bool masked = tokens[(size_t)u * rpu + i] == mask_id;
                float c = s_conf[i];
                if (masked && c > best) { best = c; best_i = i; }
            }
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) {
                float ob = __shfl_xor(best, o);
                int oi = __shfl_xor(best_i, o);
                if (ob > best || (ob == best && oi < best_i)) { best = ob; best_i = oi; }
            }
            for (int i = lane; i < rpu; i += 64) {
                bool masked = tokens[(size_t)u * rpu + i] == mask_id;
                unmask[(size_t)u * rpu + i] = (masked && (s_conf[i] > tau || i == best_i)) ? 1 : 0;
            }
        }
    }
}

}  // namespace odb
