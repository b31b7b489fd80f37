// Row-wise device functions of rows.hip:
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
                for (int j = 0; j < 4; j++) {
                    const float y0 = x[half * 8 + 2 * j] * gn[half * 8 + 2 * j], y1 = x[half * 8 + 2 * j + 1] * gn[half * 8 + 2 * j + 1];
                    note_saturation(no.status, y0, y1, 0.f, 0.f);
                    f.w[j] = pack2(y0, y1);
                }
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

// UN independent partials per lane, loaded back to back, folded into the lane's running (max, sum, argmax):
// one exponential per partial (against the maximum of the pass) plus one for the running sum.
template <int UN>
__device__ __forceinline__ Stat merge_partials_pass(const float *p, int q0, int n_part, int lane, Stat acc) {
    Stat t[UN];
    float mp = acc.m;
#pragma unroll
    for (int j = 0; j < UN; j++) {
        int q = q0 + lane + 64 * j;
        if (q < n_part) t[j] = Stat{p[q * 3], p[q * 3 + 1], __float_as_int(p[q * 3 + 2])};
        else t[j] = Stat{-INFINITY, 0.f, 0x7fffffff};
        mp = fmaxf(mp, t[j].m);
    }
    // equal maxima (including empty -inf partials) must not evaluate inf - inf
    float sum = acc.m == mp ? acc.s : acc.s * __expf(acc.m - mp);
    int a = acc.m == mp ? acc.a : 0x7fffffff;
#pragma unroll
    for (int j = 0; j < UN; j++) {
        sum += t[j].m == mp ? t[j].s : t[j].s * __expf(t[j].m - mp);
        a = t[j].m == mp && t[j].a < a ? t[j].a : a;         // lowest token id among equal maxima
    }
    return Stat{mp, sum, a};
}

// The same for groups of four partials (48 contiguous bytes: three 16-byte loads per lane instead of twelve
// 4-byte loads at a 12-byte stride, which the address unit of the one compute unit this kernel runs on serves
// at a fraction of the rate).  p must be 16-byte aligned.
template <int UG>
__device__ __forceinline__ Stat merge_partials_pass4(const float *p, int g0, int n_grp, int lane, Stat acc) {
    f32x4 v[UG][3];
#pragma unroll
    for (int j = 0; j < UG; j++) {
        const int g = g0 + lane + 64 * j;
        if (g < n_grp) {
            const f32x4 *q = reinterpret_cast<const f32x4 *>(p + (size_t)g * 12);
            v[j][0] = q[0]; v[j][1] = q[1]; v[j][2] = q[2];
        } else {
            const float e = __int_as_float(0x7fffffff);          // empty partials: (-inf, 0, no id)
            v[j][0] = f32x4{-INFINITY, 0.f, e, -INFINITY};
            v[j][1] = f32x4{0.f, e, -INFINITY, 0.f};
            v[j][2] = f32x4{e, -INFINITY, 0.f, e};
        }
    }
    Stat t[UG * 4];
    float mp = acc.m;
#pragma unroll
    for (int j = 0; j < UG; j++) {
        t[4 * j + 0] = Stat{v[j][0][0], v[j][0][1], __float_as_int(v[j][0][2])};
        t[4 * j + 1] = Stat{v[j][0][3], v[j][1][0], __float_as_int(v[j][1][1])};
        t[4 * j + 2] = Stat{v[j][1][2], v[j][1][3], __float_as_int(v[j][2][0])};
        t[4 * j + 3] = Stat{v[j][2][1], v[j][2][2], __float_as_int(v[j][2][3])};
#pragma unroll
        for (int k = 0; k < 4; k++) mp = fmaxf(mp, t[4 * j + k].m);
    }
    float sum = acc.m == mp ? acc.s : acc.s * __expf(acc.m - mp);
    int a = acc.m == mp ? acc.a : 0x7fffffff;
#pragma unroll
    for (int j = 0; j < UG * 4; j++) {
        sum += t[j].m == mp ? t[j].s : t[j].s * __expf(t[j].m - mp);
        a = t[j].m == mp && t[j].a < a ? t[j].a : a;
    }
    return Stat{mp, sum, a};
}

// the whole wave merges the n_part partials of one row (p = first partial of the row); every lane gets the result.
// Each lane folds its partials against their common maximum (the pairwise merge costs two exponentials in a
// dependent chain per partial, and a 1536-partial row of the few-row LM head made this kernel take 22 us on its
// single compute unit); the 64 lane results are combined the same way: wave maximum, one rescale, butterfly sum.
__device__ __forceinline__ Stat merge_row_partials(const float *p, int n_part, int lane) {
    Stat acc = {-INFINITY, 0.f, 0x7fffffff};
    if (n_part % 4 == 0 && (reinterpret_cast<uintptr_t>(p) & 15) == 0) {
        const int n_grp = n_part / 4;
        int g0 = 0;
        for (; n_grp - g0 > 64 * 2; g0 += 64 * 6) acc = merge_partials_pass4<6>(p, g0, n_grp, lane, acc);
        if (g0 < n_grp) acc = merge_partials_pass4<2>(p, g0, n_grp, lane, acc);
    } else {
        int q0 = 0;
        for (; n_part - q0 > 64 * 8; q0 += 64 * 24) acc = merge_partials_pass<24>(p, q0, n_part, lane, acc);
        if (q0 < n_part) acc = merge_partials_pass<8>(p, q0, n_part, lane, acc);
    }
    float wm = acc.m;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) wm = fmaxf(wm, __shfl_xor(wm, o));
    float sum = acc.m == wm ? acc.s : acc.s * __expf(acc.m - wm);
    int a = acc.m == wm ? acc.a : 0x7fffffff;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        sum += __shfl_xor(sum, o);                              // commutative: every lane ends with the same bits
        const int oa = __shfl_xor(a, o);
        a = oa < a ? oa : a;
    }
    return Stat{wm, sum, a};
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
