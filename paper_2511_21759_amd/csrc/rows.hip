// Row-wise kernels: embedding gather, RMSNorm into the tiled operand layout,
// and the final reduction of the LM-head statistics with the threshold unmask.
#include "model.h"

namespace odb {

// h[r, :] = E[token(r), :] as fp32 (the residual stream stays in fp32).  One thread per 16 columns.
__global__ void embed_kernel(const u16 *embed, const int32_t *tokens, RowMap rm, int d, int vocab, float *h,
                             NormOut no, int mt_total) {
    int r = blockIdx.x;
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
                    f.w[j] = pack2bf(x[half * 8 + 2 * j] * gn[half * 8 + 2 * j],
                                     x[half * 8 + 2 * j + 1] * gn[half * 8 + 2 * j + 1]);
                const int chunk = (nt & 1) * 2 + half;
                *reinterpret_cast<frag_t *>(no.hb + ((size_t)(nt >> 1) * mt_total + (r >> 4)) * kTileElems +
                                            (chunk * 16 + (r & 15)) * 8) = f;
            }
        }
    }
}

void launch_embed(const Model &m, const int32_t *tokens, RowMap rm, float *h, NormOut no, hipStream_t s) {
    int rows = rm.units * rm.rpu_pad;
    int threads = m.cfg.d_model / 16 < 256 ? 64 : 256;
    embed_kernel<<<dim3(rows), threads, 0, s>>>(m.w[PK_EMBED], tokens, rm, m.cfg.d_model, m.cfg.vocab, h, no,
                                                rows / 16);
}

__device__ inline float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// One wave per destination row.  xa tile (kt, mt) holds rows 16*mt.., k 32*kt.. .
__global__ __launch_bounds__(256) void rmsnorm_kernel(const float *h, const float *gain, float eps, int d, RowMap rm,
                                                      int skip, int compact, int dst_rows, int dst_mt_total, u16 *xa) {
    int lane = threadIdx.x & 63;
    int j = blockIdx.x * 4 + (threadIdx.x >> 6);          // destination row
    if (j >= dst_mt_total * 16) return;
    int n_chunks = d / 8;
    int mt = j >> 4, r = j & 15;
    bool live = j < dst_rows;
    size_t src = j;
    if (compact && live) {
        int per = rm.valid - skip;
        src = (size_t)(j / per) * rm.rpu_pad + skip + (j % per);
    }
    const float *x = h + src * d;
    float ss = 0.f;
    if (live) {
        for (int q = lane; q < n_chunks; q += 64) {
            float4 a = *reinterpret_cast<const float4 *>(x + q * 8);
            float4 b = *reinterpret_cast<const float4 *>(x + q * 8 + 4);
            ss += a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w + b.x * b.x + b.y * b.y + b.z * b.z + b.w * b.w;
        }
    }
    ss = wave_sum(ss);
    float rstd = 1.0f / sqrtf(ss / (float)d + eps);
    for (int q = lane; q < n_chunks; q += 64) {
        frag_t f = {{0, 0, 0, 0}};
        if (live) {
            float4 a = *reinterpret_cast<const float4 *>(x + q * 8);
            float4 b = *reinterpret_cast<const float4 *>(x + q * 8 + 4);
            float4 ga = *reinterpret_cast<const float4 *>(gain + q * 8);
            float4 gb = *reinterpret_cast<const float4 *>(gain + q * 8 + 4);
            f.w[0] = pack2bf(a.x * rstd * ga.x, a.y * rstd * ga.y);
            f.w[1] = pack2bf(a.z * rstd * ga.z, a.w * rstd * ga.w);
            f.w[2] = pack2bf(b.x * rstd * gb.x, b.y * rstd * gb.y);
            f.w[3] = pack2bf(b.z * rstd * gb.z, b.w * rstd * gb.w);
        }
        int kt = q >> 2, kg = q & 3;
        *reinterpret_cast<frag_t *>(xa + ((size_t)kt * dst_mt_total + mt) * kTileElems + (kg * 16 + r) * 8) = f;
    }
}

void launch_rmsnorm(const float *h, const float *gain, float eps, int d, RowMap rm, int skip, bool compact,
                    int dst_mt_total, u16 *xa, hipStream_t s) {
    int dst_rows = compact ? rm.units * (rm.valid - skip) : rm.units * rm.rpu_pad;
    int padded = dst_mt_total * 16;
    rmsnorm_kernel<<<dim3((padded + 3) / 4), 256, 0, s>>>(h, gain, eps, d, rm, skip, compact ? 1 : 0, dst_rows,
                                                          dst_mt_total, xa);
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

__global__ __launch_bounds__(256) void lm_finish_kernel(const float *stats, int n_part, int rows, int rpu, int rpu_pad,
                                                        const int32_t *tokens, int mask_id, float tau, float *conf,
                                                        int32_t *argmax, uint8_t *unmask) {
    __shared__ float s_conf[256];
    int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int u = blockIdx.x;
    for (int i = wave; i < rpu; i += 4) {
        int row = u * rpu + i;                                  // compact output row
        if (row >= rows) break;
        const float *p = stats + ((size_t)u * rpu_pad + i) * n_part * 3;
        Stat acc = {-INFINITY, 0.f, 0x7fffffff};
        for (int q = lane; q < n_part; q += 64) {
            Stat t = {p[q * 3], p[q * 3 + 1], __float_as_int(p[q * 3 + 2])};
            acc = merge(acc, t);
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            Stat t = {__shfl_xor(acc.m, o), __shfl_xor(acc.s, o), __shfl_xor(acc.a, o)};
            acc = merge(acc, t);
        }
        if (lane == 0) {
            float c = 1.0f / acc.s;
            if (conf) conf[row] = c;
            if (argmax) argmax[row] = acc.a;
            s_conf[i & 255] = c;
        }
    }
    if (!unmask) return;
    __syncthreads();
    if (wave != 0) return;
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

void launch_lm_finish(const float *stats, int n_part, int rows, int rpu, int rpu_pad, const int32_t *tokens,
                      int mask_id, float tau, float *conf, int32_t *argmax, uint8_t *unmask, hipStream_t s) {
    int units = (rows + rpu - 1) / rpu;
    lm_finish_kernel<<<dim3(units), 256, 0, s>>>(stats, n_part, rows, rpu, rpu_pad, tokens, mask_id, tau, conf,
                                                 argmax, unmask);
}

}  // namespace odb
