// Row-wise kernels: embedding gather, RMSNorm into the tiled operand layout,
// and the final reduction of the LM-head statistics with the threshold unmask.
#include "rows_core.h"

namespace odb {

__global__ void embed_kernel(const u16 *embed, const int32_t *tokens, RowMap rm, int d, int vocab, float *h,
                             NormOut no, int mt_total) {
    embed_row(blockIdx.x, embed, tokens, rm, d, vocab, h, no, mt_total);
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
            f.w[0] = pack2(a.x * rstd * ga.x, a.y * rstd * ga.y);
            f.w[1] = pack2(a.z * rstd * ga.z, a.w * rstd * ga.w);
            f.w[2] = pack2(b.x * rstd * gb.x, b.y * rstd * gb.y);
            f.w[3] = pack2(b.z * rstd * gb.z, b.w * rstd * gb.w);
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

__global__ __launch_bounds__(1024) void lm_finish_kernel(const float *stats, int n_part, int rows, int rpu, int rpu_pad,
                                                        const int32_t *tokens, int mask_id, float tau, float *conf,
                                                        int32_t *argmax, uint8_t *unmask) {
    __shared__ float s_conf[256];
    lm_finish_wg(blockIdx.x, stats, n_part, rows, rpu, rpu_pad, tokens, mask_id, tau, conf, argmax, unmask, s_conf);
}

void launch_lm_finish(const float *stats, int n_part, int rows, int rpu, int rpu_pad, const int32_t *tokens,
                      int mask_id, float tau, float *conf, int32_t *argmax, uint8_t *unmask, hipStream_t s) {
    int units = (rows + rpu - 1) / rpu;
    lm_finish_kernel<<<dim3(units), 1024, 0, s>>>(stats, n_part, rows, rpu, rpu_pad, tokens, mask_id, tau, conf,
                                                 argmax, unmask);
}

// Adaptive length prediction (ODB-dLLM Sec. 4.1): one workgroup per sequence scans the response for the
// earliest position whose drafted token is [EOS] - an attempted one (position still MASK) must exceed the
// truncate threshold, a decoded one counts as it stands - and writes the length that keeps it as last position.
__global__ __launch_bounds__(256) void predict_length_kernel(const int32_t *tokens, const float *conf,
                                                             const int32_t *argmax, int L, int resp_off, int mask_id,
                                                             int eos_id, float thr, int32_t *new_len) {
    __shared__ int s_min[4];
    const int b = blockIdx.x, R = L - resp_off;
    const int32_t *tok = tokens + (size_t)b * L + resp_off;
    const float *c = conf + (size_t)b * R;
    const int32_t *a = argmax + (size_t)b * R;
    int best = R;                                   // index of the earliest hit seen by this thread
    for (int i = threadIdx.x; i < R; i += blockDim.x) {
        const int t = tok[i];
        const bool hit = t == mask_id ? (a[i] == eos_id && c[i] > thr) : t == eos_id;
        if (hit) { best = i; break; }               // this thread's indices only grow
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) best = min(best, __shfl_xor(best, o));
    if ((threadIdx.x & 63) == 0) s_min[threadIdx.x >> 6] = best;
    __syncthreads();
    if (threadIdx.x == 0) {
        best = min(min(s_min[0], s_min[1]), min(s_min[2], s_min[3]));
        new_len[b] = best < R ? resp_off + best + 1 : L;
    }
}

void launch_predict_length(const int32_t *tokens, const float *conf, const int32_t *argmax, int batch, int L,
                           int resp_off, int mask_id, int eos_id, float thr, int32_t *new_len, hipStream_t s) {
    predict_length_kernel<<<dim3(batch), 256, 0, s>>>(tokens, conf, argmax, L, resp_off, mask_id, eos_id, thr, new_len);
}

}  // namespace odb
