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
                                                      int skip, int compact, int dst_rows, int dst_mt_total, u16 *xa,
                                                      unsigned *status) {
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
            note_saturation(status, a.x * rstd * ga.x, a.y * rstd * ga.y, a.z * rstd * ga.z, a.w * rstd * ga.w);
            note_saturation(status, b.x * rstd * gb.x, b.y * rstd * gb.y, b.z * rstd * gb.z, b.w * rstd * gb.w);
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
                    int dst_mt_total, u16 *xa, unsigned *status, hipStream_t s) {
    int dst_rows = compact ? rm.units * (rm.valid - skip) : rm.units * rm.rpu_pad;
    int padded = dst_mt_total * 16;
    rmsnorm_kernel<<<dim3((padded + 3) / 4), 256, 0, s>>>(h, gain, eps, d, rm, skip, compact ? 1 : 0, dst_rows,
                                                          dst_mt_total, xa, status);
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

// ---- decoded-share step (ODB-dLLM Sec. 4.2.2): row bookkeeping and the finish ----------------------
// One wave per sequence builds the tables of SharedMap from the drafts (see model.h) and presets the
// outputs of the positions of the speculative blocks that are not computed.
__global__ __launch_bounds__(64) void shared_setup_kernel(const int32_t *drafts, SharedMap sm, int block_off, int mask_id,
                                                          int m_cap, float *conf, int32_t *argmax, uint8_t *unmask,
                                                          unsigned int *status) {
    const int seq = blockIdx.x, lane = threadIdx.x, b = sm.b, S = sm.S;
    const int32_t *d0 = drafts + (size_t)seq * S * b;
    // b <= 64: lane i looks at position i of block_0
    const bool in = lane < b, masked = in && d0[lane] == mask_id;
    const unsigned long long mm = __ballot(masked), dm = __ballot(in && !masked);
    const int m = __popcll(mm);
    if (lane == 0) {
        sm.mcount[seq] = m < m_cap ? m : m_cap;
        sm.dmask[seq] = dm;
        if (m > m_cap) atomicOr(status, 2u);
    }
    // block_0: bp rows, row i = position i
    const int rowA = seq * sm.bp;
    for (int i = lane; i < sm.bp; i += 64) {
        sm.rowtok[rowA + i] = i < b ? d0[i] : 0;
        sm.rowpos[rowA + i] = block_off + (i < b ? i : 0);
        sm.rowout[rowA + i] = i < b ? (seq * S + 0) * b + i : -1;
    }
    // pooled speculative unit: row j = block 1 + j / mc, its (j % mc)-th masked position; rows past the last
    // block are padding (token 0 at the block's first position, no output)
    const int mc = m < m_cap ? m : m_cap;
    const int rowB = sm.batch * sm.bp + seq * sm.mp;
    for (int j = lane; j < sm.mp; j += 64) {
        const int s = mc > 0 ? 1 + j / mc : S, r = mc > 0 ? j % mc : 0;
        int tok = 0, pos = 0, out = -1;
        if (s < S) {
            unsigned long long t = mm;
            for (int k = 0; k < r; k++) t &= t - 1;                  // drop the r lowest set bits
            pos = __ffsll(t) - 1;                                    // the r-th masked position (r < mc <= m)
            tok = d0[(size_t)s * b + pos];
            out = (seq * S + s) * b + pos;
        }
        sm.rowtok[rowB + j] = tok;
        sm.rowpos[rowB + j] = block_off + pos;
        sm.rowout[rowB + j] = out;
    }
    // decoded positions of the speculative blocks are not computed: they read as "nothing to decide here"
    if (in && !masked)
        for (int s = 1; s < S; s++) {
            const size_t o = (size_t)(seq * S + s) * b + lane;
            if (conf) conf[o] = 0.f;
            if (argmax) argmax[o] = d0[(size_t)s * b + lane];
            if (unmask) unmask[o] = 0;
        }
}

void launch_shared_setup(const int32_t *drafts, SharedMap sm, int block_off, int mask_id, int m_cap, float *conf,
                         int32_t *argmax, uint8_t *unmask, unsigned int *status, hipStream_t s) {
    shared_setup_kernel<<<dim3(sm.batch), 64, 0, s>>>(drafts, sm, block_off, mask_id, m_cap, conf, argmax, unmask, status);
}

// One workgroup per unit (block_0 of a sequence, or one of its speculative blocks): confidence and greedy token
// of every real row, then the acceptance rule over the unit's rows that still hold MASK; results are scattered
// to their positions in the [batch, S, b] outputs.
__global__ __launch_bounds__(512) void lm_finish_shared_kernel(const float *stats, int n_part, SharedMap sm, int mask_id,
                                                               float tau, float *conf, int32_t *argmax, uint8_t *unmask) {
    __shared__ float s_conf[64];
    const int u = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    const bool spec = u >= sm.batch;
    const int seq = spec ? (u - sm.batch) / (sm.S - 1) : u, blk = spec ? (u - sm.batch) % (sm.S - 1) : 0;
    const int nrows = spec ? sm.mcount[seq] : sm.b;
    const int row0 = spec ? sm.batch * sm.bp + seq * sm.mp + blk * nrows : u * sm.bp;
    for (int i = wave; i < nrows; i += nw) {
        const Stat acc = merge_row_partials(stats + (size_t)(row0 + i) * n_part * 3, n_part, lane);
        if (lane == 0) {
            const float c = 1.0f / acc.s;
            const int o = sm.rowout[row0 + i];
            conf[o] = c;
            argmax[o] = acc.a;
            s_conf[i] = c;
        }
    }
    __syncthreads();
    if (wave == 0) {
        float best = -1.f;
        int best_i = 0x7fffffff;
        const bool masked = lane < nrows && sm.rowtok[row0 + lane] == mask_id;
        if (masked) { best = s_conf[lane]; best_i = lane; }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            float ob = __shfl_xor(best, o);
            int oi = __shfl_xor(best_i, o);
            if (ob > best || (ob == best && oi < best_i)) { best = ob; best_i = oi; }
        }
        if (lane < nrows) unmask[sm.rowout[row0 + lane]] = (masked && (s_conf[lane] > tau || lane == best_i)) ? 1 : 0;
    }
}

void launch_lm_finish_shared(const float *stats, int n_part, SharedMap sm, int mask_id, float tau, float *conf,
                             int32_t *argmax, uint8_t *unmask, hipStream_t s) {
    lm_finish_shared_kernel<<<dim3(sm.batch * sm.S), 512, 0, s>>>(stats, n_part, sm, mask_id, tau, conf, argmax, unmask);
}

// Accept-jump controller (ODB-dLLM Sec. 4.2.1), one wave per sequence.  Inputs are the four drafts of a
// block step (block_0; B unmasked; D unmasked; both) and that step's outputs.  A candidate is verified in a
// draft when the draft's step unmasks its position with the speculated token.  Both verified in block_0 ->
// block_3; only one -> the draft that had it unmasked beforehand, and on to block_3 if the other one is
// verified there; neither -> block_0.  The adopted draft plus its step's unmaskings is the new block; its
// two most confident still-masked positions (lower index first on ties) become the next candidates.
struct Cand { float c; int i; };
__device__ inline bool cand_better(Cand a, Cand b) { return a.c > b.c || (a.c == b.c && a.i < b.i); }
__device__ inline void cand_push(Cand &x0, Cand &x1, Cand y) {         // keeps the two best, x0 the better
    if (cand_better(y, x0)) { x1 = x0; x0 = y; }
    else if (cand_better(y, x1)) x1 = y;
}

__global__ __launch_bounds__(64) void accept_jump_kernel(const int32_t *drafts, const float *conf, const int32_t *argmax,
                                                         const uint8_t *unmask, const int32_t *cand_pos,
                                                         const int32_t *cand_tok, int b, int mask_id, int32_t *chosen_out,
                                                         int32_t *new_drafts, int32_t *new_cand_pos, int32_t *new_cand_tok) {
    const int seq = blockIdx.x, lane = threadIdx.x;
    const size_t base = (size_t)seq * 4 * b;
    const int32_t *dr = drafts + base, *am = argmax + base;
    const float *cf = conf + base;
    const uint8_t *um = unmask + base;
    const int p0 = cand_pos[seq * 2], p1 = cand_pos[seq * 2 + 1], t0 = cand_tok[seq * 2], t1 = cand_tok[seq * 2 + 1];
    auto verified = [&](int s, int p, int t) {
        return p >= 0 && p < b && dr[s * b + p] == mask_id && um[s * b + p] != 0 && am[s * b + p] == t;
    };
    const bool b0 = verified(0, p0, t0), d0 = verified(0, p1, t1);
    int ch;
    if (b0 && d0) ch = 3;
    else if (b0) ch = verified(1, p1, t1) ? 3 : 1;
    else if (d0) ch = verified(2, p0, t0) ? 3 : 2;
    else ch = 0;

    // the new block, and this lane's two best still-masked positions
    const Cand none{-INFINITY, 0x7fffffff};
    Cand x0 = none, x1 = none;
    int32_t *nd = new_drafts + base;
    for (int i = lane; i < b; i += 64) {
        const int t = um[ch * b + i] ? am[ch * b + i] : dr[ch * b + i];
        nd[i] = t;
        if (t == mask_id) cand_push(x0, x1, Cand{cf[ch * b + i], i});
    }
    // the two best of the wave: butterfly over the lanes, every lane ends with the same pair
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        Cand y0{__shfl_xor(x0.c, o), __shfl_xor(x0.i, o)}, y1{__shfl_xor(x1.c, o), __shfl_xor(x1.i, o)};
        cand_push(x0, x1, y0);
        cand_push(x0, x1, y1);
    }
    const int q0 = x0.i != 0x7fffffff ? x0.i : -1, q1 = x1.i != 0x7fffffff ? x1.i : -1;
    const int u0 = q0 >= 0 ? am[ch * b + q0] : 0, u1 = q1 >= 0 ? am[ch * b + q1] : 0;
    if (lane == 0) {
        chosen_out[seq] = ch;
        new_cand_pos[seq * 2] = q0; new_cand_pos[seq * 2 + 1] = q1;
        new_cand_tok[seq * 2] = u0; new_cand_tok[seq * 2 + 1] = u1;
    }
    // block_1 .. block_3 of the next step (each lane rewrites the positions it wrote above, so no lane reads
    // another lane's stores)
    for (int i = lane; i < b; i += 64) {
        const int t = nd[i];
        nd[b + i] = i == q0 ? u0 : t;
        nd[2 * b + i] = i == q1 ? u1 : t;
        nd[3 * b + i] = i == q0 ? u0 : (i == q1 ? u1 : t);
    }
}

// The k <= 4 most confident positions of blk[0 .. bb) that hold MASK, best first, lower index first on equal
// confidence; -1 where fewer are left.  One wave; every lane ends with the same q.  (A lane only reads the
// positions lane, lane + 64, ... of blk: the ones it may have written itself just before.)
__device__ inline void top_masked(const int32_t *blk, const float *conf, int bb, int mask_id, int k, int (&q)[4]) {
    const int lane = threadIdx.x;
#pragma unroll
    for (int r = 0; r < 4; r++) {
        q[r] = -1;
        if (r < k) {
            Cand best{-INFINITY, 0x7fffffff};
            for (int i = lane; i < bb; i += 64) {
                bool taken = false;
#pragma unroll
                for (int j = 0; j < 4; j++) taken = taken || (j < r && q[j] == i);
                const Cand y{conf[i], i};
                if (!taken && blk[i] == mask_id && cand_better(y, best)) best = y;
            }
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) {
                const Cand y{__shfl_xor(best.c, o), __shfl_xor(best.i, o)};
                if (cand_better(y, best)) best = y;
            }
            q[r] = best.i != 0x7fffffff ? best.i : -1;
        }
    }
}

// Candidate sets of the up to eight blocks of a step as bit masks over the ranked candidates (ODB-dLLM
// Sec. 4.2.1: block_0, B, D, B + D; Sec. 4.2.2: the third, the top three, the fourth, the top four).
__device__ __constant__ int kSpecSets[8] = {0, 1, 2, 3, 4, 7, 8, 15};

// block s of the next step: the block with the candidates of its set unmasked beforehand
__device__ inline int spec_token(int s, int i, int t, const int (&q)[4], const int (&u)[4]) {
#pragma unroll
    for (int c = 0; c < 4; c++)
        if (((kSpecSets[s] >> c) & 1) && q[c] == i) t = u[c];
    return t;
}

// The jump rule over S = 4 or 8 blocks, one wave per sequence.  From block_0: at a block with candidate set X the
// verified set is X plus the candidates that this block's own step unmasks with the speculated token; the block
// whose set lies strictly above X inside the verified set and holds the most candidates (lowest number among
// equals) is next, and the walk ends where there is none.  For S = 4 this is the rule of Sec. 4.2.1 (the paper
// states none for eight blocks).  The adopted block plus its step's unmaskings is the new block; its n_next / 2
// most confident still-masked positions become the candidates of the n_next blocks written to new_drafts.
__global__ __launch_bounds__(64) void spec_jump_kernel(const int32_t *drafts, const float *conf, const int32_t *argmax,
                                                       const uint8_t *unmask, const int32_t *cand_pos,
                                                       const int32_t *cand_tok, int S, int n_next, int b, int mask_id,
                                                       int32_t *chosen_out, int32_t *new_drafts, int32_t *new_cand_pos,
                                                       int32_t *new_cand_tok) {
    const int seq = blockIdx.x, lane = threadIdx.x;
    const size_t base = (size_t)seq * S * b;
    const int32_t *dr = drafts + base, *am = argmax + base;
    const float *cf = conf + base;
    const uint8_t *um = unmask + base;
    const int n_cand = S / 2;
    int p[4], t[4];
#pragma unroll
    for (int c = 0; c < 4; c++) {
        p[c] = c < n_cand ? cand_pos[seq * 4 + c] : -1;
        t[c] = c < n_cand ? cand_tok[seq * 4 + c] : 0;
    }
    int ch = 0;
    for (int hop = 0; hop < 4; hop++) {
        const int X = kSpecSets[ch];
        int V = X;
#pragma unroll
        for (int c = 0; c < 4; c++) {
            const int pc = p[c];
            if (!((X >> c) & 1) && pc >= 0 && pc < b && dr[ch * b + pc] == mask_id && um[ch * b + pc] != 0 &&
                am[ch * b + pc] == t[c])
                V |= 1 << c;
        }
        int best = -1, best_n = __popc(X);
        for (int s = 0; s < S; s++) {
            const int m = kSpecSets[s];
            if ((m & ~V) == 0 && (m & X) == X && m != X && __popc(m) > best_n) { best = s; best_n = __popc(m); }
        }
        if (best < 0) break;
        ch = best;
    }

    int32_t *nd = new_drafts + (size_t)seq * n_next * b;
    for (int i = lane; i < b; i += 64) nd[i] = um[ch * b + i] ? am[ch * b + i] : dr[ch * b + i];
    int q[4], u[4];
    top_masked(nd, cf + ch * b, b, mask_id, n_next / 2, q);
#pragma unroll
    for (int c = 0; c < 4; c++) u[c] = q[c] >= 0 ? am[ch * b + q[c]] : 0;
    if (lane == 0) {
        chosen_out[seq] = ch;
#pragma unroll
        for (int c = 0; c < 4; c++) { new_cand_pos[seq * 4 + c] = q[c]; new_cand_tok[seq * 4 + c] = u[c]; }
    }
    for (int i = lane; i < b; i += 64) {
        const int tk = nd[i];
        for (int s = 1; s < n_next; s++) nd[s * b + i] = spec_token(s, i, tk, q, u);
    }
}

// ---- generation loop bookkeeping (ODB-dLLM Sec. 2.1 / 4.1 / 4.2.1), one wave ------------------------
// ctl words written for the host: [0] sequence length, [1] MASK positions left in the block, [2] adopted
// draft, [3..4] positions of candidates B and D, [5..6] their tokens, [7] length of the block, [9..10] positions
// of the third and fourth candidate, [11..12] their tokens ([8] belongs to the length prediction).
//
// Adoption of one forward's attempt at the current block.  The block is tokens[off .. off+bb) with
// bb = min(b, len - off), len read from len_ptr (the length prediction's output) when given.  Position i
// takes argmax[i] if unmask[i] (a step's own decision) or, without an unmask array (a refresh), if it holds
// MASK and its confidence exceeds tau or is the largest among the block's MASK positions (lower index on
// ties).  The two (n_build = 8: four) most confident positions still MASK afterwards become the candidates
// (cand: four positions, then four tokens), and with drafts given the block and its n_build - 1 speculative
// variants are written there.
__global__ __launch_bounds__(64) void gen_adopt_kernel(int32_t *tokens, int off, int b, const int32_t *len_ptr, int len,
                                                       const float *conf, const int32_t *argmax, const uint8_t *unmask,
                                                       int mask_id, float tau, int32_t *drafts, int n_build, int32_t *cand,
                                                       int32_t *ctl) {
    const int lane = threadIdx.x;
    if (len_ptr) len = *len_ptr;
    const int bb = min(b, len - off);
    if (bb <= 0) {
        if (lane == 0) {
            ctl[0] = len; ctl[1] = 0; ctl[2] = 0; ctl[3] = ctl[4] = -1; ctl[5] = ctl[6] = 0; ctl[7] = 0;
            ctl[9] = ctl[10] = -1; ctl[11] = ctl[12] = 0;
        }
        return;
    }
    int32_t *blk = tokens + off;
    const Cand none{-INFINITY, 0x7fffffff};
    int forced = -1;
    if (!unmask) {
        Cand f = none, f1 = none;
        for (int i = lane; i < bb; i += 64)
            if (blk[i] == mask_id) cand_push(f, f1, Cand{conf[i], i});
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) cand_push(f, f1, Cand{__shfl_xor(f.c, o), __shfl_xor(f.i, o)});
        forced = f.i;
    }
    int left = 0;
    for (int i = lane; i < bb; i += 64) {
        const int t0 = blk[i];
        const bool take = unmask ? unmask[i] != 0 : (t0 == mask_id && (conf[i] > tau || i == forced));
        const int t = take ? argmax[i] : t0;
        blk[i] = t;
        left += t == mask_id;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) left += __shfl_xor(left, o);
    int q[4], u[4];
    top_masked(blk, conf, bb, mask_id, n_build == 8 ? 4 : 2, q);
#pragma unroll
    for (int c = 0; c < 4; c++) u[c] = q[c] >= 0 ? argmax[q[c]] : 0;
    if (lane == 0) {
        ctl[0] = len; ctl[1] = left; ctl[2] = 0; ctl[3] = q[0]; ctl[4] = q[1]; ctl[5] = u[0]; ctl[6] = u[1]; ctl[7] = bb;
        ctl[9] = q[2]; ctl[10] = q[3]; ctl[11] = u[2]; ctl[12] = u[3];
        if (cand)
#pragma unroll
            for (int c = 0; c < 4; c++) { cand[c] = q[c]; cand[4 + c] = u[c]; }
    }
    if (drafts)     // each lane re-reads only the positions it wrote itself
        for (int i = lane; i < bb; i += 64) {
            const int t = blk[i];
            for (int s = 0; s < n_build; s++) drafts[s * bb + i] = spec_token(s, i, t, q, u);
        }
}

// After the accept-jump controller: the adopted block (new_drafts[0]) goes back into the sequence and the
// controller's decision is packed for the host.
__global__ __launch_bounds__(64) void gen_commit_kernel(int32_t *tokens, int off, int bb, int len, const int32_t *new_drafts,
                                                        const int32_t *chosen, const int32_t *cand, int mask_id,
                                                        int32_t *ctl) {
    const int lane = threadIdx.x;
    int left = 0;
    for (int i = lane; i < bb; i += 64) {
        const int t = new_drafts[i];
        tokens[off + i] = t;
        left += t == mask_id;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) left += __shfl_xor(left, o);
    if (lane == 0) {
        ctl[0] = len; ctl[1] = left; ctl[2] = chosen[0];
        ctl[3] = cand[0]; ctl[4] = cand[1]; ctl[5] = cand[4]; ctl[6] = cand[5]; ctl[7] = bb;
        ctl[9] = cand[2]; ctl[10] = cand[3]; ctl[11] = cand[6]; ctl[12] = cand[7];
    }
}

void launch_gen_adopt(int32_t *tokens, int off, int b, const int32_t *len_ptr, int len, const float *conf,
                      const int32_t *argmax, const uint8_t *unmask, int mask_id, float tau, int32_t *drafts, int n_build,
                      int32_t *cand, int32_t *ctl, hipStream_t s) {
    gen_adopt_kernel<<<1, 64, 0, s>>>(tokens, off, b, len_ptr, len, conf, argmax, unmask, mask_id, tau, drafts, n_build, cand,
                                      ctl);
}

void launch_spec_jump(const int32_t *drafts, const float *conf, const int32_t *argmax, const uint8_t *unmask,
                      const int32_t *cand_pos, const int32_t *cand_tok, int batch, int S, int n_next, int b, int mask_id,
                      int32_t *chosen, int32_t *new_drafts, int32_t *new_cand_pos, int32_t *new_cand_tok, hipStream_t s) {
    spec_jump_kernel<<<dim3(batch), 64, 0, s>>>(drafts, conf, argmax, unmask, cand_pos, cand_tok, S, n_next, b, mask_id, chosen,
                                                new_drafts, new_cand_pos, new_cand_tok);
}

void launch_gen_commit(int32_t *tokens, int off, int bb, int len, const int32_t *new_drafts, const int32_t *chosen,
                       const int32_t *cand, int mask_id, int32_t *ctl, hipStream_t s) {
    gen_commit_kernel<<<1, 64, 0, s>>>(tokens, off, bb, len, new_drafts, chosen, cand, mask_id, ctl);
}

void launch_accept_jump(const int32_t *drafts, const float *conf, const int32_t *argmax, const uint8_t *unmask,
                        const int32_t *cand_pos, const int32_t *cand_tok, int batch, int b, int mask_id, int32_t *chosen,
                        int32_t *new_drafts, int32_t *new_cand_pos, int32_t *new_cand_tok, hipStream_t s) {
    accept_jump_kernel<<<dim3(batch), 64, 0, s>>>(drafts, conf, argmax, unmask, cand_pos, cand_tok, b, mask_id, chosen,
                                                  new_drafts, new_cand_pos, new_cand_tok);
}

void launch_predict_length(const int32_t *tokens, const float *conf, const int32_t *argmax, int batch, int L,
                           int resp_off, int mask_id, int eos_id, float thr, int32_t *new_len, hipStream_t s) {
    predict_length_kernel<<<dim3(batch), 256, 0, s>>>(tokens, conf, argmax, L, resp_off, mask_id, eos_id, thr, new_len);
}

}  // namespace odb
