// Host-side structures of the library and the prototypes of the kernel
// launchers that the API layer (api.hip) strings together.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/odb.h"
#include "common.h"

namespace odb {

// ---- physical layouts -----------------------------------------------------
// W_qkv  [3d, d]  tiles [n_tile][k_tile]; rows 0..d-1 = Wq, d..2d-1 = Wk with
//                 the channels of each head interleaved (physical 2j -> channel
//                 j, 2j+1 -> channel j + dh/2) so that a RoPE pair sits in one
//                 lane of the GEMM result; rows 2d..3d-1 = Wv in logical order.
// W_o    [d, d], W_d [d, F], W_lm [V, d]: logical row order, tiles [n_tile][k_tile].
// W_gu   [2F, d]: physical row 2j = row j of W_gate, 2j+1 = row j of W_up, so a
//                 lane of the GEMM result holds (gate, up) pairs.
// E      [V, d] plain row-major (gathered by row).
enum PhysKind { PK_QKV = 0, PK_O, PK_GU, PK_D, PK_LM, PK_EMBED, PK_COUNT };

struct Model {
    odb_config cfg;
    odb_allocator alloc;
    bool has_alloc;
    int device;
    u16 *w[PK_COUNT];          // per kind, all layers contiguous
    size_t layer_elems[PK_COUNT];
    float *g1, *g2, *gf;       // [NL][d], [NL][d], [d]
    // scratch, grown on demand (see api.hip)
    void *scratch;
    size_t scratch_bytes;
    unsigned *counters;        // [0] status word (kStatus* bits), [1024..2048) arrival counters of the K-split GEMM
    bool ksplit_reduce;        // the K-split streaming GEMM with its in-kernel reduction may be used (ODB_OPT_KSPLIT_REDUCE)
    int n_cu;
    u16 *staging;              // set/get tensor staging
    size_t staging_bytes;
    // optional per-kernel-class timing (odb_profile_begin / odb_profile_end)
    int prof_class, prof_cap, prof_used;
    hipEvent_t *prof_ev;       // 3 * prof_cap events: before, after, and once more after (an empty pair)
};

struct Cache {
    Model *m;
    int batch, max_len, lmax32, length;
    u16 *k, *v;                // [NL][B][H][lmax32/16][dh/32][512], [NL][B][H][lmax32/32][dh/16][512]
    float *rope;               // [lmax32][dh/2][2] = (cos, sin)
    size_t layer_elems;        // B*H*lmax32*dh
};

// ---- weights.hip ------------------------------------------------------------
void launch_init_random(const Model &m, uint64_t seed, double std, hipStream_t s);
// copy between a logical row-major bf16 staging buffer (device) and the physical layout
void launch_tensor_copy(const Model &m, int tensor_id, int layer, u16 *staging, bool to_model, hipStream_t s);
void launch_gain_copy(float *gain, u16 *staging, int n, bool to_model, hipStream_t s);
void launch_fill_f32(float *p, float v, size_t n, hipStream_t s);
void launch_fill_i32(int32_t *p, int32_t v, size_t n, hipStream_t s);
void launch_rope_table(float *table, int n_pos, int dh, double base, hipStream_t s);
void launch_cache_read(const Cache &c, int layer, int kv, int batch_index, int pos0, int n, float *out, hipStream_t s);

// Fused RMSNorm.  NormIn: the GEMM input holds binary16(x * gain) and ssq[row][0..n_ssq) are partial
// sums of x^2 over the row; output rows are scaled by 1/sqrt(sum/d + eps) (ssq == nullptr: off).
// NormOut: the residual epilogue also emits that pair for the next norm (hb == nullptr: off);
// status: the model's status word, where a value beyond the binary16 range is reported (may be nullptr).
struct NormIn { const float *ssq; int n_ssq; float eps; };
struct NormOut { u16 *hb; float *ssq; const float *gain; int n_ssq; unsigned *status; };

// ---- rows.hip ---------------------------------------------------------------
// Row bookkeeping.  Rows are grouped in "units" (a draft in the step, a
// sequence in the prefill) of rpu_pad rows (multiple of 16) of which the first
// `valid` are real.
struct RowMap { int units, rpu_pad, valid; };
// h = E[token] (fp32); with a NormOut also hb = bf16(h * gain) and the per-tile sums of squares
void launch_embed(const Model &m, const int32_t *tokens, RowMap rm, float *h, NormOut no, hipStream_t s);
// xa = bf16(rmsnorm(h) * gain) in tile-major [d/32][mt_total][512]; if `compact`, destination
// row j = u*(valid-skip) + (i-skip) for source row (u, i >= skip), else the same row.
void launch_rmsnorm(const float *h, const float *gain, float eps, int d, RowMap rm, int skip, bool compact,
                    int dst_mt_total, u16 *xa, unsigned *status, hipStream_t s);
// stats rows come in units of rpu_pad rows of which the first rpu are real; the `rows` outputs are compact
void launch_accept_jump(const int32_t *drafts, const float *conf, const int32_t *argmax, const uint8_t *unmask,
                        const int32_t *cand_pos, const int32_t *cand_tok, int batch, int b, int mask_id, int32_t *chosen,
                        int32_t *new_drafts, int32_t *new_cand_pos, int32_t *new_cand_tok, hipStream_t s);
// the jump rule over S = 4 or 8 blocks (cand_pos / cand_tok: four entries per sequence); builds n_next blocks
void launch_spec_jump(const int32_t *drafts, const float *conf, const int32_t *argmax, const uint8_t *unmask,
                      const int32_t *cand_pos, const int32_t *cand_tok, int batch, int S, int n_next, int b, int mask_id,
                      int32_t *chosen, int32_t *new_drafts, int32_t *new_cand_pos, int32_t *new_cand_tok, hipStream_t s);
// generation loop bookkeeping (see rows.hip): adoption of a forward's attempt at the current block, and the
// write-back after the jump controller; both pack ctl[0..13) for the host.  cand = four candidate positions, then
// their four tokens; n_build = blocks written to drafts (4 or 8)
void launch_gen_adopt(int32_t *tokens, int off, int b, const int32_t *len_ptr, int len, const float *conf,
                      const int32_t *argmax, const uint8_t *unmask, int mask_id, float tau, int32_t *drafts, int n_build,
                      int32_t *cand, int32_t *ctl, hipStream_t s);
void launch_gen_commit(int32_t *tokens, int off, int bb, int len, const int32_t *new_drafts, const int32_t *chosen,
                       const int32_t *cand, int mask_id, int32_t *ctl, hipStream_t s);
void launch_predict_length(const int32_t *tokens, const float *conf, const int32_t *argmax, int batch, int L,
                           int resp_off, int mask_id, int eos_id, float thr, int32_t *new_len, hipStream_t s);
void launch_lm_finish(const float *stats, int n_part, int rows, int rpu, int rpu_pad, const int32_t *tokens,
                      int mask_id, float tau, float *conf, int32_t *argmax, uint8_t *unmask, hipStream_t s);
// Decoded-share step: row bookkeeping built on the device from the drafts.  Rows: block_0 of every sequence
// first (batch units of bp rows), then one pooled speculative unit per sequence (mp rows): its S-1 speculative
// blocks one after the other, each the positions that are MASK in block_0, in increasing order (mcount[seq]
// rows per block, so the pooled unit is dense and only its end is padding).
struct SharedMap {
    int batch, S, b, bp, mp;           // bp, mp: rows per unit, multiples of 16
    int32_t *rowtok, *rowpos, *rowout; // per row: token, absolute position, index into [batch, S, b] (-1: padding)
    int32_t *mcount;                   // [batch] masked positions of block_0
    unsigned long long *dmask;         // [batch] bit i set: position i of the block is decoded
    int rows() const { return batch * (bp + mp); }
};
// fills the tables, presets the outputs of the positions that are not computed (conf 0, argmax = token,
// unmask 0) and raises status bit 2 if a block has more than m_cap masked positions
void launch_shared_setup(const int32_t *drafts, SharedMap sm, int block_off, int mask_id, int m_cap, float *conf,
                         int32_t *argmax, uint8_t *unmask, unsigned int *status, hipStream_t s);
void launch_lm_finish_shared(const float *stats, int n_part, SharedMap sm, int mask_id, float tau, float *conf,
                             int32_t *argmax, uint8_t *unmask, hipStream_t s);

// ---- gemm.hip ---------------------------------------------------------------
struct GemmShape { int M_tiles, N_tiles, K_tiles; };
// Division by a run-time constant below 2^16 for dividends below 2^16: q = (x * mul) >> 32 with
// mul = floor(2^32 / div) + 1 is exact there (the error term x * (mul * div - 2^32) stays below 2^32).
struct FastDiv {
    unsigned mul, div;
    __host__ __device__ static FastDiv make(int d) {
        FastDiv f;
        f.div = d > 0 ? (unsigned)d : 1u;
        f.mul = (unsigned)(0x100000000ull / f.div) + 1u;       // (div = 1: wraps to 1 - handled in quot)
        return f;
    }
    __device__ __forceinline__ int quot(int x) const { return div == 1u ? x : (int)__umulhi((unsigned)x, mul); }
};

struct QkvOut {
    u16 *q;                    // [H][mt_total][dh/32][512]
    u16 *k; size_t k_unit_stride, k_head_stride;   // tiles [pos/16][dh/32]
    u16 *v; size_t v_unit_stride, v_head_stride;   // tiles [pos/32][dh/16], keys permuted inside
    const float *rope;         // (cos,sin) table
    unsigned *status;          // the model's status word (saturation of a binary16 conversion), may be nullptr
    int tiles_per_unit, pos_off, H, dh, d;
    FastDiv fd_d, fd_dh, fd_tpu, fd_tpu_b;     // by d / 16, dh / 16, tiles_per_unit, tiles_per_unit_b: set_divisors()
    void set_divisors() {
        fd_d = FastDiv::make(d / 16); fd_dh = FastDiv::make(dh / 16);
        fd_tpu = FastDiv::make(tiles_per_unit); fd_tpu_b = FastDiv::make(tiles_per_unit_b);
    }
    // Decoded-share step (rowpos != nullptr): row r sits at absolute position rowpos[r]; m-tiles from
    // split_tile on belong to the speculative units (tiles_per_unit_b each), whose fresh K/V go to k_b / v_b.
    const int32_t *rowpos;
    int split_tile, tiles_per_unit_b;
    u16 *k_b; size_t k_b_unit_stride, k_b_head_stride;
    u16 *v_b; size_t v_b_unit_stride, v_b_head_stride;
};
// fp32 workspace for K-split partial sums (multi-draft step)
// partial: K-split partial sums; arrive: 1024 arrival counters of the K-split streaming kernel (zero between launches)
struct Workspace { float *partial; size_t partial_bytes; unsigned *arrive; };
void launch_gemm_qkv(const u16 *xa, const u16 *w, GemmShape sh, NormIn ni, QkvOut out, Workspace ws, hipStream_t s);
void launch_gemm_resid(const u16 *a, const u16 *w, GemmShape sh, float *h, int ldh, NormOut no, Workspace ws,
                       hipStream_t s);
void launch_gemm_swiglu(const u16 *xa, const u16 *w, GemmShape sh, NormIn ni, u16 *act, unsigned *status, Workspace ws,
                        hipStream_t s);
// stats[row][lm_stats_parts(N_tiles, M_tiles)][3]: one partial (max, sum exp, argmax) per row and (workgroup, n-slot)
int lm_stats_parts(int n_tiles, int m_tiles);
void launch_gemm_lmstats(const u16 *xa, const u16 *w, GemmShape sh, NormIn ni, float *stats, Workspace ws,
                         hipStream_t s);
// fp32 store of the valid rows (unit u, i < valid of rpu_pad) to a compact row-major [units*valid, ld]
void launch_gemm_store(const u16 *xa, const u16 *w, GemmShape sh, NormIn ni, float *out, int units, int rpu_pad,
                       int valid, int ld, Workspace ws, hipStream_t s);

// ---- attn.hip ---------------------------------------------------------------
struct AttnArgs {
    const u16 *q;              // [H][mt_total][dh/32][512]
    const u16 *kc, *vc;        // cache of this layer
    size_t kc_seq_stride, kc_head_stride, vc_seq_stride, vc_head_stride;
    const u16 *kf, *vf;        // fresh K/V of the units (step only)
    size_t kf_unit_stride, kf_head_stride, vf_unit_stride, vf_head_stride;
    u16 *out;                  // [d/32][mt_total][512]
    int H, dh, mt_total, tiles_per_unit, units, units_per_seq;
    int L;                     // cached length
    int blk_lo, blk_hi;        // cached keys in [blk_lo, blk_hi) are ignored
    int fresh;                 // number of fresh keys per unit (0 in the prefill)
    // Decoded-share step (split_tile > 0): m-tiles below split_tile are block_0 units (one per sequence, the
    // fields above), the others the pooled speculative units (one per sequence, tiles_per_unit_b tiles: the
    // rows of its spec_blocks speculative blocks, mcount[seq] each, one after the other).  Their fresh K/V are in
    // kf_b / vf_b; a row sees the pooled keys of its own block and block_0's fresh K/V of its sequence at the
    // positions set in dmask[seq] (the decoded ones).
    int split_tile, tiles_per_unit_b, spec_blocks;
    const u16 *kf_b, *vf_b;
    size_t kf_b_unit_stride, kf_b_head_stride, vf_b_unit_stride, vf_b_head_stride;
    const int32_t *mcount;
    const unsigned long long *dmask;
};
void launch_attention(AttnArgs a, hipStream_t s);

}  // namespace odb
