// C ABI of the library (include/odb.h): argument validation, memory, and the
// sequence of kernel launches that make up the prefill and the block step.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <chrono>
#include <mutex>
#include <new>

#include "model.h"

using namespace odb;

struct odb_model { Model m; };
struct odb_cache { Cache c; };

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

#define HIP_TRY(expr)                                                                         \
    do {                                                                                      \
        hipError_t e_ = (expr);                                                               \
        if (e_ != hipSuccess) return fail(ODB_E_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int ru(int x, int a) { return (x + a - 1) / a * a; }

void *dev_alloc(const Model &m, size_t bytes) {
    if (bytes == 0) bytes = 256;
    if (m.has_alloc) return m.alloc.alloc(bytes, m.alloc.user);
    void *p = nullptr;
    if (hipMalloc(&p, bytes) != hipSuccess) return nullptr;
    return p;
}

void dev_free(const Model &m, void *p) {
    if (!p) return;
    if (m.has_alloc) m.alloc.free(p, m.alloc.user);
    else (void)hipFree(p);
}

constexpr int kCounters = 1 << 12;     // status word and arrival counters
constexpr size_t kPartialBytes = 32u << 20;   // K-split partial sums of the tile GEMM

// byte offsets of the per-call buffers inside the scratch area of a call
struct Plan {
    size_t h, xa, q, kf, vf, ao, act, ssq, stats, part, extra, total;
    size_t part_bytes;
};

// part_bytes: room for K-split partial sums (the GEMM launchers split K only as far as it allows)
Plan make_plan(const odb_config &c, int rows_pad, int fresh_rows, int lm_rows_pad, bool need_stats, size_t extra_bytes = 0,
               size_t part_bytes = kPartialBytes) {
    Plan p;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    size_t d = c.d_model;
    p.h = take((size_t)rows_pad * d * 4);
    p.xa = take((size_t)rows_pad * d * 2);
    p.q = take((size_t)rows_pad * d * 2);
    p.kf = take((size_t)fresh_rows * d * 2);
    p.vf = take((size_t)fresh_rows * d * 2);
    p.ao = take((size_t)rows_pad * d * 2);
    p.act = take((size_t)rows_pad * c.d_ff * 2);
    p.ssq = take((size_t)rows_pad * (d / 16) * 4);
    // one (max, sum exp, argmax) partial per row and part, as many parts as the LM-head launch for these rows writes
    p.stats = take(need_stats ? (size_t)lm_rows_pad * lm_stats_parts(c.vocab / 16, lm_rows_pad / 16) * 3 * 4 : 0);
    p.part = take(part_bytes);
    p.part_bytes = part_bytes;
    p.extra = take(extra_bytes);
    p.total = off;
    return p;
}

int ensure_scratch(Model &m, size_t bytes, hipStream_t s) {
    if (bytes <= m.scratch_bytes) return ODB_OK;
    HIP_TRY(hipStreamSynchronize(s));
    dev_free(m, m.scratch);
    m.scratch = nullptr;
    m.scratch_bytes = 0;
    size_t want = align_up(bytes + bytes / 8, 1 << 20);
    m.scratch = dev_alloc(m, want);
    if (!m.scratch) return fail(ODB_E_NOMEM, "cannot allocate %zu bytes of scratch", want);
    m.scratch_bytes = want;
    HIP_TRY(hipMemsetAsync(m.scratch, 0, want, s));
    HIP_TRY(hipStreamSynchronize(s));
    return ODB_OK;
}

int check_config(const odb_config *c) {
    if (!c) return fail(ODB_E_INVALID_ARG, "config is NULL");
    if (c->n_layers < 1 || c->d_model < 1 || c->n_heads < 1 || c->d_ff < 1 || c->vocab < 1)
        return fail(ODB_E_INVALID_ARG, "config: sizes must be positive");
    if (c->n_heads * c->head_dim != c->d_model) return fail(ODB_E_INVALID_ARG, "config: d_model != n_heads*head_dim");
    if (c->head_dim != 64 && c->head_dim != 128) return fail(ODB_E_UNSUPPORTED, "config: head_dim must be 64 or 128");
    if (c->d_model % 256 || c->d_ff % 256) return fail(ODB_E_INVALID_ARG, "config: d_model and d_ff must be multiples of 256");
    if (c->vocab % 16) return fail(ODB_E_INVALID_ARG, "config: vocab must be a multiple of 16");
    if (c->mask_id < 0 || c->mask_id >= c->vocab) return fail(ODB_E_INVALID_ARG, "config: mask_id out of range");
    if (!(c->rope_base > 0.f) || !(c->rms_eps >= 0.f)) return fail(ODB_E_INVALID_ARG, "config: rope_base/rms_eps");
    return ODB_OK;
}

size_t tensor_elems(const odb_config &c, int tid) {
    size_t d = c.d_model, f = c.d_ff, v = c.vocab;
    switch (tid) {
    case ODB_T_EMBED: case ODB_T_LM: return v * d;
    case ODB_T_WQ: case ODB_T_WK: case ODB_T_WV: case ODB_T_WO: return d * d;
    case ODB_T_WG: case ODB_T_WU: case ODB_T_WD: return f * d;
    default: return d;
    }
}

struct LayerPtrs { const u16 *qkv, *o, *gu, *dn; const float *g1, *g2; };

LayerPtrs layer_ptrs(const Model &m, int l) {
    LayerPtrs p;
    p.qkv = m.w[PK_QKV] + (size_t)l * m.layer_elems[PK_QKV];
    p.o = m.w[PK_O] + (size_t)l * m.layer_elems[PK_O];
    p.gu = m.w[PK_GU] + (size_t)l * m.layer_elems[PK_GU];
    p.dn = m.w[PK_D] + (size_t)l * m.layer_elems[PK_D];
    p.g1 = m.g1 + (size_t)l * m.cfg.d_model;
    p.g2 = m.g2 + (size_t)l * m.cfg.d_model;
    return p;
}

// brackets the launches of one kernel class with events while profiling is on
struct ProfScope {
    Model &m;
    hipStream_t s;
    int slot;
    ProfScope(Model &m_, int cls, hipStream_t s_) : m(m_), s(s_), slot(-1) {
        if (m.prof_class == cls && m.prof_used < m.prof_cap) {
            slot = m.prof_used++;
            (void)hipEventRecord(m.prof_ev[3 * slot], s);
        }
    }
    ~ProfScope() {
        if (slot >= 0) {
            (void)hipEventRecord(m.prof_ev[3 * slot + 1], s);
            (void)hipEventRecord(m.prof_ev[3 * slot + 2], s);     // an empty pair: what a pair costs by itself
        }
    }
};

// The transformer stack shared by both calls.  `rm` describes the rows; K/V go
// to the cache (prefill) or to the fresh buffers (step).
//
// fused_norm (the step): every RMSNorm is folded into its neighbours - the
// kernel that produces the residual stream h also writes bf16(h * gain) and
// per-tile sums of squares, the consuming GEMM turns them into row scales (both calls run this way).
// Otherwise a separate RMSNorm kernel writes the GEMM input.
struct StackIO {
    RowMap rm;
    int pos_off;
    bool to_cache;      // prefill: K/V are written into the cache
    int blk_lo, blk_hi, fresh, units_per_seq;
    bool fused_norm;
    const SharedMap *shared;    // decoded-share step: ragged units (see model.h), else nullptr
};

Workspace workspace(const Model &m, char *base, const Plan &pl) {
    return Workspace{(float *)(base + pl.part), pl.part_bytes, m.ksplit_reduce ? m.counters + 1024 : nullptr};
}

int run_stack(Model &m, const Cache &c, char *base, const Plan &pl, const StackIO &io, hipStream_t s) {
    const odb_config &cfg = m.cfg;
    float *h = (float *)(base + pl.h), *ssq = (float *)(base + pl.ssq);
    u16 *xa = (u16 *)(base + pl.xa), *q = (u16 *)(base + pl.q), *kf = (u16 *)(base + pl.kf),
        *vf = (u16 *)(base + pl.vf), *ao = (u16 *)(base + pl.ao), *act = (u16 *)(base + pl.act);
    const int d = cfg.d_model, H = cfg.n_heads, dh = cfg.head_dim, F = cfg.d_ff;
    const SharedMap *sm = io.shared;
    const int rows_pad = sm ? sm->rows() : io.rm.units * io.rm.rpu_pad, mt = rows_pad / 16, tpu = io.rm.rpu_pad / 16;
    // decoded-share step: fresh K/V of the batch block_0 units (bp32 rows each) first, then of the pooled speculative units (mp32 rows each)
    const int mp32 = sm ? ru(sm->mp, 32) : 0;
    const size_t spec_off = sm ? (size_t)sm->batch * H * ru(sm->bp, 32) * dh : 0;
    const size_t seq_elems = (size_t)H * c.lmax32 * dh;
    const int fresh32 = ru(io.rm.rpu_pad, 32);
    const int n_ssq = d / 16;
    const Workspace ws = workspace(m, base, pl);
    unsigned *status = m.counters;
    const NormIn ni = io.fused_norm ? NormIn{ssq, n_ssq, cfg.rms_eps} : NormIn{nullptr, 0, 0.f};

    for (int l = 0; l < cfg.n_layers; l++) {
        LayerPtrs w = layer_ptrs(m, l);
        if (!io.fused_norm) {
            ProfScope ps(m, ODB_K_RMSNORM, s);
            launch_rmsnorm(h, w.g1, cfg.rms_eps, d, io.rm, 0, false, mt, xa, status, s);
        }
        QkvOut qo{};
        qo.q = q;
        qo.rope = c.rope;
        qo.status = status;
        qo.tiles_per_unit = tpu; qo.pos_off = io.pos_off; qo.H = H; qo.dh = dh; qo.d = d;
        u16 *kc = c.k + (size_t)l * c.layer_elems, *vc = c.v + (size_t)l * c.layer_elems;
        if (io.to_cache) {
            qo.k = kc; qo.k_unit_stride = seq_elems; qo.k_head_stride = (size_t)c.lmax32 * dh;
            qo.v = vc; qo.v_unit_stride = seq_elems; qo.v_head_stride = (size_t)c.lmax32 * dh;
        } else {
            qo.k = kf; qo.k_head_stride = (size_t)fresh32 * dh; qo.k_unit_stride = (size_t)H * fresh32 * dh;
            qo.v = vf; qo.v_head_stride = (size_t)fresh32 * dh; qo.v_unit_stride = (size_t)H * fresh32 * dh;
        }
        if (sm) {
            qo.rowpos = sm->rowpos;
            qo.split_tile = sm->batch * sm->bp / 16;
            qo.tiles_per_unit_b = sm->mp / 16;
            qo.k_b = kf + spec_off; qo.k_b_head_stride = (size_t)mp32 * dh; qo.k_b_unit_stride = (size_t)H * mp32 * dh;
            qo.v_b = vf + spec_off; qo.v_b_head_stride = (size_t)mp32 * dh; qo.v_b_unit_stride = (size_t)H * mp32 * dh;
        }
        qo.set_divisors();
        {
            ProfScope ps(m, ODB_K_GEMM_QKV, s);
            launch_gemm_qkv(xa, w.qkv, GemmShape{mt, 3 * d / 16, d / 32}, ni, qo, ws, s);
        }

        AttnArgs a{};
        a.q = q; a.kc = kc; a.vc = vc;
        a.kc_seq_stride = seq_elems; a.kc_head_stride = (size_t)c.lmax32 * dh;
        a.vc_seq_stride = seq_elems; a.vc_head_stride = (size_t)c.lmax32 * dh;
        a.kf = kf; a.vf = vf;
        a.kf_unit_stride = qo.k_unit_stride; a.kf_head_stride = qo.k_head_stride;
        a.vf_unit_stride = qo.v_unit_stride; a.vf_head_stride = qo.v_head_stride;
        a.out = ao;
        a.H = H; a.dh = dh; a.mt_total = mt; a.tiles_per_unit = tpu; a.units = io.rm.units;
        a.units_per_seq = io.units_per_seq; a.L = c.length; a.blk_lo = io.blk_lo; a.blk_hi = io.blk_hi;
        a.fresh = io.fresh;
        if (sm) {
            a.split_tile = qo.split_tile; a.tiles_per_unit_b = qo.tiles_per_unit_b; a.spec_blocks = sm->S - 1;
            a.kf_b = qo.k_b; a.kf_b_unit_stride = qo.k_b_unit_stride; a.kf_b_head_stride = qo.k_b_head_stride;
            a.vf_b = qo.v_b; a.vf_b_unit_stride = qo.v_b_unit_stride; a.vf_b_head_stride = qo.v_b_head_stride;
            a.mcount = sm->mcount; a.dmask = sm->dmask;
        }
        {
            ProfScope ps(m, ODB_K_ATTENTION, s);
            launch_attention(a, s);
        }
        // the residual epilogues prepare the norm that follows them
        const float *g_after_mlp = l + 1 < cfg.n_layers ? m.g1 + (size_t)(l + 1) * d : m.gf;
        NormOut no_attn = io.fused_norm ? NormOut{xa, ssq, w.g2, n_ssq, status} : NormOut{nullptr, nullptr, nullptr, 0, nullptr};
        NormOut no_mlp = io.fused_norm ? NormOut{xa, ssq, g_after_mlp, n_ssq, status} : NormOut{nullptr, nullptr, nullptr, 0, nullptr};
        {
            ProfScope ps(m, ODB_K_GEMM_O, s);
            launch_gemm_resid(ao, w.o, GemmShape{mt, d / 16, d / 32}, h, d, no_attn, ws, s);
        }
        if (!io.fused_norm) {
            ProfScope ps(m, ODB_K_RMSNORM, s);
            launch_rmsnorm(h, w.g2, cfg.rms_eps, d, io.rm, 0, false, mt, xa, status, s);
        }
        {
            ProfScope ps(m, ODB_K_GEMM_GATE_UP, s);
            launch_gemm_swiglu(xa, w.gu, GemmShape{mt, 2 * F / 16, d / 32}, ni, act, status, ws, s);
        }
        {
            ProfScope ps(m, ODB_K_GEMM_DOWN, s);
            launch_gemm_resid(act, w.dn, GemmShape{mt, d / 16, F / 32}, h, d, no_mlp, ws, s);
        }
    }
    return ODB_OK;
}

// final norm + LM head.  Fused mode: on the padded rows, straight from hb/ssq.
// Otherwise on the compacted rows (unit u, i >= skip) through the RMSNorm kernel.
int run_head(Model &m, char *base, const Plan &pl, RowMap rm, int skip, bool fused_norm, const int32_t *tokens, int rpu_out,
             float tau, float *conf, int32_t *argmax, uint8_t *unmask, float *logits, hipStream_t s) {
    const odb_config &cfg = m.cfg;
    float *h = (float *)(base + pl.h);
    u16 *xa = (u16 *)(base + pl.xa);
    float *stats = (float *)(base + pl.stats);
    const Workspace ws = workspace(m, base, pl);
    const int rows = rm.units * (rm.valid - skip);
    int lm_mt, rpu_pad, valid;
    NormIn ni{nullptr, 0, 0.f};
    if (fused_norm) {
        lm_mt = rm.units * rm.rpu_pad / 16;
        rpu_pad = rm.rpu_pad;
        valid = rm.valid;
        ni = NormIn{(float *)(base + pl.ssq), cfg.d_model / 16, cfg.rms_eps};
    } else {
        lm_mt = (rows + 15) / 16;
        rpu_pad = valid = rpu_out;
        launch_rmsnorm(h, m.gf, cfg.rms_eps, cfg.d_model, rm, skip, true, lm_mt, xa, m.counters, s);
    }
    GemmShape sh{lm_mt, cfg.vocab / 16, cfg.d_model / 32};
    if (logits) {
        if (fused_norm) launch_gemm_store(xa, m.w[PK_LM], sh, ni, logits, rm.units, rpu_pad, valid, cfg.vocab, ws, s);
        else launch_gemm_store(xa, m.w[PK_LM], sh, ni, logits, 1, lm_mt * 16, rows, cfg.vocab, ws, s);
    } else {
        {
            ProfScope ps(m, ODB_K_GEMM_LM_HEAD, s);
            launch_gemm_lmstats(xa, m.w[PK_LM], sh, ni, stats, ws, s);
        }
        launch_lm_finish(stats, lm_stats_parts(cfg.vocab / 16, lm_mt), rows, rpu_out, rpu_pad, tokens, cfg.mask_id, tau, conf, argmax, unmask,
                         s);
    }
    HIP_TRY(hipGetLastError());
    return ODB_OK;
}

int prefill_impl(odb_model *mh, odb_cache *ch, const int32_t *tokens, int L, int resp_off, float *conf,
                 int32_t *argmax, float *logits, void *stream) {
    if (!mh || !ch || !tokens) return fail(ODB_E_INVALID_ARG, "prefill: NULL handle or tokens");
    Model &m = mh->m;
    Cache &c = ch->c;
    if (c.m != &m) return fail(ODB_E_INVALID_ARG, "prefill: cache belongs to another model");
    if (L < 1 || L > c.max_len) return fail(ODB_E_INVALID_ARG, "prefill: L=%d outside [1, %d]", L, c.max_len);
    if (resp_off < 0 || resp_off >= L) return fail(ODB_E_INVALID_ARG, "prefill: resp_off=%d outside [0, %d)", resp_off, L);
    if (!logits && (!conf || !argmax)) return fail(ODB_E_INVALID_ARG, "prefill: NULL output");
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(hipSetDevice(m.device));
    const int lp = ru(L, 16), rows_pad = c.batch * lp, lm_rows = c.batch * (L - resp_off);
    Plan pl = make_plan(m.cfg, rows_pad, 0, ru(lm_rows, 16), logits == nullptr);
    int rc = ensure_scratch(m, pl.total, s);
    if (rc) return rc;
    RowMap rm{c.batch, lp, L};
    c.length = L;
    char *base = (char *)m.scratch;
    launch_embed(m, tokens, rm, (float *)(base + pl.h),
                 NormOut{(u16 *)(base + pl.xa), (float *)(base + pl.ssq), m.g1, m.cfg.d_model / 16, m.counters}, s);
    StackIO io{rm, 0, true, 0, 0, 0, 1, true};
    rc = run_stack(m, c, base, pl, io, s);
    if (rc) return rc;
    return run_head(m, base, pl, rm, resp_off, false, nullptr, 64, 0.f, conf, argmax, nullptr, logits, s);
}

// The library's fixed scratch area for callers that cannot allocate (odb_block_step_static): one array per GPU,
// held from the moment the library is loaded until the process ends.  Host code never uses the array's name as
// an address: static_scratch_ptr() asks the runtime for this device's copy once and keeps the pointer.
constexpr size_t kStaticScratchBytes = ODB_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
char *g_static_scratch[kMaxDevices];
std::mutex g_static_scratch_mutex;

int static_scratch_ptr(int device, char **out);      // defined behind the array, at the end of this file

// scratch_base == nullptr: the model's own scratch, grown on demand.  Otherwise the call runs in the given area of
// scratch_bytes bytes and allocates nothing.
int step_impl(odb_model *mh, const odb_cache *ch, const int32_t *drafts, int block_off, int b, int S, float tau,
              float *conf, int32_t *argmax, uint8_t *unmask, float *logits, void *stream, char *scratch_base = nullptr,
              size_t scratch_bytes = 0) {
    if (!mh || !ch || !drafts) return fail(ODB_E_INVALID_ARG, "block_step: NULL handle or drafts");
    Model &m = mh->m;
    const Cache &c = ch->c;
    if (c.m != &m) return fail(ODB_E_INVALID_ARG, "block_step: cache belongs to another model");
    if (c.length < 1) return fail(ODB_E_INVALID_ARG, "block_step: cache has not been prefilled");
    if (b < 1 || b > 256) return fail(ODB_E_INVALID_ARG, "block_step: b=%d outside [1, 256]", b);
    if (S < 1 || S > 4096) return fail(ODB_E_INVALID_ARG, "block_step: S=%d outside [1, 4096]", S);
    if (block_off < 0 || block_off + b > c.length)
        return fail(ODB_E_INVALID_ARG, "block_step: block [%d, %d) outside the cached length %d", block_off,
                    block_off + b, c.length);
    if (!logits && (!conf || !argmax || !unmask)) return fail(ODB_E_INVALID_ARG, "block_step: NULL output");
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(hipSetDevice(m.device));
    const odb_config &cfg = m.cfg;
    const int bp = ru(b, 16), bp32 = ru(b, 32), units = c.batch * S, rows_pad = units * bp;
    Plan pl;
    char *base;
    if (scratch_base) {
        // everything but the K-split partial sums first; they get what is left of the fixed area (the GEMM launchers
        // split K only as far as the room allows), at most what the growing scratch would give them
        pl = make_plan(cfg, rows_pad, units * bp32, rows_pad, true, 0, 0);
        if (pl.total + (1u << 20) > scratch_bytes)
            return fail(ODB_E_UNSUPPORTED, "block_step_static: %d rows of this model need %zu bytes of scratch, the fixed "
                        "area holds %zu", rows_pad, pl.total + (1u << 20), scratch_bytes);
        size_t part = (scratch_bytes - pl.total) / 256 * 256;
        pl = make_plan(cfg, rows_pad, units * bp32, rows_pad, true, 0, part < kPartialBytes ? part : kPartialBytes);
        base = scratch_base;
    } else {
        pl = make_plan(cfg, rows_pad, units * bp32, rows_pad, logits == nullptr);
        int rc = ensure_scratch(m, pl.total, s);
        if (rc) return rc;
        base = (char *)m.scratch;
    }
    RowMap rm{units, bp, b};
    launch_embed(m, drafts, rm, (float *)(base + pl.h),
                 NormOut{(u16 *)(base + pl.xa), (float *)(base + pl.ssq), m.g1, cfg.d_model / 16, m.counters}, s);
    if (b % 32)   // slots of padded keys must hold finite values: they meet zero probabilities in the P*V product
        launch_fill_f32((float *)(base + pl.vf), 0.f, (size_t)units * bp32 * cfg.d_model / 2, s);
    StackIO io{rm, block_off, false, block_off, block_off + b, b, S, true};
    int rc = run_stack(m, c, base, pl, io, s);
    if (rc) return rc;
    return run_head(m, base, pl, rm, 0, true, drafts, b, tau, conf, argmax, unmask, logits, s);
}

}  // namespace

extern "C" {

const char *odb_last_error(void) { return g_err; }

const char *odb_strerror(int code) {
    switch (code) {
    case ODB_OK: return "ok";
    case ODB_E_INVALID_ARG: return "invalid argument";
    case ODB_E_NOMEM: return "out of device memory";
    case ODB_E_HIP: return "HIP runtime error";
    case ODB_E_UNSUPPORTED: return "unsupported configuration, device or value range";
    case ODB_E_NO_PROGRESS: return "a decode step unmasked nothing";
    default: return "unknown error";
    }
}

int odb_model_create(const odb_config *cfg, const odb_allocator *allocator, odb_model **out) {
    if (!out) return fail(ODB_E_INVALID_ARG, "model_create: out is NULL");
    *out = nullptr;
    int rc = check_config(cfg);
    if (rc) return rc;
    if (allocator && (!allocator->alloc || !allocator->free))
        return fail(ODB_E_INVALID_ARG, "model_create: allocator needs alloc and free");
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    hipDeviceProp_t prop;
    HIP_TRY(hipGetDeviceProperties(&prop, dev));
    if (strncmp(prop.gcnArchName, "gfx950", 6) != 0)
        return fail(ODB_E_UNSUPPORTED, "device %d is %s; this library is built for gfx950 only", dev, prop.gcnArchName);
    odb_model *mh = new (std::nothrow) odb_model();
    if (!mh) return fail(ODB_E_NOMEM, "model_create: host allocation failed");
    Model &m = mh->m;
    memset(&m, 0, sizeof(m));
    m.cfg = *cfg;
    m.device = dev;
    m.prof_class = -1;
    m.n_cu = prop.multiProcessorCount;
    m.ksplit_reduce = true;
    {
        char *fixed = nullptr;          // this device's copy of the fixed scratch area: looked up once, here
        rc = static_scratch_ptr(dev, &fixed);
        if (rc) { delete mh; return rc; }
    }
    if (allocator) { m.alloc = *allocator; m.has_alloc = true; }
    const size_t d = cfg->d_model, f = cfg->d_ff, v = cfg->vocab, nl = cfg->n_layers;
    m.layer_elems[PK_QKV] = 3 * d * d;
    m.layer_elems[PK_O] = d * d;
    m.layer_elems[PK_GU] = 2 * f * d;
    m.layer_elems[PK_D] = d * f;
    m.layer_elems[PK_LM] = v * d;
    m.layer_elems[PK_EMBED] = v * d;
    bool ok = true;
    for (int pk = 0; pk < PK_COUNT; pk++) {
        size_t layers = (pk == PK_LM || pk == PK_EMBED) ? 1 : nl;
        m.w[pk] = (u16 *)dev_alloc(m, m.layer_elems[pk] * layers * 2);
        ok = ok && m.w[pk];
    }
    m.g1 = (float *)dev_alloc(m, nl * d * 4);
    m.g2 = (float *)dev_alloc(m, nl * d * 4);
    m.gf = (float *)dev_alloc(m, d * 4);
    m.counters = (unsigned *)dev_alloc(m, kCounters * sizeof(unsigned));
    ok = ok && m.g1 && m.g2 && m.gf && m.counters;
    if (!ok) {
        odb_model_destroy(mh);
        return fail(ODB_E_NOMEM, "model_create: device allocation failed");
    }
    hipError_t e = hipMemset(m.counters, 0, kCounters * sizeof(unsigned));
    if (e != hipSuccess) {
        odb_model_destroy(mh);
        return fail(ODB_E_HIP, "hipMemset: %s", hipGetErrorString(e));
    }
    *out = mh;
    return ODB_OK;
}

void odb_model_destroy(odb_model *mh) {
    if (!mh) return;
    Model &m = mh->m;
    (void)hipSetDevice(m.device);
    (void)hipDeviceSynchronize();
    for (int pk = 0; pk < PK_COUNT; pk++) dev_free(m, m.w[pk]);
    dev_free(m, m.g1);
    dev_free(m, m.g2);
    dev_free(m, m.gf);
    dev_free(m, m.counters);
    dev_free(m, m.scratch);
    dev_free(m, m.staging);
    if (m.prof_ev) {
        for (int i = 0; i < 3 * m.prof_cap; i++) (void)hipEventDestroy(m.prof_ev[i]);
        delete[] m.prof_ev;
    }
    delete mh;
}

int odb_model_init_random(odb_model *mh, uint64_t seed, double std, void *stream) {
    if (!mh) return fail(ODB_E_INVALID_ARG, "init_random: model is NULL");
    if (!(std >= 0.0)) return fail(ODB_E_INVALID_ARG, "init_random: std must be >= 0");
    HIP_TRY(hipSetDevice(mh->m.device));
    launch_init_random(mh->m, seed, std, (hipStream_t)stream);
    HIP_TRY(hipGetLastError());
    return ODB_OK;
}

static int tensor_io(Model &m, int tensor_id, int layer, uint16_t *host, size_t n, bool to_model) {
    if (tensor_id < 0 || tensor_id >= ODB_T_COUNT) return fail(ODB_E_INVALID_ARG, "tensor id %d", tensor_id);
    if (!host) return fail(ODB_E_INVALID_ARG, "tensor buffer is NULL");
    bool global = tensor_id == ODB_T_EMBED || tensor_id == ODB_T_LM || tensor_id == ODB_T_GF;
    if (!global && (layer < 0 || layer >= m.cfg.n_layers)) return fail(ODB_E_INVALID_ARG, "layer %d", layer);
    if (global) layer = 0;
    size_t want = tensor_elems(m.cfg, tensor_id);
    if (n != want) return fail(ODB_E_INVALID_ARG, "tensor %d has %zu elements, got %zu", tensor_id, want, n);
    HIP_TRY(hipSetDevice(m.device));
    HIP_TRY(hipDeviceSynchronize());
    if (m.staging_bytes < n * 2) {
        dev_free(m, m.staging);
        m.staging_bytes = 0;
        m.staging = (u16 *)dev_alloc(m, n * 2);
        if (!m.staging) return fail(ODB_E_NOMEM, "tensor staging of %zu bytes", n * 2);
        m.staging_bytes = n * 2;
    }
    if (to_model && tensor_id != ODB_T_EMBED && tensor_id < ODB_T_G1) {
        // projection matrices are held as binary16: a bf16 value beyond its range (or a NaN) would be clamped silently
        for (size_t i = 0; i < n; i++)
            if ((host[i] & 0x7fffu) > 0x477fu)          // |x| > 65280, the largest bf16 value that binary16 holds
                return fail(ODB_E_UNSUPPORTED, "set_tensor: element %zu of tensor %d (bf16 bits 0x%04x) lies outside the "
                            "binary16 range the projection matrices are stored in", i, tensor_id, host[i]);
    }
    if (to_model) HIP_TRY(hipMemcpy(m.staging, host, n * 2, hipMemcpyHostToDevice));
    if (tensor_id >= ODB_T_G1) {
        float *g = tensor_id == ODB_T_G1 ? m.g1 + (size_t)layer * m.cfg.d_model
                 : tensor_id == ODB_T_G2 ? m.g2 + (size_t)layer * m.cfg.d_model : m.gf;
        launch_gain_copy(g, m.staging, (int)n, to_model, nullptr);
    } else {
        launch_tensor_copy(m, tensor_id, layer, m.staging, to_model, nullptr);
    }
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipDeviceSynchronize());
    if (!to_model) HIP_TRY(hipMemcpy(host, m.staging, n * 2, hipMemcpyDeviceToHost));
    return ODB_OK;
}

int odb_model_set_tensor(odb_model *mh, int tensor_id, int layer, const uint16_t *host_bf16, size_t n) {
    if (!mh) return fail(ODB_E_INVALID_ARG, "set_tensor: model is NULL");
    return tensor_io(mh->m, tensor_id, layer, const_cast<uint16_t *>(host_bf16), n, true);
}

int odb_model_get_tensor(const odb_model *mh, int tensor_id, int layer, uint16_t *host_bf16, size_t n) {
    if (!mh) return fail(ODB_E_INVALID_ARG, "get_tensor: model is NULL");
    return tensor_io(const_cast<odb_model *>(mh)->m, tensor_id, layer, host_bf16, n, false);
}

int odb_cache_create(odb_model *mh, int batch, int max_len, odb_cache **out) {
    if (!out) return fail(ODB_E_INVALID_ARG, "cache_create: out is NULL");
    *out = nullptr;
    if (!mh) return fail(ODB_E_INVALID_ARG, "cache_create: model is NULL");
    if (batch < 1 || batch > 1024) return fail(ODB_E_INVALID_ARG, "cache_create: batch=%d outside [1, 1024]", batch);
    if (max_len < 1 || max_len > (1 << 20)) return fail(ODB_E_INVALID_ARG, "cache_create: max_len=%d", max_len);
    Model &m = mh->m;
    HIP_TRY(hipSetDevice(m.device));
    odb_cache *ch = new (std::nothrow) odb_cache();
    if (!ch) return fail(ODB_E_NOMEM, "cache_create: host allocation failed");
    Cache &c = ch->c;
    memset(&c, 0, sizeof(c));
    c.m = &m;
    c.batch = batch;
    c.max_len = max_len;
    c.lmax32 = ru(max_len, 32);
    c.layer_elems = (size_t)batch * m.cfg.d_model * c.lmax32;
    size_t bytes = c.layer_elems * m.cfg.n_layers * 2;
    c.k = (u16 *)dev_alloc(m, bytes);
    c.v = (u16 *)dev_alloc(m, bytes);
    const int rope_rows = c.lmax32 + 16;      // padded rows of the last tile may look one tile past the end
    c.rope = (float *)dev_alloc(m, (size_t)rope_rows * m.cfg.head_dim * 4);
    if (!c.k || !c.v || !c.rope) {
        odb_cache_destroy(ch);
        return fail(ODB_E_NOMEM, "cache_create: cannot allocate 2 x %zu bytes", bytes);
    }
    hipError_t e = hipMemset(c.k, 0, bytes);
    if (e == hipSuccess) e = hipMemset(c.v, 0, bytes);
    if (e == hipSuccess) {
        launch_rope_table(c.rope, rope_rows, m.cfg.head_dim, (double)m.cfg.rope_base, nullptr);
        e = hipDeviceSynchronize();
    }
    if (e != hipSuccess) {
        odb_cache_destroy(ch);
        return fail(ODB_E_HIP, "cache_create: %s", hipGetErrorString(e));
    }
    *out = ch;
    return ODB_OK;
}

void odb_cache_destroy(odb_cache *ch) {
    if (!ch) return;
    Cache &c = ch->c;
    (void)hipSetDevice(c.m->device);
    (void)hipDeviceSynchronize();
    dev_free(*c.m, c.k);
    dev_free(*c.m, c.v);
    dev_free(*c.m, c.rope);
    delete ch;
}

int odb_cache_length(const odb_cache *ch) { return ch ? ch->c.length : 0; }

int odb_cache_truncate(odb_cache *ch, int new_len) {
    if (!ch) return fail(ODB_E_INVALID_ARG, "cache_truncate: cache is NULL");
    if (new_len < 1 || new_len > ch->c.length)
        return fail(ODB_E_INVALID_ARG, "cache_truncate: new_len=%d outside [1, %d]", new_len, ch->c.length);
    ch->c.length = new_len;
    return ODB_OK;
}

int odb_prefill(odb_model *m, odb_cache *c, const int32_t *tokens_dev, int L, int resp_off, float *conf_dev,
                int32_t *argmax_dev, void *stream) {
    return prefill_impl(m, c, tokens_dev, L, resp_off, conf_dev, argmax_dev, nullptr, stream);
}

int odb_prefill_logits(odb_model *m, odb_cache *c, const int32_t *tokens_dev, int L, int resp_off, float *logits_dev,
                       void *stream) {
    if (!logits_dev) return fail(ODB_E_INVALID_ARG, "prefill_logits: logits is NULL");
    return prefill_impl(m, c, tokens_dev, L, resp_off, nullptr, nullptr, logits_dev, stream);
}

int odb_block_step(odb_model *m, const odb_cache *c, const int32_t *drafts_dev, int block_off, int b, int S, float tau,
                   float *conf_dev, int32_t *argmax_dev, uint8_t *unmask_dev, void *stream) {
    return step_impl(m, c, drafts_dev, block_off, b, S, tau, conf_dev, argmax_dev, unmask_dev, nullptr, stream);
}

int odb_block_step_logits(odb_model *m, const odb_cache *c, const int32_t *drafts_dev, int block_off, int b, int S,
                          float *logits_dev, void *stream) {
    if (!logits_dev) return fail(ODB_E_INVALID_ARG, "block_step_logits: logits is NULL");
    return step_impl(m, c, drafts_dev, block_off, b, S, 0.f, nullptr, nullptr, nullptr, logits_dev, stream);
}

// Decode step in the decoded-share stage (ODB-dLLM Sec. 4.2.2): block_0 in full, the speculative blocks reduced to
// the positions that block_0 still has masked, block_0's fresh K/V of the decoded positions shared with them.
static int step_shared_impl(odb_model *mh, const odb_cache *ch, const int32_t *drafts, int block_off, int b, int S,
                            int n_masked, float tau, float *conf, int32_t *argmax, uint8_t *unmask, float *logits,
                            int32_t *rowout, void *stream) {
    if (!mh || !ch || !drafts) return fail(ODB_E_INVALID_ARG, "block_step_shared: NULL handle or drafts");
    Model &m = mh->m;
    const Cache &c = ch->c;
    if (c.m != &m) return fail(ODB_E_INVALID_ARG, "block_step_shared: cache belongs to another model");
    if (c.length < 1) return fail(ODB_E_INVALID_ARG, "block_step_shared: cache has not been prefilled");
    if (b < 1 || b > 64) return fail(ODB_E_INVALID_ARG, "block_step_shared: b=%d outside [1, 64]", b);
    if (S < 2 || S > 64) return fail(ODB_E_INVALID_ARG, "block_step_shared: S=%d outside [2, 64]", S);
    if (n_masked < 0 || n_masked > b) return fail(ODB_E_INVALID_ARG, "block_step_shared: n_masked=%d outside [0, %d]", n_masked, b);
    if (block_off < 0 || block_off + b > c.length)
        return fail(ODB_E_INVALID_ARG, "block_step_shared: block [%d, %d) outside the cached length %d", block_off,
                    block_off + b, c.length);
    if (!logits && (!conf || !argmax || !unmask)) return fail(ODB_E_INVALID_ARG, "block_step_shared: NULL output");
    if (logits && !rowout) return fail(ODB_E_INVALID_ARG, "block_step_shared: NULL row map");
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(hipSetDevice(m.device));
    const odb_config &cfg = m.cfg;
    SharedMap sm;
    sm.batch = c.batch; sm.S = S; sm.b = b; sm.bp = ru(b, 16); sm.mp = ru(n_masked > 0 ? (S - 1) * n_masked : 1, 16);
    const int rows_pad = sm.rows();
    const int fresh_rows = c.batch * (ru(sm.bp, 32) + ru(sm.mp, 32));
    const size_t tables = align_up((size_t)rows_pad * 4, 256) * 3 + align_up((size_t)c.batch * 4, 256) +
                          align_up((size_t)c.batch * 8, 256);
    Plan pl = make_plan(cfg, rows_pad, fresh_rows, rows_pad, logits == nullptr, tables);
    int rc = ensure_scratch(m, pl.total, s);
    if (rc) return rc;
    char *base = (char *)m.scratch, *t = base + pl.extra;
    sm.rowtok = (int32_t *)t; t += align_up((size_t)rows_pad * 4, 256);
    sm.rowpos = (int32_t *)t; t += align_up((size_t)rows_pad * 4, 256);
    sm.rowout = (int32_t *)t; t += align_up((size_t)rows_pad * 4, 256);
    sm.mcount = (int32_t *)t; t += align_up((size_t)c.batch * 4, 256);
    sm.dmask = (unsigned long long *)t;
    launch_shared_setup(drafts, sm, block_off, cfg.mask_id, n_masked, conf, argmax, unmask, m.counters, s);
    // rows are embedded through the token-per-row table: every row is its own unit of one
    launch_embed(m, sm.rowtok, RowMap{rows_pad, 1, 1}, (float *)(base + pl.h),
                 NormOut{(u16 *)(base + pl.xa), (float *)(base + pl.ssq), m.g1, cfg.d_model / 16, m.counters}, s);
    // slots of padded keys must hold finite values: they meet zero probabilities in the P*V product
    launch_fill_f32((float *)(base + pl.vf), 0.f, (size_t)fresh_rows * cfg.d_model / 2, s);
    RowMap rm{c.batch, sm.bp, b};
    StackIO io{rm, block_off, false, block_off, block_off + b, b, 1, true, &sm};
    rc = run_stack(m, c, base, pl, io, s);
    if (rc) return rc;
    // final norm (fused) + LM head on all rows, then the per-unit finish
    u16 *xa = (u16 *)(base + pl.xa);
    const Workspace ws = workspace(m, base, pl);
    const NormIn ni{(float *)(base + pl.ssq), cfg.d_model / 16, cfg.rms_eps};
    const GemmShape sh{rows_pad / 16, cfg.vocab / 16, cfg.d_model / 32};
    if (logits) {
        launch_gemm_store(xa, m.w[PK_LM], sh, ni, logits, 1, rows_pad, rows_pad, cfg.vocab, ws, s);
        HIP_TRY(hipMemcpyAsync(rowout, sm.rowout, (size_t)rows_pad * 4, hipMemcpyDeviceToDevice, s));
    } else {
        float *stats = (float *)(base + pl.stats);
        {
            ProfScope ps(m, ODB_K_GEMM_LM_HEAD, s);
            launch_gemm_lmstats(xa, m.w[PK_LM], sh, ni, stats, ws, s);
        }
        launch_lm_finish_shared(stats, lm_stats_parts(cfg.vocab / 16, rows_pad / 16), sm, cfg.mask_id, tau, conf, argmax,
                                unmask, s);
    }
    HIP_TRY(hipGetLastError());
    return ODB_OK;
}

int odb_block_step_shared(odb_model *m, const odb_cache *c, const int32_t *drafts_dev, int block_off, int b, int S,
                          int n_masked, float tau, float *conf_dev, int32_t *argmax_dev, uint8_t *unmask_dev,
                          void *stream) {
    return step_shared_impl(m, c, drafts_dev, block_off, b, S, n_masked, tau, conf_dev, argmax_dev, unmask_dev, nullptr,
                            nullptr, stream);
}

int odb_block_step_shared_rows(int batch, int b, int S, int n_masked) {
    if (batch < 1 || b < 1 || S < 2 || n_masked < 0 || n_masked > b) return fail(ODB_E_INVALID_ARG, "block_step_shared_rows");
    return batch * (ru(b, 16) + ru(n_masked > 0 ? (S - 1) * n_masked : 1, 16));
}

int odb_block_step_shared_logits(odb_model *m, const odb_cache *c, const int32_t *drafts_dev, int block_off, int b,
                                 int S, int n_masked, float *logits_dev, int32_t *rowout_dev, void *stream) {
    if (!logits_dev) return fail(ODB_E_INVALID_ARG, "block_step_shared_logits: logits is NULL");
    return step_shared_impl(m, c, drafts_dev, block_off, b, S, n_masked, 0.f, nullptr, nullptr, nullptr, logits_dev,
                            rowout_dev, stream);
}

int odb_set_option(odb_model *mh, int option, int value) {
    if (!mh) return fail(ODB_E_INVALID_ARG, "set_option: model is NULL");
    switch (option) {
    case ODB_OPT_KSPLIT_REDUCE:
        if (value != 0 && value != 1) return fail(ODB_E_INVALID_ARG, "set_option: KSPLIT_REDUCE takes 0 or 1");
        mh->m.ksplit_reduce = value != 0;
        return ODB_OK;
    default:
        return fail(ODB_E_INVALID_ARG, "set_option: unknown option %d", option);
    }
}

int odb_model_status(odb_model *mh) {
    if (!mh) return fail(ODB_E_INVALID_ARG, "model_status: model is NULL");
    Model &m = mh->m;
    HIP_TRY(hipSetDevice(m.device));
    HIP_TRY(hipDeviceSynchronize());
    unsigned host = 0;
    HIP_TRY(hipMemcpy(&host, m.counters, sizeof(host), hipMemcpyDeviceToHost));
    if (host != 0) {
        // bring flags, epoch and status back to a clean state
        // back to a clean state (only the status word: the arrival counters are zero between launches anyway)
        HIP_TRY(hipMemset(m.counters, 0, sizeof(unsigned)));
        if (host & kStatusSaturated)
            return fail(ODB_E_UNSUPPORTED, "an activation left the binary16 range (|x| > 65504, or not a number) and was "
                        "clamped: the outputs of the calls since the last status check are not to be trusted");
        if (host & kStatusSharedOverflow)
            return fail(ODB_E_INVALID_ARG, "block_step_shared: a block held more MASK positions than n_masked");
        return fail(ODB_E_HIP, "unknown status bits 0x%x", host);
    }
    return ODB_OK;
}

int odb_profile_begin(odb_model *mh, int kernel_class, int max_launches) {
    if (!mh) return fail(ODB_E_INVALID_ARG, "profile_begin: model is NULL");
    Model &m = mh->m;
    if (kernel_class < 0 || kernel_class >= ODB_K_COUNT) return fail(ODB_E_INVALID_ARG, "profile_begin: class %d", kernel_class);
    if (max_launches < 1 || max_launches > (1 << 20)) return fail(ODB_E_INVALID_ARG, "profile_begin: max_launches");
    if (m.prof_ev) return fail(ODB_E_INVALID_ARG, "profile_begin: already profiling");
    HIP_TRY(hipSetDevice(m.device));
    m.prof_ev = new (std::nothrow) hipEvent_t[3 * (size_t)max_launches];
    if (!m.prof_ev) return fail(ODB_E_NOMEM, "profile_begin: host allocation");
    for (int i = 0; i < 3 * max_launches; i++) {
        hipError_t e = hipEventCreate(&m.prof_ev[i]);
        if (e != hipSuccess) {
            for (int j = 0; j < i; j++) (void)hipEventDestroy(m.prof_ev[j]);
            delete[] m.prof_ev;
            m.prof_ev = nullptr;
            return fail(ODB_E_HIP, "hipEventCreate: %s", hipGetErrorString(e));
        }
    }
    m.prof_cap = max_launches;
    m.prof_used = 0;
    m.prof_class = kernel_class;
    return ODB_OK;
}

int odb_profile_end(odb_model *mh, int *n_launches, float *total_ms, float *empty_pairs_ms) {
    if (!mh || !n_launches || !total_ms) return fail(ODB_E_INVALID_ARG, "profile_end: NULL argument");
    Model &m = mh->m;
    if (!m.prof_ev) return fail(ODB_E_INVALID_ARG, "profile_end: not profiling");
    HIP_TRY(hipSetDevice(m.device));
    hipError_t e = hipDeviceSynchronize();
    float total = 0.f, empty = 0.f;
    for (int i = 0; i < m.prof_used && e == hipSuccess; i++) {
        float ms = 0.f;
        e = hipEventElapsedTime(&ms, m.prof_ev[3 * i], m.prof_ev[3 * i + 1]);
        total += ms;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, m.prof_ev[3 * i + 1], m.prof_ev[3 * i + 2]);
        empty += ms;
    }
    for (int i = 0; i < 3 * m.prof_cap; i++) (void)hipEventDestroy(m.prof_ev[i]);
    delete[] m.prof_ev;
    m.prof_ev = nullptr;
    *n_launches = m.prof_used;
    *total_ms = total;
    if (empty_pairs_ms) *empty_pairs_ms = empty;
    m.prof_class = -1;
    m.prof_cap = m.prof_used = 0;
    if (e != hipSuccess) return fail(ODB_E_HIP, "profile_end: %s", hipGetErrorString(e));
    return ODB_OK;
}

int odb_accept_jump(const odb_model *mh, const int32_t *drafts, const float *conf, const int32_t *argmax,
                    const uint8_t *unmask, const int32_t *cand_pos, const int32_t *cand_tok, int batch, int b,
                    int32_t *chosen, int32_t *new_drafts, int32_t *new_cand_pos, int32_t *new_cand_tok, void *stream) {
    if (!mh || !drafts || !conf || !argmax || !unmask || !cand_pos || !cand_tok || !chosen || !new_drafts || !new_cand_pos ||
        !new_cand_tok)
        return fail(ODB_E_INVALID_ARG, "accept_jump: NULL argument");
    if (batch < 1 || b < 1) return fail(ODB_E_INVALID_ARG, "accept_jump: batch=%d, b=%d", batch, b);
    const Model &m = mh->m;
    HIP_TRY(hipSetDevice(m.device));
    launch_accept_jump(drafts, conf, argmax, unmask, cand_pos, cand_tok, batch, b, m.cfg.mask_id, chosen, new_drafts,
                       new_cand_pos, new_cand_tok, (hipStream_t)stream);
    HIP_TRY(hipGetLastError());
    return ODB_OK;
}

int odb_speculative_jump(const odb_model *mh, const int32_t *drafts, const float *conf, const int32_t *argmax,
                         const uint8_t *unmask, const int32_t *cand_pos, const int32_t *cand_tok, int batch, int b, int S,
                         int n_next, int32_t *chosen, int32_t *new_drafts, int32_t *new_cand_pos, int32_t *new_cand_tok,
                         void *stream) {
    if (!mh || !drafts || !conf || !argmax || !unmask || !cand_pos || !cand_tok || !chosen || !new_drafts || !new_cand_pos ||
        !new_cand_tok)
        return fail(ODB_E_INVALID_ARG, "speculative_jump: NULL argument");
    if (batch < 1 || b < 1) return fail(ODB_E_INVALID_ARG, "speculative_jump: batch=%d, b=%d", batch, b);
    if ((S != 4 && S != 8) || (n_next != 4 && n_next != 8))
        return fail(ODB_E_INVALID_ARG, "speculative_jump: S=%d, n_next=%d (4 or 8)", S, n_next);
    const Model &m = mh->m;
    HIP_TRY(hipSetDevice(m.device));
    launch_spec_jump(drafts, conf, argmax, unmask, cand_pos, cand_tok, batch, S, n_next, b, m.cfg.mask_id, chosen, new_drafts,
                     new_cand_pos, new_cand_tok, (hipStream_t)stream);
    HIP_TRY(hipGetLastError());
    return ODB_OK;
}

int odb_predict_length(const odb_model *mh, const int32_t *tokens, const float *conf, const int32_t *argmax, int batch,
                       int L, int resp_off, int eos_id, float truncate_thr, int32_t *new_len, void *stream) {
    if (!mh || !tokens || !conf || !argmax || !new_len) return fail(ODB_E_INVALID_ARG, "predict_length: NULL argument");
    const Model &m = mh->m;
    if (batch < 1 || L < 1) return fail(ODB_E_INVALID_ARG, "predict_length: batch=%d, L=%d", batch, L);
    if (resp_off < 0 || resp_off >= L) return fail(ODB_E_INVALID_ARG, "predict_length: resp_off=%d outside [0, %d)", resp_off, L);
    if (eos_id < 0 || eos_id >= m.cfg.vocab || eos_id == m.cfg.mask_id)
        return fail(ODB_E_INVALID_ARG, "predict_length: eos_id=%d (vocab %d, MASK %d)", eos_id, m.cfg.vocab, m.cfg.mask_id);
    HIP_TRY(hipSetDevice(m.device));
    launch_predict_length(tokens, conf, argmax, batch, L, resp_off, m.cfg.mask_id, eos_id, truncate_thr, new_len,
                          (hipStream_t)stream);
    HIP_TRY(hipGetLastError());
    return ODB_OK;
}

// The generation loop (ODB-dLLM Sec. 2.1 + 4.1 + 4.2): see odb.h for the order of events.  Every decision is
// a kernel's; the host reads sixteen words (64 bytes) back per forward to learn the length, the block's MASK count (loop
// exit, row bound of the decoded-share step) and what to record.
int odb_generate(odb_model *mh, odb_cache *ch, int32_t *tokens, int prompt_len, int resp_len,
                 const odb_generate_params *gp, odb_generate_stats *st, odb_generate_event *events,
                 int32_t *event_tokens, int max_events, void *stream) {
    if (!mh || !ch || !tokens || !gp || !st) return fail(ODB_E_INVALID_ARG, "generate: NULL argument");
    Model &m = mh->m;
    Cache &c = ch->c;
    const int P = prompt_len, R = resp_len, b = gp->block_len, mask_id = m.cfg.mask_id;
    if (c.m != &m) return fail(ODB_E_INVALID_ARG, "generate: cache belongs to another model");
    if (P < 1 || R < 1) return fail(ODB_E_INVALID_ARG, "generate: prompt_len=%d, resp_len=%d", P, R);
    if (c.batch != 1 || c.max_len < P + R)
        return fail(ODB_E_INVALID_ARG, "generate: needs a cache of batch 1 and max_len >= %d (has batch %d, max_len %d)",
                    P + R, c.batch, c.max_len);
    const int nd = gp->n_drafts;
    if ((nd != 1 && nd != 4 && nd != 8) || (nd == 8 && gp->share_from < 0))
        return fail(ODB_E_INVALID_ARG, "generate: n_drafts=%d, share_from=%d", nd, gp->share_from);
    const bool share = nd >= 4 && gp->share_from >= 0;
    if (b < 1 || b > 256 || (share && b > 64)) return fail(ODB_E_INVALID_ARG, "generate: block_len=%d", b);
    if (gp->eos_id >= m.cfg.vocab || gp->eos_id == mask_id) return fail(ODB_E_INVALID_ARG, "generate: eos_id=%d", gp->eos_id);
    if (max_events < 0 || ((events || event_tokens) && max_events < 1))
        return fail(ODB_E_INVALID_ARG, "generate: max_events=%d", max_events);
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(hipSetDevice(m.device));
    memset(st, 0, sizeof(*st));

    // working buffers: the refresh's attempt, two sets of drafts and candidates (the controller reads one and
    // writes the other), one step's outputs, the words for the host
    const size_t nb = (size_t)(nd == 8 ? 8 : 4) * b;
    const size_t bytes = align_up((size_t)R * 4, 256) * 2 + align_up(nb * 4, 256) * 4 + align_up(nb, 256) + 256 * 4;
    char *buf = (char *)dev_alloc(m, bytes);
    int32_t *host_ctl = nullptr;
    if (!buf) return fail(ODB_E_NOMEM, "generate: cannot allocate %zu bytes", bytes);
    if (hipHostMalloc((void **)&host_ctl, 64, hipHostMallocDefault) != hipSuccess) {
        dev_free(m, buf);
        return fail(ODB_E_NOMEM, "generate: cannot allocate pinned host memory");
    }
    char *t = buf;
    auto take = [&](size_t n) { char *r = t; t += align_up(n, 256); return r; };
    float *att_conf = (float *)take((size_t)R * 4);
    int32_t *att_am = (int32_t *)take((size_t)R * 4);
    int32_t *drafts[2] = {(int32_t *)take(nb * 4), (int32_t *)take(nb * 4)};
    float *conf = (float *)take(nb * 4);
    int32_t *am = (int32_t *)take(nb * 4);
    uint8_t *um = (uint8_t *)take(nb);
    int32_t *cand[2] = {(int32_t *)take(32), (int32_t *)take(32)};          // four positions, then four tokens
    int32_t *chosen = (int32_t *)take(4), *ctl = (int32_t *)take(64);     // ctl[0..8) for the host, ctl[8] the predicted length

    using clk = std::chrono::steady_clock;
    auto ms_since = [](clk::time_point a) { return std::chrono::duration<double, std::milli>(clk::now() - a).count(); };
    int rc = ODB_OK, L = P + R, off = P, cur = 0;
    const int L0 = P + R;
    const auto t_all = clk::now();
    auto read_back = [&](int kind) -> int {      // ctl -> host, one record; the only synchronisation of a forward
        if (event_tokens && st->n_events < max_events)
            HIP_TRY(hipMemcpyAsync(event_tokens + (size_t)st->n_events * L0, tokens, (size_t)L0 * 4, hipMemcpyDeviceToDevice, s));
        HIP_TRY(hipMemcpyAsync(host_ctl, ctl, 64, hipMemcpyDeviceToHost, s));
        HIP_TRY(hipStreamSynchronize(s));
        if (events && st->n_events < max_events) {
            odb_generate_event &e = events[st->n_events];
            e.kind = kind; e.length = host_ctl[0]; e.block_off = off; e.block_len = host_ctl[7]; e.chosen = host_ctl[2];
            e.n_masked = host_ctl[1];
            e.cand_pos[0] = host_ctl[3]; e.cand_pos[1] = host_ctl[4]; e.cand_tok[0] = host_ctl[5]; e.cand_tok[1] = host_ctl[6];
            e.cand_pos[2] = host_ctl[9]; e.cand_pos[3] = host_ctl[10]; e.cand_tok[2] = host_ctl[11]; e.cand_tok[3] = host_ctl[12];
        }
        st->n_events++;
        return ODB_OK;
    };
    launch_fill_i32(tokens + P, mask_id, (size_t)R, s);
    while (rc == ODB_OK && off < L) {
        // ---- refresh, length prediction, adoption of the attempt at the block
        auto t0 = clk::now();
        rc = prefill_impl(mh, ch, tokens, L, P, att_conf, att_am, nullptr, stream);
        if (rc) break;
        st->n_refresh++;
        st->refresh_positions += L;
        if (gp->eos_id >= 0)
            launch_predict_length(tokens, att_conf, att_am, 1, L, P, mask_id, gp->eos_id, gp->truncate_thr, ctl + 8, s);
        launch_gen_adopt(tokens, off, b, gp->eos_id >= 0 ? ctl + 8 : nullptr, L, att_conf + (off - P), att_am + (off - P),
                         nullptr, mask_id, gp->tau, nd >= 4 ? drafts[cur] : nullptr, nd, cand[cur], ctl, s);
        if ((rc = read_back(ODB_EV_REFRESH))) break;
        st->refresh_ms += ms_since(t0);
        L = host_ctl[0];
        c.length = L;
        const int bb = host_ctl[7];
        int n_masked = host_ctl[1];
        if (bb <= 0) break;
        // ---- decode steps against this cycle's cache
        while (n_masked > 0) {
            t0 = clk::now();
            int kind = ODB_EV_STEP;
            if (gp->n_drafts == 1) {
                rc = step_impl(mh, ch, tokens + off, off, bb, 1, gp->tau, conf, am, um, nullptr, stream);
                if (rc) break;
                launch_gen_adopt(tokens, off, bb, nullptr, L, conf, am, um, mask_id, gp->tau, nullptr, 0, cand[cur], ctl, s);
                st->step_rows += bb;
            } else {
                // (the first four of eight blocks are the accept-jump drafts: the steps before the switch use those)
                int S = 4;
                if (share && bb - n_masked >= gp->share_from) {
                    kind = ODB_EV_STEP_SHARED;
                    S = nd == 8 && gp->row_budget > 0 && bb + 7 * n_masked > gp->row_budget ? 4 : nd;
                    rc = step_shared_impl(mh, ch, drafts[cur], off, bb, S, n_masked, gp->tau, conf, am, um, nullptr, nullptr, stream);
                    st->step_rows += bb + (S - 1) * n_masked;
                    st->n_step_shared++;
                } else {
                    rc = step_impl(mh, ch, drafts[cur], off, bb, 4, gp->tau, conf, am, um, nullptr, stream);
                    st->step_rows += 4 * bb;
                }
                if (rc) break;
                launch_spec_jump(drafts[cur], conf, am, um, cand[cur], cand[cur] + 4, 1, S, nd, bb, mask_id, chosen,
                                 drafts[cur ^ 1], cand[cur ^ 1], cand[cur ^ 1] + 4, s);
                cur ^= 1;
                launch_gen_commit(tokens, off, bb, L, drafts[cur], chosen, cand[cur], mask_id, ctl, s);
            }
            st->n_step++;
            if ((rc = read_back(kind))) break;
            st->step_ms += ms_since(t0);
            if (host_ctl[1] >= n_masked) {           // forced progress makes this impossible; never spin on it
                rc = fail(ODB_E_NO_PROGRESS, "generate: a step left %d of %d positions masked", host_ctl[1], n_masked);
                break;
            }
            n_masked = host_ctl[1];
        }
        off += bb;
    }
    hipError_t e = hipStreamSynchronize(s);
    st->final_len = L;
    st->total_ms = ms_since(t_all);
    (void)hipHostFree(host_ctl);
    dev_free(m, buf);
    if (rc == ODB_OK && e != hipSuccess) rc = fail(ODB_E_HIP, "generate: %s", hipGetErrorString(e));
    return rc;
}

int odb_cache_read(const odb_cache *ch, int layer, int kv, int batch_index, int pos0, int n, float *host_f32) {
    if (!ch || !host_f32) return fail(ODB_E_INVALID_ARG, "cache_read: NULL argument");
    const Cache &c = ch->c;
    Model &m = *c.m;
    if (layer < 0 || layer >= m.cfg.n_layers || kv < 0 || kv > 1 || batch_index < 0 || batch_index >= c.batch)
        return fail(ODB_E_INVALID_ARG, "cache_read: layer/kv/batch out of range");
    if (pos0 < 0 || n < 1 || pos0 + n > c.length) return fail(ODB_E_INVALID_ARG, "cache_read: positions [%d, %d) outside the cached length %d", pos0, pos0 + n, c.length);
    HIP_TRY(hipSetDevice(m.device));
    HIP_TRY(hipDeviceSynchronize());
    size_t bytes = (size_t)n * m.cfg.d_model * 4;
    if (m.staging_bytes < bytes) {
        dev_free(m, m.staging);
        m.staging_bytes = 0;
        m.staging = (u16 *)dev_alloc(m, bytes);
        if (!m.staging) return fail(ODB_E_NOMEM, "cache_read staging");
        m.staging_bytes = bytes;
    }
    launch_cache_read(c, layer, kv, batch_index, pos0, n, (float *)m.staging, nullptr);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipDeviceSynchronize());
    HIP_TRY(hipMemcpy(host_f32, m.staging, bytes, hipMemcpyDeviceToHost));
    return ODB_OK;
}

int odb_block_step_static(odb_model *m, const odb_cache *c, const int32_t *drafts_dev, int block_off, int b, int S,
                          float tau, float *conf_dev, int32_t *argmax_dev, uint8_t *unmask_dev, void *stream) {
    if (!m) return fail(ODB_E_INVALID_ARG, "block_step_static: model is NULL");
    if (!conf_dev || !argmax_dev || !unmask_dev) return fail(ODB_E_INVALID_ARG, "block_step_static: NULL output");
    char *base = nullptr;
    int rc = static_scratch_ptr(m->m.device, &base);      // a table look-up after model creation
    if (rc) return rc;
    return step_impl(m, c, drafts_dev, block_off, b, S, tau, conf_dev, argmax_dev, unmask_dev, nullptr, stream, base,
                     kStaticScratchBytes);
}

}  // extern "C"

// ---- the fixed scratch area ---------------------------------------------------------------------------------
// Device memory that exists without any allocation call: every GPU the library runs on holds its own copy of
// this array at its own address.  In host code the name `scratch` is only a handle for hipGetSymbolAddress;
// the address it yields (per device, with that device current) is what kernels and copies are given.
static __device__ __align__(256) unsigned char scratch[ODB_STATIC_SCRATCH_BYTES];

namespace {
int static_scratch_ptr(int device, char **out) {
    if (device < 0 || device >= kMaxDevices) return fail(ODB_E_UNSUPPORTED, "device index %d", device);
    std::lock_guard<std::mutex> lock(g_static_scratch_mutex);
    if (!g_static_scratch[device]) {
        int cur = -1;
        HIP_TRY(hipGetDevice(&cur));
        if (cur != device) HIP_TRY(hipSetDevice(device));
        void *p = nullptr;
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (cur != device && cur >= 0) (void)hipSetDevice(cur);
        if (e != hipSuccess || !p) return fail(ODB_E_HIP, "hipGetSymbolAddress(scratch) on device %d: %s", device, hipGetErrorString(e));
        g_static_scratch[device] = (char *)p;
    }
    *out = g_static_scratch[device];
    return ODB_OK;
}
}  // namespace
