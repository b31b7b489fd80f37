// Weight generation, logical <-> physical layout copies, RoPE table, cache read-back.
#include "model.h"

namespace odb {

// ---- physical row -> (tensor id, logical row) -------------------------------
__host__ __device__ inline void phys_to_logical(int pk, int prow, int d, int dh, int &tid, int &lrow) {
    switch (pk) {
    case PK_QKV: {
        int sec = prow / d, r = prow % d;
        if (sec < 2) {
            int hd = r / dh, p = r % dh;
            int ch = (p & 1) ? (p >> 1) + dh / 2 : (p >> 1);
            lrow = hd * dh + ch;
            tid = sec == 0 ? ODB_T_WQ : ODB_T_WK;
        } else {
            lrow = r;
            tid = ODB_T_WV;
        }
        break;
    }
    case PK_GU: {
        lrow = prow >> 1;
        tid = (prow & 1) ? ODB_T_WU : ODB_T_WG;
        break;
    }
    case PK_O: tid = ODB_T_WO; lrow = prow; break;
    case PK_D: tid = ODB_T_WD; lrow = prow; break;
    case PK_LM: tid = ODB_T_LM; lrow = prow; break;
    default: tid = ODB_T_EMBED; lrow = prow; break;
    }
}

// chunk c (8 consecutive k-elements, 16 bytes) of a tiled [N,K] matrix -> (physical row, k)
__device__ inline void chunk_to_row_k(size_t c, int k_tiles, int &prow, int &k) {
    size_t tile = c >> 6;
    int lane = (int)(c & 63);
    int nt = (int)(tile / k_tiles), kt = (int)(tile % k_tiles);
    prow = nt * 16 + (lane & 15);
    k = kt * 32 + (lane >> 4) * 8;
}

// ---- counter-based normal generator ------------------------------------------
constexpr uint64_t kGamma = 0x9E3779B97F4A7C15ull;

__host__ __device__ inline uint64_t sm_finalise(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

static uint64_t stream_key(uint64_t seed, int tid, int layer) {
    uint64_t a = sm_finalise(seed + kGamma);
    uint64_t tag = ((uint64_t)(uint32_t)tid << 32) | (uint32_t)layer;
    return sm_finalise(a + tag + kGamma);
}

__device__ inline u16 normal_bf16(uint64_t key, uint64_t i, double std) {
    uint64_t z = sm_finalise(key + (i + 1) * kGamma);
    const double two32 = 1.0 / 4294967296.0;
    double u1 = ((double)(uint32_t)(z >> 32) + 0.5) * two32;
    double u2 = ((double)(uint32_t)z + 0.5) * two32;
    double x = sqrt(-2.0 * log(u1)) * cos(6.283185307179586 * u2);
    // binary64 -> binary32 -> bfloat16, each step to nearest even.  The second step is done on
    // the bit pattern so that the two roundings cannot be merged into one (they differ on ties).
    uint32_t u = __builtin_bit_cast(uint32_t, (float)(std * x));
    return (u16)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

// weights enter the MFMA as binary16: exact for bfloat16 values of magnitude 2^-16 .. 65504
__device__ inline u16 bf_to_h(u16 b) { return f2h(bf2f(b)); }
__device__ inline u16 h_to_bf(u16 h) { return f2bf(h2f(h)); }

struct GenKeys { uint64_t key[ODB_T_COUNT]; };

__global__ void gen_tiled_kernel(u16 *dst, size_t n_chunks, int pk, int K, int d, int dh, GenKeys keys, double std) {
    size_t c = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= n_chunks) return;
    int prow, k, tid, lrow;
    if (pk == PK_EMBED) {
        prow = (int)((c * 8) / K);
        k = (int)((c * 8) % K);
    } else {
        chunk_to_row_k(c, K / 32, prow, k);
    }
    phys_to_logical(pk, prow, d, dh, tid, lrow);
    uint64_t i0 = (uint64_t)lrow * K + k;
    uint64_t key = keys.key[tid];
    frag_t f;
#pragma unroll
    for (int j = 0; j < 4; j++) {
        u16 lo = normal_bf16(key, i0 + 2 * j, std);
        u16 hi = normal_bf16(key, i0 + 2 * j + 1, std);
        if (pk != PK_EMBED) { lo = bf_to_h(lo); hi = bf_to_h(hi); }
        f.w[j] = (uint32_t)lo | ((uint32_t)hi << 16);
    }
    *reinterpret_cast<frag_t *>(dst + c * 8) = f;
}

__global__ void fill_f32_kernel(float *p, float v, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

void launch_fill_f32(float *p, float v, size_t n, hipStream_t s) {
    if (n == 0) return;
    fill_f32_kernel<<<dim3((unsigned)((n + 255) / 256)), 256, 0, s>>>(p, v, n);
}

__global__ void fill_i32_kernel(int32_t *p, int32_t v, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

void launch_fill_i32(int32_t *p, int32_t v, size_t n, hipStream_t s) {
    if (n == 0) return;
    fill_i32_kernel<<<dim3((unsigned)((n + 255) / 256)), 256, 0, s>>>(p, v, n);
}

static int kind_k(const odb_config &c, int pk) { return pk == PK_D ? c.d_ff : c.d_model; }

void launch_init_random(const Model &m, uint64_t seed, double std, hipStream_t s) {
    const odb_config &c = m.cfg;
    for (int pk = 0; pk < PK_COUNT; pk++) {
        int layers = (pk == PK_LM || pk == PK_EMBED) ? 1 : c.n_layers;
        size_t n_chunks = m.layer_elems[pk] / 8;
        for (int l = 0; l < layers; l++) {
            GenKeys keys;
            for (int t = 0; t < ODB_T_COUNT; t++) keys.key[t] = stream_key(seed, t, l);
            gen_tiled_kernel<<<dim3((unsigned)((n_chunks + 255) / 256)), 256, 0, s>>>(
                m.w[pk] + (size_t)l * m.layer_elems[pk], n_chunks, pk, kind_k(c, pk), c.d_model, c.head_dim,
                keys, std);
        }
    }
    launch_fill_f32(m.g1, 1.0f, (size_t)c.n_layers * c.d_model, s);
    launch_fill_f32(m.g2, 1.0f, (size_t)c.n_layers * c.d_model, s);
    launch_fill_f32(m.gf, 1.0f, (size_t)c.d_model, s);
}

// ---- logical <-> physical copies ---------------------------------------------
__global__ void tensor_copy_kernel(u16 *phys, u16 *logical, size_t n_chunks, int pk, int K, int d, int dh,
                                   int want_tid, int to_model) {
    size_t c = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= n_chunks) return;
    int prow, k, tid, lrow;
    if (pk == PK_EMBED) {
        prow = (int)((c * 8) / K);
        k = (int)((c * 8) % K);
    } else {
        chunk_to_row_k(c, K / 32, prow, k);
    }
    phys_to_logical(pk, prow, d, dh, tid, lrow);
    if (tid != want_tid) return;
    frag_t *p = reinterpret_cast<frag_t *>(phys + c * 8);
    frag_t *q = reinterpret_cast<frag_t *>(logical + (size_t)lrow * K + k);
    frag_t v = to_model ? *q : *p;
    if (pk != PK_EMBED) {
#pragma unroll
        for (int j = 0; j < 4; j++) {
            u16 lo = (u16)(v.w[j] & 0xffff), hi = (u16)(v.w[j] >> 16);
            lo = to_model ? bf_to_h(lo) : h_to_bf(lo);
            hi = to_model ? bf_to_h(hi) : h_to_bf(hi);
            v.w[j] = (uint32_t)lo | ((uint32_t)hi << 16);
        }
    }
    if (to_model) *p = v; else *q = v;
}

static int tensor_kind(int tid) {
    switch (tid) {
    case ODB_T_EMBED: return PK_EMBED;
    case ODB_T_WQ: case ODB_T_WK: case ODB_T_WV: return PK_QKV;
    case ODB_T_WO: return PK_O;
    case ODB_T_WG: case ODB_T_WU: return PK_GU;
    case ODB_T_WD: return PK_D;
    default: return PK_LM;
    }
}

void launch_tensor_copy(const Model &m, int tensor_id, int layer, u16 *staging, bool to_model, hipStream_t s) {
    int pk = tensor_kind(tensor_id);
    if (pk == PK_LM || pk == PK_EMBED) layer = 0;
    size_t n_chunks = m.layer_elems[pk] / 8;
    tensor_copy_kernel<<<dim3((unsigned)((n_chunks + 255) / 256)), 256, 0, s>>>(
        m.w[pk] + (size_t)layer * m.layer_elems[pk], staging, n_chunks, pk, kind_k(m.cfg, pk), m.cfg.d_model,
        m.cfg.head_dim, tensor_id, to_model ? 1 : 0);
}

__global__ void gain_copy_kernel(float *gain, u16 *staging, int n, int to_model) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    if (to_model) gain[i] = bf2f(staging[i]); else staging[i] = f2bf(gain[i]);
}

void launch_gain_copy(float *gain, u16 *staging, int n, bool to_model, hipStream_t s) {
    gain_copy_kernel<<<dim3((n + 255) / 256), 256, 0, s>>>(gain, staging, n, to_model ? 1 : 0);
}

// ---- RoPE table -----------------------------------------------------------------
// table[pos][j] = (cos, sin)(pos * base^(-2j/dh)), evaluated in binary64.
__global__ void rope_table_kernel(float *table, int n_pos, int half, double base, double dh) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_pos * half) return;
    int pos = i / half, j = i % half;
    double ang = (double)pos * pow(base, -2.0 * (double)j / dh);
    table[2 * (size_t)i] = (float)cos(ang);
    table[2 * (size_t)i + 1] = (float)sin(ang);
}

void launch_rope_table(float *table, int n_pos, int dh, double base, hipStream_t s) {
    int n = n_pos * (dh / 2);
    rope_table_kernel<<<dim3((n + 255) / 256), 256, 0, s>>>(table, n_pos, dh / 2, base, (double)dh);
}

// ---- cache read-back ---------------------------------------------------------------
__global__ void cache_read_kernel(const u16 *kc, const u16 *vc, int kv, int H, int dh, int lmax32, int pos0, int n,
                                  float *out) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n * H * dh) return;
    int ch = i % dh, hd = (i / dh) % H, pos = pos0 + i / (dh * H);
    if (kv == 0) {
        int p = ch < dh / 2 ? 2 * ch : 2 * (ch - dh / 2) + 1;       // physical channel
        size_t tile = ((size_t)hd * (lmax32 / 16) + pos / 16) * (dh / 32) + p / 32;
        out[i] = h2f(kc[tile * kTileElems + tile_elem(pos & 15, p & 31)]);
    } else {
        int pl = pos & 31, t = pl >> 4, g = (pl & 15) >> 2, r = pl & 3;
        size_t tile = ((size_t)hd * (lmax32 / 32) + pos / 32) * (dh / 16) + ch / 16;
        out[i] = h2f(vc[tile * kTileElems + tile_elem(ch & 15, g * 8 + 4 * t + r)]);
    }
}

void launch_cache_read(const Cache &c, int layer, int kv, int batch_index, int pos0, int n, float *out, hipStream_t s) {
    const odb_config &cfg = c.m->cfg;
    size_t seq_elems = (size_t)cfg.n_heads * c.lmax32 * cfg.head_dim;
    const u16 *kc = c.k + (size_t)layer * c.layer_elems + (size_t)batch_index * seq_elems;
    const u16 *vc = c.v + (size_t)layer * c.layer_elems + (size_t)batch_index * seq_elems;
    int total = n * cfg.n_heads * cfg.head_dim;
    cache_read_kernel<<<dim3((total + 255) / 256), 256, 0, s>>>(kc, vc, kv, cfg.n_heads, cfg.head_dim, c.lmax32, pos0,
                                                                n, out);
}

}  // namespace odb
