// Stand-alone launches of the weight-streaming GEMM (see gemm_core.h).
#include "gemm_core.h"

namespace odb {

template <int MT, int NG, int PF, class Epi>
__global__ __launch_bounds__(64 * WK) void gemm_stream_kernel(GemmArgs g, Epi epi) {
    __shared__ __attribute__((aligned(16))) char smem[kGemmSmemBytes];
    frag_t wb[PF][NG];
    gemm_wg<MT, NG, PF, false>(g, epi, blockIdx.x, gridDim.x, blockIdx.y * MT, wb, smem);
}

// an epilogue "maker" yields the epilogue object for a given m-tile count (most are independent of it)
template <class Epi> struct Same {
    Epi e;
    template <int MT> Epi for_mt() const { return e; }
};
struct LMStatsMaker {
    float *stats;
    int n_part;
    template <int MT> EpiLMStats<MT / 2> for_mt() const { return EpiLMStats<MT / 2>(stats, n_part); }
};

// ---- launch ---------------------------------------------------------------------
constexpr int kStreamWGs = 256;      // one workgroup per compute unit

template <int NG, class Maker>
static void launch(const u16 *a, const u16 *w, GemmShape sh, NormIn ni, Maker mk, hipStream_t s) {
    GemmArgs g;
    g.A = a; g.W = w; g.KT = sh.K_tiles; g.MT_total = sh.M_tiles; g.NT = sh.N_tiles;
    g.ssq = ni.ssq; g.n_ssq = ni.n_ssq; g.eps = ni.eps; g.inv_d = 1.0f / (float)(sh.K_tiles * 32);
    const int kw = sh.K_tiles / WK;                 // K_tiles is a multiple of 8 (checked at model creation)
    const int groups = (sh.N_tiles + NG - 1) / NG;
    const int wgs = groups < kStreamWGs ? groups : kStreamWGs;
    if (sh.M_tiles <= 2) {
        dim3 grid(wgs, 1);
        auto e = mk.template for_mt<2>();
        if (kw % 8 == 0) gemm_stream_kernel<2, NG, 8, decltype(e)><<<grid, 64 * WK, 0, s>>>(g, e);
        else gemm_stream_kernel<2, NG, 1, decltype(e)><<<grid, 64 * WK, 0, s>>>(g, e);
    } else {
        dim3 grid(wgs, (sh.M_tiles + 7) / 8);
        auto e = mk.template for_mt<8>();
        if (kw % 2 == 0) gemm_stream_kernel<8, NG, 2, decltype(e)><<<grid, 64 * WK, 0, s>>>(g, e);
        else gemm_stream_kernel<8, NG, 1, decltype(e)><<<grid, 64 * WK, 0, s>>>(g, e);
    }
}

void launch_gemm_qkv(const u16 *xa, const u16 *w, GemmShape sh, NormIn ni, QkvOut out, hipStream_t s) {
    launch<3>(xa, w, sh, ni, Same<EpiQKV>{EpiQKV{out, sh.M_tiles}}, s);
}
void launch_gemm_resid(const u16 *a, const u16 *w, GemmShape sh, float *h, int ldh, NormOut no, hipStream_t s) {
    launch<1>(a, w, sh, NormIn{nullptr, 0, 0.f}, Same<EpiResid>{EpiResid{h, ldh, no, sh.M_tiles}}, s);
}
void launch_gemm_swiglu(const u16 *xa, const u16 *w, GemmShape sh, NormIn ni, u16 *act, hipStream_t s) {
    launch<3>(xa, w, sh, ni, Same<EpiSwiGLU>{EpiSwiGLU{act, sh.M_tiles}}, s);
}
int lm_stats_parts(int n_tiles) {
    const int groups = (n_tiles + 2) / 3;
    return (groups < kStreamWGs ? groups : kStreamWGs) * 3;
}

void launch_gemm_lmstats(const u16 *xa, const u16 *w, GemmShape sh, NormIn ni, float *stats, hipStream_t s) {
    launch<3>(xa, w, sh, ni, LMStatsMaker{stats, lm_stats_parts(sh.N_tiles)}, s);
}
void launch_gemm_store(const u16 *xa, const u16 *w, GemmShape sh, NormIn ni, float *out, int units, int rpu_pad,
                       int valid, int ld, hipStream_t s) {
    launch<3>(xa, w, sh, ni, Same<EpiStore>{EpiStore{out, units, rpu_pad, valid, ld}}, s);
}

}  // namespace odb
