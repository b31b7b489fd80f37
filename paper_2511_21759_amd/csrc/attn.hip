// Stand-alone launches of the attention core (see attn_core.h).
#include "attn_core.h"

namespace odb {

template <int DH, int QT, int NW>
__global__ __launch_bounds__(64 * NW) void attn_kernel(AttnArgs a, float sc) {
    __shared__ __attribute__((aligned(16))) char smem[attn_smem_bytes<QT, NW>()];
    attn_wg<DH, QT, NW>(a, sc, blockIdx.x, blockIdx.y, smem);
}

void launch_attention(AttnArgs a, hipStream_t s) {
    const float sc = 1.4426950408889634f / sqrtf((float)a.dh);
    if (a.fresh > 0 && a.tiles_per_unit >= 3 && a.units * ((a.tiles_per_unit + 3) / 4) * a.H >= 512) {
        // decode step with long blocks and many drafts or sequences: four row tiles of a draft per workgroup,
        // so that a K/V tile fetched from L2 serves 64 rows (a quarter of the cache traffic of the case below)
        dim3 grid(a.units * ((a.tiles_per_unit + 3) / 4), a.H);
        if (a.dh == 128) attn_kernel<128, 4, 4><<<grid, 256, 0, s>>>(a, sc);
        else attn_kernel<64, 4, 4><<<grid, 256, 0, s>>>(a, sc);
    } else if (a.fresh > 0) {
        // decode step: few rows, one 16-row tile per workgroup and eight waves over the keys
        dim3 grid(a.units * a.tiles_per_unit, a.H);
        if (a.dh == 128) attn_kernel<128, 1, 8><<<grid, 512, 0, s>>>(a, sc);
        else attn_kernel<64, 1, 8><<<grid, 512, 0, s>>>(a, sc);
    } else {
        constexpr int QT = 4;
        dim3 grid(a.units * ((a.tiles_per_unit + QT - 1) / QT), a.H);
        if (a.dh == 128) attn_kernel<128, QT, 4><<<grid, 256, 0, s>>>(a, sc);
        else attn_kernel<64, QT, 4><<<grid, 256, 0, s>>>(a, sc);
    }
}

}  // namespace odb
