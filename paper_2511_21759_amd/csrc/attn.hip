// Stand-alone launches of the attention core (see attn_core.h).
#include <mutex>

#include "attn_rows.h"

namespace odb {

template <int DH, int QT, int NW, bool SHARED = false>
__global__ __launch_bounds__(64 * NW) void attn_kernel(AttnArgs a, float sc) {
    __shared__ __attribute__((aligned(16))) char smem[attn_smem_bytes<QT, NW>()];
    attn_wg<DH, QT, NW, SHARED>(a, sc, blockIdx.x, blockIdx.y, smem);
}

// The same with a one-dimensional grid whose ids are mapped so that the gx work items of a head (the row tiles of
// a draft, the drafts of a block: they read the same cached K/V) run on one XCD (id % 8) and share its L2:
// id = xcd + 8 * (item + gx * (head / 8)), head = xcd + 8 * (head / 8).  H must be a multiple of 8.
template <int DH, int QT, int NW, bool SHARED = false>
__global__ __launch_bounds__(64 * NW) void attn_xcd_kernel(AttnArgs a, float sc, int gx) {
    __shared__ __attribute__((aligned(16))) char smem[attn_smem_bytes<QT, NW>()];
    const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
    attn_wg<DH, QT, NW, SHARED>(a, sc, j % gx, xcd + 8 * (j / gx), smem);
}

// Many rows per (sequence, head): K/V tiles shared through LDS by all rows of a workgroup (attn_rows.h)
template <int DH, int NW, int QTW, int NS>
static void launch_rows(AttnArgs a, float sc, hipStream_t s) {
    static std::once_flag attr_once;        // once per instantiation: the ring may need more than the default LDS limit
    std::call_once(attr_once, [] {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_rows_kernel<DH, NW, QTW, NS>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, attn_rows_smem_bytes<DH, NS>());
    });
    const int tiles_per_seq = a.units_per_seq * a.tiles_per_unit;
    const int chunks = (tiles_per_seq + NW * QTW - 1) / (NW * QTW);
    dim3 grid((a.units / a.units_per_seq) * chunks, a.H);
    // (flattened: the kernel then maps all row chunks of a head to one XCD - 38.9 -> 38.2 us at 1024 rows)
    if (a.H % 8 == 0 && grid.x > 1) grid = dim3(grid.x * grid.y, 1);
    attn_rows_kernel<DH, NW, QTW, NS><<<grid, 64 * NW, attn_rows_smem_bytes<DH, NS>(), s>>>(a, sc);
}

void launch_attention(AttnArgs a, hipStream_t s) {
    const float sc = 1.4426950408889634f / sqrtf((float)a.dh);
    if (a.split_tile > 0) {
        // decoded-share step: one row tile per workgroup, block_0 tiles first, then the speculative units'
        dim3 grid(a.mt_total, a.H);
        if (a.dh == 128 && a.H % 8 == 0 && grid.x > 1) attn_xcd_kernel<128, 1, 8, true><<<dim3(grid.x * grid.y), 512, 0, s>>>(a, sc, grid.x);
        else if (a.dh == 128) attn_kernel<128, 1, 8, true><<<grid, 512, 0, s>>>(a, sc);
        else attn_kernel<64, 1, 8, true><<<grid, 512, 0, s>>>(a, sc);
        return;
    }
    const int tiles_per_seq = a.units_per_seq * a.tiles_per_unit;
    if (tiles_per_seq >= 16 && (a.fresh == 0 || a.tiles_per_unit % 2 == 0)) {
        // 256 rows per workgroup when that still gives every compute unit a workgroup, else 128
        const int wgs8 = (a.units / a.units_per_seq) * ((tiles_per_seq + 15) / 16) * a.H;
        if (a.dh == 128) {
            if (wgs8 >= 256) launch_rows<128, 8, 2, 8>(a, sc, s);
            else launch_rows<128, 4, 2, 6>(a, sc, s);
        } else {
            if (wgs8 >= 256) launch_rows<64, 8, 2, 8>(a, sc, s);
            else launch_rows<64, 4, 2, 6>(a, sc, s);
        }
        return;
    }
    if (a.fresh > 0 && a.tiles_per_unit >= 2 && a.units * ((a.tiles_per_unit + 1) / 2) * a.H >= 128) {
        // decode step with at least 128 such workgroups (four drafts of 32 rows at 32 heads; fewer measured
        // slower than one row tile per workgroup): two row tiles of a draft per workgroup, so that a K/V tile
        // fetched from L2 serves 32 rows
        dim3 grid(a.units * ((a.tiles_per_unit + 1) / 2), a.H);
        // (the drafts of a head on one XCD: 11.8 -> 11.3 us at four drafts, a quarter of the K/V fetches)
        if (a.dh == 128 && a.H % 8 == 0 && grid.x > 1) attn_xcd_kernel<128, 2, 4><<<dim3(grid.x * grid.y), 256, 0, s>>>(a, sc, grid.x);
        else if (a.dh == 128) attn_kernel<128, 2, 4><<<grid, 256, 0, s>>>(a, sc);
        else attn_kernel<64, 2, 4><<<grid, 256, 0, s>>>(a, sc);
    } else if (a.fresh > 0) {
        // decode step: few rows, one 16-row tile per workgroup and eight waves over the keys
        dim3 grid(a.units * a.tiles_per_unit, a.H);
        // (both row tiles of a head on one XCD: 8.7 -> 8.4 us at 32 rows)
        if (a.dh == 128 && a.H % 8 == 0 && grid.x > 1) attn_xcd_kernel<128, 1, 8><<<dim3(grid.x * grid.y), 512, 0, s>>>(a, sc, grid.x);
        else if (a.dh == 128) attn_kernel<128, 1, 8><<<grid, 512, 0, s>>>(a, sc);
        else attn_kernel<64, 1, 8><<<grid, 512, 0, s>>>(a, sc);
    } else {
        constexpr int QT = 2;
        dim3 grid(a.units * ((a.tiles_per_unit + QT - 1) / QT), a.H);
        if (a.dh == 128) attn_kernel<128, QT, 4><<<grid, 256, 0, s>>>(a, sc);
        else attn_kernel<64, QT, 4><<<grid, 256, 0, s>>>(a, sc);
    }
}

}  // namespace odb
