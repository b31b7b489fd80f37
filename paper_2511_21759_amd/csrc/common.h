// Shared device-side definitions: MFMA fragment types and the tiled layouts.
//
// Every matrix that feeds an MFMA lives in HBM as a sequence of 1 KiB "operand
// tiles" of 16 rows x 32 k-elements of binary16, stored in the register order of
// v_mfma_f32_16x16x32_f16: lane l of a wavefront owns row (l & 15) and the 8
// consecutive k-elements starting at 8*(l >> 4).  A wave loads a tile with one
// 16-byte load per lane from 1 KiB of contiguous memory and hands the register
// straight to the MFMA, as either operand:
//     D = mfma(X, Y, D)   computes   D[i][j] += sum_k X[i][k] * Y[j][k]
// with the result held as lane l -> D[4*(l>>4) + r][l & 15], r = 0..3.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace odb {

// Operands are IEEE binary16 (11-bit significand), accumulation is fp32.  The model's weights are
// bfloat16 VALUES (8-bit significand); every such value of magnitude 2^-16 .. 65504 is exactly
// representable in binary16, so they are converted once when they enter the library.  Activations
// rounded to bfloat16 instead would cost 8x the rounding noise per GEMM input, which after 32 layers
// exceeds the 1e-2 bound on the K/V cache (measured 2.3e-2) - at the same MFMA rate.
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned short u16;

constexpr int kTileRows = 16;
constexpr int kTileK = 32;
constexpr int kTileElems = 512;   // 1 KiB of binary16
constexpr int kWave = 64;

struct __attribute__((aligned(16))) frag_t { uint32_t w[4]; };   // 8 binary16

// offset of element (row r, k-element kk) inside a tile
__host__ __device__ inline int tile_elem(int r, int kk) {
    return ((kk >> 3) * 16 + r) * 8 + (kk & 7);
}

__device__ inline u16 f2bf(float x) {          // bfloat16, round to nearest even
    return __builtin_bit_cast(u16, (__bf16)x);
}
__device__ inline float bf2f(u16 b) {
    return __builtin_bit_cast(float, (uint32_t)b << 16);
}
__device__ inline u16 f2h(float x) {           // binary16, round to nearest even, saturating
    x = fminf(fmaxf(x, -65504.f), 65504.f);
    return __builtin_bit_cast(u16, (_Float16)x);
}
// Conversions to binary16 saturate silently; a kernel that rounds activations calls this beside them so that a value
// beyond the binary16 range (or a NaN) is reported instead: bit kStatusSaturated of the model's status word is set
// and odb_model_status turns it into an error.  Rare path: one compare per four values otherwise.
constexpr unsigned kStatusSharedOverflow = 2u, kStatusSaturated = 4u;
__device__ __forceinline__ void note_saturation(unsigned *status, float a, float b, float c, float d) {
    const float m = fmaxf(fmaxf(fabsf(a), fabsf(b)), fmaxf(fabsf(c), fabsf(d)));
    if (status && !(m <= 65504.f)) atomicOr(status, kStatusSaturated);
}
__device__ inline float h2f(u16 b) {
    return (float)__builtin_bit_cast(_Float16, b);
}
__device__ inline uint32_t pack2(float lo, float hi) {      // two operand elements
    return (uint32_t)f2h(lo) | ((uint32_t)f2h(hi) << 16);
}

// Two operand elements from values known to lie inside the binary16 range (attention probabilities, at most
// 2^kAttnSlack): round to nearest even, no clamp - one packed conversion instead of two clamps, two conversions and a merge.
__device__ inline uint32_t pack2_inrange(float lo, float hi) {
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{lo, hi}, f16x2_t));
}

__device__ inline frag_t ld_frag(const u16 *p) {
    return *reinterpret_cast<const frag_t *>(p);
}

// The same load marked non-temporal, for data that is read once per kernel (weight tiles): the plain streaming
// read of 8 GiB measures 5.9-6.25 TB/s on MI355X with ordinary loads and 6.6-7.1 TB/s with these.
__device__ inline frag_t ld_frag_stream(const u16 *p) {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    return __builtin_bit_cast(frag_t, __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p)));
}

__device__ inline f32x4 mfma16(const frag_t &x, const frag_t &y, f32x4 acc) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(
        __builtin_bit_cast(f16x8, x), __builtin_bit_cast(f16x8, y), acc, 0, 0, 0);
}

// s_waitcnt vmcnt(n) for a run-time n (the instruction takes an immediate)
__device__ __forceinline__ void wait_vmcnt(int n) {
    switch (n) {
#define ODB_VMCNT_CASE(N) case N: asm volatile("s_waitcnt vmcnt(" #N ")" ::: "memory"); break;
        ODB_VMCNT_CASE(1) ODB_VMCNT_CASE(2) ODB_VMCNT_CASE(3) ODB_VMCNT_CASE(4) ODB_VMCNT_CASE(5) ODB_VMCNT_CASE(6)
        ODB_VMCNT_CASE(7) ODB_VMCNT_CASE(8) ODB_VMCNT_CASE(9) ODB_VMCNT_CASE(10) ODB_VMCNT_CASE(11) ODB_VMCNT_CASE(12)
        ODB_VMCNT_CASE(13) ODB_VMCNT_CASE(14) ODB_VMCNT_CASE(15) ODB_VMCNT_CASE(16) ODB_VMCNT_CASE(18) ODB_VMCNT_CASE(20)
        ODB_VMCNT_CASE(24) ODB_VMCNT_CASE(28)
#undef ODB_VMCNT_CASE
        default: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;      // also every count not listed: waits for more
    }
}

}  // namespace odb
