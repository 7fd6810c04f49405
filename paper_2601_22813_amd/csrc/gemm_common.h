// Pieces shared by the GEMM kernels of libqii: vector types, the epilogue that stages a wave's
// 128 x 128 accumulator tile through LDS and stores full rows (optionally emitting max |C|), and the
// host helper that raises a kernel's dynamic LDS limit once per device.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "qii_device.h"

namespace qii {
namespace {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float float2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Optional by-product of the epilogue: max |C| over the stored values, for a consumer that
// quantizes C next and would otherwise have to read it once more just for its abs-max (the
// paper's layer timings assume the abs-max comes from the producing kernel, App. D).  One
// atomic without return per wave; non-negative floats order like their bit patterns.
__device__ __forceinline__ void emit_tile_max(float cmax, uint32_t *amax_out)
{
    if (!amax_out) return;   // uniform
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) cmax = fmaxf(cmax, __shfl_xor(cmax, off));
    if ((threadIdx.x & 63) == 0) atomicMax(amax_out, f2u(cmax));
}

// epilogue: C = acc * (x32_A * x32_B).  acc[r] of a 32x32 tile is row
// 8*(r/4) + 4*(lane/32) + r%4, column lane%32.  One 32-row band of the wave's 128x128 tile
// at a time goes through a per-wave LDS tile (row pitch padded by 16 bytes) and leaves as
// 16-byte pieces of full rows.  The caller guarantees that nobody reads the stages any more.
template <bool kBf16Out, bool kStreaming = true>
__device__ __forceinline__ void store_tile_through_lds(floatx16 (&acc)[4][4], uint8_t *smem, float ts,
                                                       void *Cout, int64_t ldc, int64_t M, int64_t N,
                                                       int64_t m0, int64_t n0, int wave, int wm, int wn,
                                                       int lane, int li, int kb, uint32_t *amax_out)
{
    float cmax = 0.0f;
    constexpr int esz = kBf16Out ? 2 : 4;
    constexpr int pitch = 128 * esz + 16;
    uint8_t *wtile = smem + wave * (32 * pitch);
    constexpr int per_row = 128 * esz / 16;          // 16-byte pieces per row
    constexpr int rows_per_pass = 64 / per_row;      // rows covered by one wave-wide store
#pragma unroll
    for (int ti = 0; ti < 4; ++ti) {
#pragma unroll
        for (int tj = 0; tj < 4; ++tj)
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
                // two consecutive rows of one column: one packed conversion (round to nearest even)
                const int row = 8 * (r >> 2) + 4 * kb + (r & 3), col = tj * 32 + li;
                const float v0 = acc[ti][tj][r] * ts, v1 = acc[ti][tj][r + 1] * ts;
                if (kBf16Out) {
                    const bf16x2_t pk = __builtin_convertvector(float2_t{v0, v1}, bf16x2_t);
                    const uint32_t bits = __builtin_bit_cast(uint32_t, pk);
                    *reinterpret_cast<uint16_t *>(wtile + row * pitch + col * 2) = (uint16_t)bits;
                    *reinterpret_cast<uint16_t *>(wtile + (row + 1) * pitch + col * 2) = (uint16_t)(bits >> 16);
                } else {
                    *reinterpret_cast<float *>(wtile + row * pitch + col * 4) = v0;
                    *reinterpret_cast<float *>(wtile + (row + 1) * pitch + col * 4) = v1;
                }
            }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // wave-local: same wave reads below
#pragma unroll
        for (int pass = 0; pass < 32 / rows_per_pass; ++pass) {
            const int row = pass * rows_per_pass + lane / per_row, piece = lane % per_row;
            const uint4 v = *reinterpret_cast<const uint4 *>(wtile + row * pitch + piece * 16);
            const int64_t grow = m0 + wm * 128 + ti * 32 + row;
            const int64_t gcol = n0 + wn * 128 + piece * (16 / esz);
            if (grow < M) {
                if (amax_out) {   // uniform: max |C| over the entries of this piece that lie inside the matrix
                    const uint32_t w4[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                    for (int e = 0; e < 16 / esz; ++e)
                        if (gcol + e < N)
                            cmax = fmaxf(cmax, fabsf(kBf16Out ? u2f((e & 1) ? (w4[e >> 1] & 0xFFFF0000u) : (w4[e >> 1] << 16)) : u2f(w4[e])));
                }
                uint8_t *dst = reinterpret_cast<uint8_t *>(Cout) + (grow * ldc + gcol) * esz;
                if (gcol + 16 / esz <= N && ((reinterpret_cast<uintptr_t>(dst) & 15) == 0)) {
                    // C is written once and not read again here: a streaming (non-temporal) store
                    // (kStreaming = false: a partial tile that the next kernel reads back)
                    if (kStreaming) __builtin_nontemporal_store(u32x4{v.x, v.y, v.z, v.w}, reinterpret_cast<u32x4 *>(dst));
                    else *reinterpret_cast<u32x4 *>(dst) = u32x4{v.x, v.y, v.z, v.w};
                } else {
                    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                    for (int e = 0; e < 16 / esz; ++e)
                        if (gcol + e < N) {
                            if (kBf16Out) reinterpret_cast<uint16_t *>(dst)[e] = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
                            else reinterpret_cast<uint32_t *>(dst)[e] = w[e];
                        }
                }
            }
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // reads done before the next band overwrites
    }
    emit_tile_max(cmax, amax_out);
}

// The kernels need more dynamic LDS than the default limit; the attribute is set once per kernel
// and device, not per launch (a launch may sit inside a stream capture).
template <class Kern>
hipError_t allow_dynamic_lds(Kern kern, int bytes)
{
    constexpr int kMaxDevices = 64;
    static bool done[kMaxDevices] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < kMaxDevices && done[dev]) return hipSuccess;
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess && dev >= 0 && dev < kMaxDevices) done[dev] = true;
    return e;
}

}  // namespace
}  // namespace qii
