// Small elementwise kernels used by more than one translation unit (each gets its own copy).
#pragma once
#include "ckks_internal.h"

namespace ckks {

constexpr u32 EW_THREADS = 256;

// canonical -> Montgomery form in rows [rows][N]; row r is modulo limb (r % period)
static __global__ __launch_bounds__(EW_THREADS) void to_mont_kernel(const u64 *in, u64 *out,
                                                                    const ModConst *__restrict__ mods, u32 period,
                                                                    u32 N) {
    const u32 n = blockIdx.x * EW_THREADS + threadIdx.x;
    const u32 row = blockIdx.y;
    const ModConst m = mods[row % period];
    const size_t idx = (size_t)row * N + n;
    out[idx] = mont_mul(in[idx], m.r2, m);
}

// dst[row][n] = dst[row][n] + src[row][n] mod limb (row % period)
static __global__ __launch_bounds__(EW_THREADS) void add_rows_kernel(u64 *dst, const u64 *__restrict__ src,
                                                                     const ModConst *__restrict__ mods, u32 period,
                                                                     u32 N) {
    const u32 n = blockIdx.x * EW_THREADS + threadIdx.x;
    const u32 row = blockIdx.y;
    const size_t idx = (size_t)row * N + n;
    dst[idx] = add_mod(dst[idx], src[idx], mods[row % period].q);
}

}  // namespace ckks
