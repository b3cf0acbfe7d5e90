// 64-bit modular arithmetic for gfx950, built from 32x32->64 multiply-adds.
//
// All residues live in canonical form [0, q) with q < 2^62.  Every constant
// operand the library owns (twiddles, base-conversion factors, key and weight
// limbs) is stored in Montgomery form x*2^64 mod q, so that one Montgomery
// reduction of (canonical * Montgomery-form) lands back in canonical form.
// Sums of products are kept as 128-bit integers and reduced once.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ckks {

typedef uint64_t u64;
typedef uint32_t u32;

struct u128 {
    u64 lo, hi;
};

// Per-modulus constants, one entry per RNS limb.
struct ModConst {
    u64 q;       // the prime
    u64 qinv;    // q^-1 mod 2^64
    u64 r2;      // 2^128 mod q (canonical -> Montgomery form by mont_mul(x, r2))
    u64 one;     // 2^64 mod q  (Montgomery form of 1)
};

__host__ __device__ __forceinline__ u128 mul_wide(u64 a, u64 b) {
#if defined(__HIP_DEVICE_COMPILE__)
    // four 32x32 partial products chained through v_mad_u64_u32
    u32 a0 = (u32)a, a1 = (u32)(a >> 32), b0 = (u32)b, b1 = (u32)(b >> 32);
    u64 p00 = (u64)a0 * b0;
    u64 p01 = (u64)a0 * b1 + (p00 >> 32);           // < 2^64: (2^32-1)^2 + 2^32-1
    u64 p10 = (u64)a1 * b0 + (u32)p01;              // same bound
    u64 p11 = (u64)a1 * b1 + (p01 >> 32) + (p10 >> 32);
    u128 r;
    r.lo = (p10 << 32) | (u32)p00;
    r.hi = p11;
    return r;
#else
    unsigned __int128 p = (unsigned __int128)a * b;
    u128 r;
    r.lo = (u64)p;
    r.hi = (u64)(p >> 64);
    return r;
#endif
}

__host__ __device__ __forceinline__ u64 mul_hi(u64 a, u64 b) { return mul_wide(a, b).hi; }

__host__ __device__ __forceinline__ void acc_add(u128 &acc, u128 p) {
    acc.lo += p.lo;
    acc.hi += p.hi + (acc.lo < p.lo);
}

// acc += a*b
__host__ __device__ __forceinline__ void mac(u128 &acc, u64 a, u64 b) { acc_add(acc, mul_wide(a, b)); }

// Montgomery reduction: T*2^-64 mod q for T < q*2^64, result in [0, q).
__host__ __device__ __forceinline__ u64 redc(u128 t, const ModConst &m) {
    u64 k = t.lo * m.qinv;                 // k*q == t.lo (mod 2^64)
    u64 h = mul_hi(k, m.q);                // (T - k*q)/2^64 = t.hi - h, in (-q, q)
    u64 r = t.hi - h;
    return t.hi < h ? r + m.q : r;
}

// Montgomery reduction for T < c*q*2^64 with small c (lazy sums): result in [0, q).
__host__ __device__ __forceinline__ u64 redc_wide(u128 t, const ModConst &m) {
    u64 k = t.lo * m.qinv;
    u64 h = mul_hi(k, m.q);                // h < q
    u64 r = t.hi - h;                      // true value t.hi - h in (-q, c*q)
    if (t.hi < h) return r + m.q;
    while (r >= m.q) r -= m.q;
    return r;
}

// canonical a times Montgomery-form b -> canonical a*b mod q
__host__ __device__ __forceinline__ u64 mont_mul(u64 a, u64 b, const ModConst &m) {
    return redc(mul_wide(a, b), m);
}

__host__ __device__ __forceinline__ u64 add_mod(u64 a, u64 b, u64 q) {
    u64 s = a + b;
    return s >= q ? s - q : s;
}

__host__ __device__ __forceinline__ u64 sub_mod(u64 a, u64 b, u64 q) {
    return a >= b ? a - b : a + q - b;
}

// x in [0, 2^64) -> x mod q (an operand that comes from another modulus):
// x * (2^64 mod q) < 2^64 * q is a valid redc input and reduces to x mod q.
__host__ __device__ __forceinline__ u64 reduce_any(u64 x, const ModConst &m) {
    return redc(mul_wide(x, m.one), m);
}

// signed 64-bit integer -> canonical residue
__host__ __device__ __forceinline__ u64 reduce_signed(int64_t v, const ModConst &m) {
    u64 a = v < 0 ? (u64)0 - (u64)v : (u64)v;
    u64 r = reduce_any(a, m);
    return (v < 0 && r) ? m.q - r : r;
}

}  // namespace ckks
