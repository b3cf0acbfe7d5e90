// Hybrid key switching for rot / conj (Table 1) with the input-side work hoisted.
//
// The paper treats rot and conj as primitives and says nothing about how they
// are evaluated; this is the standard RNS hybrid method with dnum digits:
//   decompose:  INTT(c1) -> per digit D_j approximate base conversion of
//               [c1]_{Q_Dj} to every other active limb and to the special
//               primes (ModUp) -> NTT.  Done ONCE per ciphertext.
//   switch:     per Galois element g: u = sum_j sigma_g(d_j) (.) key_j over the
//               level+K limbs (the automorphism is an index gather in the NTT
//               domain, fused into the loads) -> INTT of the K special limbs ->
//               base conversion P -> Q, subtract, times P^-1 (ModDown) ->
//               + sigma_g(c0).
// Base conversions use no floating-point correction term; sums of products are
// accumulated in 128 bits and reduced once.
#include <algorithm>

#include "ckks_internal.h"
#include "common_kernels.h"
#include "ntt_device.h"

namespace ckks {

constexpr u32 KS_THREADS = EW_THREADS;
constexpr u32 DN_CHUNK = 24;   // target limbs per workgroup in ModDown (2, 3, 4, 6, 12, 24 measured: fewer, larger groups are faster)

__device__ __forceinline__ u32 galois_index(u32 k, u64 g, u32 logN) {
    // entry k holds the value at psi^(2*bitrev(k)+1); sigma_g reads the value at that exponent times g
    u32 e = 2u * (__brev(k) >> (32 - logN)) + 1u;
    u32 e2 = (u32)(((u64)e * g) & ((2ull << logN) - 1));
    return __brev((e2 - 1u) >> 1) >> (32 - logN);
}

struct PtrPack {
    const u64 *p[ROT_BATCH];
};

// tmp[r][i][n] = src_r[i][n]: collects the c1 halves of up to ROT_BATCH ciphertexts
__global__ __launch_bounds__(KS_THREADS) void gather_c1_kernel(PtrPack src, u64 *__restrict__ tmp, u32 level, u32 N) {
    const u32 n = blockIdx.x * KS_THREADS + threadIdx.x;
    const u32 i = blockIdx.y, r = blockIdx.z;
    tmp[((size_t)r * level + i) * N + n] = src.p[r][(size_t)i * N + n];
}

// The same collection fused with the first pass of the inverse transform (rings with the two-pass kernels):
// reads the c1 halves where they are, writes tmp[r][i] half transformed.  grid: x = 4096-residue tiles,
// y = r * level + i.
__global__ __launch_bounds__(NTT_THREADS) void gather_intt_kernel(PtrPack src, u64 *__restrict__ tmp,
                                                                  const ModConst *__restrict__ mods,
                                                                  const ModFp *__restrict__ modf,
                                                                  const u64 *__restrict__ tw,
                                                                  const double *__restrict__ twf,
                                                                  const u64 *__restrict__ ninv, u32 level, u32 logN) {
    __shared__ u64 lds[FAST_LDS_WORDS];
    const u32 r = blockIdx.y / level, i = blockIdx.y % level;
    const u64 *in = src.p[r] + ((size_t)i << logN);
    u64 *out = tmp + ((size_t)blockIdx.y << logN);
    auto load = [&](u32 idx) { return in[idx]; };
    auto store = [&](u32 idx, u64 v) { out[idx] = v; };
    const ModFp mf = modf[i];
    if (mf.ok)
        pass_b_body<true>(make_field_fp(mf, twf, i, logN), logN, lds, load, store);
    else
        pass_b_body<true>(make_field_int(mods, tw, ninv, i, logN), logN, lds, load, store);
}

// Per ciphertext r and digit j: y_i = c_i * (Q_D/q_i)^-1 mod q_i for the limbs of the digit, then for
// every target t outside the digit out_t = sum_i y_i * (Q_D/q_i mod t) mod t (coefficient domain).
// Targets inside the digit are left out: in the NTT domain they are the input's own rows, which the consumers
// read in place (no copy, no transform).
// grid: x = pairs of coefficients, y = digit, z = ciphertext; targets t0 .. t1-1.  A thread owns two
// adjacent coefficients (16-byte accesses) so that every conversion factor, which is workgroup-uniform and
// arrives through the scalar cache, serves two multiply-accumulates; AMAX bounds the digit size.
template <u32 AMAX, u32 VEC, bool FP>
__global__ __launch_bounds__(KS_THREADS) void modup_kernel(const u64 *__restrict__ c1_coeff,
                                                           u64 *__restrict__ digits,
                                                           const ModConst *__restrict__ mods,
                                                           const ModFp *__restrict__ modf,
                                                           const u64 *__restrict__ up_inv,
                                                           const u64 *__restrict__ up_mat,
                                                           const u64 *__restrict__ up_matf, u32 level, u32 K, u32 L,
                                                           u32 alpha, u32 N, u32 beta, u32 t0, u32 t1) {
    typedef u64 vec_t __attribute__((ext_vector_type(2)));
    const u32 n = (blockIdx.x * KS_THREADS + threadIdx.x) * VEC;
    const u32 j = blockIdx.y;
    const u32 r = blockIdx.z;
    const u32 Wl = level + K;
    const u32 lo = j * alpha, hi = min(lo + alpha, level);
    const u64 *coef = c1_coeff + (size_t)r * level * N;
    u64 *dig = digits + (size_t)r * beta * Wl * N;
    u64 y[AMAX][VEC];
#pragma unroll
    for (u32 a = 0; a < AMAX; ++a) {
#pragma unroll
        for (u32 e = 0; e < VEC; ++e) y[a][e] = 0;
        if (lo + a < hi) {
            const u64 inv = up_inv[lo + a];
            const ModConst m = mods[lo + a];
#pragma unroll
            for (u32 e = 0; e < VEC; e += 2) {
                const vec_t c = *reinterpret_cast<const vec_t *>(coef + (size_t)(lo + a) * N + n + e);
                y[a][e] = mont_mul(c[0], inv, m);
                y[a][e + 1] = mont_mul(c[1], inv, m);
            }
        }
    }
    if (FP) {
        // Every prime involved is below 2^50 (the launcher checks): y is exact in a double, every product is
        // split exactly into h + l and brought below 0.9 q before it is added, and the partial sum is reduced
        // every four terms (below 2^53).  Twice the multiply rate of the 32-bit integer pipeline.
        double yd[AMAX][VEC];
#pragma unroll
        for (u32 a = 0; a < AMAX; ++a)
#pragma unroll
            for (u32 e = 0; e < VEC; ++e) yd[a][e] = (double)y[a][e];
        for (u32 t = t0; t < t1; ++t) {
            if (t >= lo && t < hi) continue;      // the digit's own limbs: consumers read them from the source
            u64 *dst = dig + ((size_t)j * Wl + t) * N + n;
            const double q = modf[t].q, u = modf[t].u;
            double fd[AMAX], acc[VEC];
#pragma unroll
            for (u32 a = 0; a < AMAX; ++a)
                fd[a] = lo + a < hi ? __longlong_as_double((long long)up_matf[(size_t)(lo + a) * Wl + t]) : 0.0;
#pragma unroll
            for (u32 e = 0; e < VEC; ++e) acc[e] = 0.0;
#pragma unroll
            for (u32 a = 0; a < AMAX; ++a) {
#pragma unroll
                for (u32 e = 0; e < VEC; ++e) {
                    const double h = yd[a][e] * fd[a], l = fma(yd[a][e], fd[a], -h);
                    acc[e] += fma(-rint(h * u), q, h) + l;
                    if ((a & 3) == 3) acc[e] = fma(-rint(acc[e] * u), q, acc[e]);
                }
            }
#pragma unroll
            for (u32 e = 0; e < VEC; e += 2) {
                vec_t o;
#pragma unroll
                for (u32 z = 0; z < 2; ++z) {
                    double v = fma(-rint(acc[e + z] * u), q, acc[e + z]);
                    if (v < 0) v += q;
                    o[z] = (u64)v;
                }
                *reinterpret_cast<vec_t *>(dst + e) = o;
            }
        }
    } else {
        for (u32 t = t0; t < t1; ++t) {
            if (t >= lo && t < hi) continue;
            u64 *dst = dig + ((size_t)j * Wl + t) * N + n;
            const u32 gl = t < level ? t : L + (t - level);
            u64 f[AMAX];
#pragma unroll
            for (u32 a = 0; a < AMAX; ++a) f[a] = lo + a < hi ? up_mat[(size_t)(lo + a) * Wl + t] : 0;
            u128 acc[VEC];
#pragma unroll
            for (u32 e = 0; e < VEC; ++e) acc[e] = {0, 0};
#pragma unroll
            for (u32 a = 0; a < AMAX; ++a)        // a factor of 0 pads digits shorter than AMAX
#pragma unroll
                for (u32 e = 0; e < VEC; ++e) mac(acc[e], y[a][e], f[a]);
            const ModConst mt = mods[gl];
#pragma unroll
            for (u32 e = 0; e < VEC; e += 2) {
                vec_t o;
                o[0] = redc_wide(acc[e], mt);     // up to AMAX products below 2^62 * q each
                o[1] = redc_wide(acc[e + 1], mt);
                *reinterpret_cast<vec_t *>(dst + e) = o;
            }
        }
    }
}

// Decomposition between the two tile passes at N = 2^16, one kernel instead of four.  The last 4 stages of the
// inverse transform of c1, the base conversion of every digit (ModUp) and the first 4 stages of the forward transform
// of the extended rows all work on columns (residues 4096 apart); a workgroup owns UP_COLS columns of one digit of one
// ciphertext:
//   1. thread (a, col): column col of limb lo + a of the digit, 16 rows in registers, last inverse round with
//      N^-1 (Q_D/q_i)^-1 folded in -> y_a in LDS;
//   2. thread (row pair, col): for each group of UP_TG targets and each of its two coefficients: targets among the
//      ciphertext primes as the exact fp64 sums of modup_kernel; targets among the special primes from 25-bit pieces
//      of y and 20-bit parts of the factors (48 exact fp64 multiply-adds, then one Montgomery reduction of the
//      recombined 90-bit sum) -> LDS;
//   3. thread (target, col): 16 rows from LDS, first forward round (fp64 or integer butterflies), out.
// c1_half [n][level][N]: c1 after the inverse tile pass; digits [n][beta][level+K][N]: rows of targets outside the
// digit, ready for the forward tile pass.  Needs alpha, K <= 8, every active ciphertext prime below 2^50 and every
// special prime below 2^60 (the launcher checks).  grid: x = column tile, y = digit, z = ciphertext.
constexpr u32 UP_COLS = 32, UP_TG = 8;
__global__ __launch_bounds__(256) void modup_mid_kernel(const u64 *__restrict__ c1_half, u64 *__restrict__ digits,
                                                        const ModConst *__restrict__ mods,
                                                        const ModFp *__restrict__ modf,
                                                        const ModFp *__restrict__ modf_up,
                                                        const double *__restrict__ twf_inv,
                                                        const double *__restrict__ twf_fwd,
                                                        const u64 *__restrict__ tws_fwd,
                                                        const u64 *__restrict__ ninvs,
                                                        const double *__restrict__ up_ft,
                                                        const double *__restrict__ up_mats, u32 level, u32 K, u32 L,
                                                        u32 alpha, u32 beta, u32 tsplit) {
    constexpr u32 logN = 16, N = 1u << logN;
    static_assert(UP_TG == 8, "the target tiles reuse the 8 rows of source tiles");
    __shared__ u64 ylds[8 * 16 * UP_COLS];
    u64 *wlds = ylds;               // the sources live in registers once step 2 has read them: the same 32 KiB
    const u32 tid = threadIdx.x, col = tid & (UP_COLS - 1), grp = tid / UP_COLS;   // grp < 8
    // tsplit > 1 (few ciphertexts): the groups of targets of a tile go to tsplit workgroups, each of which redoes the
    // cheap step 1, so that a lone decomposition still fills the chip
    const u32 tile = blockIdx.x % (4096 / UP_COLS), tpart = blockIdx.x / (4096 / UP_COLS);
    const u32 c0 = tile * UP_COLS + col;
    const u32 j = blockIdx.y, r = blockIdx.z;
    const u32 Wl = level + K;
    const u32 lo = j * alpha, hi = min(lo + alpha, level), nd = hi - lo;
    if (grp < nd) {
        const u32 i = lo + grp;
        const u64 *src = c1_half + ((size_t)r * level + i) * N;
        auto load = [&](u32 idx) { return src[idx]; };
        auto store = [&](u32 idx, u64 v) { ylds[(grp * 16 + (idx >> 12)) * UP_COLS + col] = v; };
        pass_a16_body<true>(make_field_fp(modf_up[i], twf_inv, i, logN), c0, load, store);
    }
    __syncthreads();
    u64 yraw[2][8];
#pragma unroll
    for (u32 e = 0; e < 2; ++e)
#pragma unroll
        for (u32 a = 0; a < 8; ++a) yraw[e][a] = a < nd ? ylds[(a * 16 + 2 * grp + e) * UP_COLS + col] : 0;
    __syncthreads();                // every thread has its y: the tile may be overwritten
    u64 *dig = digits + ((size_t)r * beta + j) * Wl * N;
    const u32 nt = Wl - nd;                                          // targets: all rows outside the digit
    for (u32 u0 = tpart * UP_TG; u0 < nt; u0 += tsplit * UP_TG) {
#pragma unroll 1
        for (u32 e = 0; e < 2; ++e) {
            double yd[8], yp[8][2];
#pragma unroll
            for (u32 a = 0; a < 8; ++a) {
                const u64 v = e ? yraw[1][a] : yraw[0][a];
                yp[a][0] = __longlong_as_double((long long)(0x4330000000000000ull | (v & 0x1FFFFFFu))) - 4503599627370496.0;
                yp[a][1] = __longlong_as_double((long long)(0x4330000000000000ull | (v >> 25))) - 4503599627370496.0;
                yd[a] = fma(yp[a][1], 33554432.0, yp[a][0]);         // exact: y < 2^50
            }
            for (u32 tt = 0; tt < UP_TG && u0 + tt < nt; ++tt) {
                const u32 uu = u0 + tt, t = uu < lo ? uu : uu + nd;  // row of the extended basis
                u64 res;
                if (t < level) {
                    // target among the ciphertext primes: every product split exactly into h + l, brought below
                    // 0.9 q before it is added, the partial sum reduced every four terms
                    const double q = modf[t].q, u = modf[t].u;
                    const double *fd = up_ft + ((size_t)j * Wl + t) * 8;   // zero beyond the digit's limbs, as y is
                    double acc = 0.0;
#pragma unroll
                    for (u32 a = 0; a < 8; ++a) {
                        const double h = yd[a] * fd[a], l = fma(yd[a], fd[a], -h);
                        acc += fma(-rint(h * u), q, h) + l;
                        if ((a & 3) == 3) acc = fma(-rint(acc * u), q, acc);
                    }
                    acc = fma(-rint(acc * u), q, acc);               // |acc| <= q/2: what the forward round takes
                    res = (u64)__double_as_longlong(acc);
                } else {
                    // target among the special primes: sum_a y_a F_a with F_a 2^64 2^(25b) mod p in 20-bit parts
                    const u32 k = t - level;
                    const double *g = up_mats + ((size_t)j * K + k) * 48;   // zero beyond the digit's limbs
                    double s0 = 0.0, s1 = 0.0, s2 = 0.0;
#pragma unroll
                    for (u32 a = 0; a < 8; ++a) {
#pragma unroll
                        for (u32 b = 0; b < 2; ++b) {
                            s0 = fma(yp[a][b], g[(a * 2 + b) * 3 + 0], s0);
                            s1 = fma(yp[a][b], g[(a * 2 + b) * 3 + 1], s1);
                            s2 = fma(yp[a][b], g[(a * 2 + b) * 3 + 2], s2);
                        }
                    }
                    // each sum is an exact integer below 2^49; s0 + s1 2^20 + s2 2^40 < 2^90 as a 128-bit number
                    const u64 i0 = (u64)__double_as_longlong(s0 + 4503599627370496.0) & 0x000fffffffffffffull;
                    const u64 i1 = (u64)__double_as_longlong(s1 + 4503599627370496.0) & 0x000fffffffffffffull;
                    const u64 i2 = (u64)__double_as_longlong(s2 + 4503599627370496.0) & 0x000fffffffffffffull;
                    u128 acc;
                    acc.lo = i0;
                    acc.hi = 0;
                    acc_add(acc, u128{i1 << 20, i1 >> 44});
                    acc_add(acc, u128{i2 << 40, i2 >> 24});
                    res = redc_wide(acc, mods[L + k]);               // canonical: the factors carry 2^64
                }
                wlds[(tt * 16 + 2 * grp + e) * UP_COLS + col] = res;
            }
        }
        __syncthreads();
        if (u0 + grp < nt) {
            const u32 uu = u0 + grp, t = uu < lo ? uu : uu + nd;
            const u32 gl = t < level ? t : L + (t - level);
            u64 *dst = dig + (size_t)t * N;
            const ModFp mf = modf[gl];
            if (t < level) {
                const FieldFp ff = make_field_fp(mf, twf_fwd, gl, logN);
                double v[16];
#pragma unroll
                for (u32 jj = 0; jj < 16; ++jj)
                    v[jj] = __longlong_as_double((long long)wlds[(grp * 16 + jj) * UP_COLS + col]);
                radix16_fwd(ff, v, 0, 0);
#pragma unroll
                for (u32 jj = 0; jj < 16; ++jj) dst[jj * 4096 + c0] = ff.out(v[jj]);
            } else {
                auto load = [&](u32 idx) { return wlds[(grp * 16 + (idx >> 12)) * UP_COLS + col]; };
                auto store = [&](u32 idx, u64 v) { dst[idx] = v; };
                if (mf.ok)
                    pass_a16_body<false>(make_field_fp(mf, twf_fwd, gl, logN), c0, load, store);
                else
                    pass_a16_body<false>(make_field_int(mods, tws_fwd, ninvs, gl, logN), c0, load, store);
            }
        }
        __syncthreads();
    }
}

constexpr u32 MAX_BETA = 4;    // digits the fused kernels unroll (larger dnum uses the plain kernels)
constexpr u32 EPI = 4;         // residues whose loads are issued together in the fused kernels
constexpr u32 KEY_GROUP = 4;   // key switches that share one key are served by one thread

struct ItemPack {
    SwitchItem it[ROT_BATCH];
    uint8_t grp_first[ROT_BATCH], grp_count[ROT_BATCH];   // runs of items with the same key
};

// u[r][comp][t][k] = sum_j digits_r[j][t][sigma_g(k)] * key[j][comp][limb(t)][k] for the items r of one
// group (same key, same Galois element): each key residue is loaded once and used for all of them.
// grid: x = coefficients, y = limb t, z = group.
// accumulate: add to what u holds (merged giant step: sums over the giant index stay in the extended basis).
// fold_c0: also add sigma_g(c0) of each item into component 0 of its dst (the part of a rotation that needs
// no key), so that nothing but ModDown(u) is left to add later.
__global__ __launch_bounds__(KS_THREADS) void inner_product_kernel(ItemPack pack, u64 *__restrict__ u,
                                                                   const ModConst *__restrict__ mods, u32 level,
                                                                   u32 K, u32 L, u32 beta, u32 alpha, u32 logN) {
    const u32 N = 1u << logN;
    const u32 k = blockIdx.x * KS_THREADS + threadIdx.x;
    const u32 t = blockIdx.y;
    const u32 first = pack.grp_first[blockIdx.z], cnt = pack.grp_count[blockIdx.z];
    const u32 Wl = level + K, Wt = L + K;
    const u32 gl = t < level ? t : L + (t - level);
    const u64 *key = pack.it[first].key;
    const u32 kp = galois_index(k, pack.it[first].galois_elt, logN);
    u128 a0[KEY_GROUP], a1[KEY_GROUP];
#pragma unroll
    for (u32 r = 0; r < KEY_GROUP; ++r) {
        a0[r] = {0, 0};
        a1[r] = {0, 0};
    }
    for (u32 j = 0; j < beta; ++j) {
        const u64 k0 = key[(((size_t)j * 2 + 0) * Wt + gl) * N + k];
        const u64 k1 = key[(((size_t)j * 2 + 1) * Wt + gl) * N + k];
#pragma unroll
        for (u32 r = 0; r < KEY_GROUP; ++r) {
            if (r < cnt) {
                const SwitchItem &it = pack.it[first + r];
                const u64 d = (t < level && t / alpha == j) ? it.c1[(size_t)t * N + kp]
                                                            : it.digits[((size_t)j * Wl + t) * N + kp];
                mac(a0[r], d, k0);
                mac(a1[r], d, k1);
            }
        }
    }
    const ModConst m = mods[gl];
#pragma unroll
    for (u32 r = 0; r < KEY_GROUP; ++r) {
        if (r < cnt) {
            u64 *u0 = u + (((size_t)(first + r) * 2 + 0) * Wl + t) * N + k;
            u64 *u1 = u + (((size_t)(first + r) * 2 + 1) * Wl + t) * N + k;
            *u0 = redc_wide(a0[r], m);
            *u1 = redc_wide(a1[r], m);
        }
    }
}

// Inner products of several rotations summed in the extended basis (the merged giant step): a thread owns one
// coefficient of one limb for MR ciphertexts, so that a key residue, read once, serves MR multiply-accumulates.
// The 128-bit sums are folded before more than 16 products (each below 2^124) have been added.
constexpr u32 MR = 3;
__global__ __launch_bounds__(KS_THREADS) void merged_ip_kernel(MergedRot rots, const u64 *__restrict__ digits,
                                                               size_t dig_w, const u64 *__restrict__ c0_base,
                                                               size_t c0_stride_r, u64 *__restrict__ dst_base,
                                                               size_t dst_stride, u64 *__restrict__ u,
                                                               const ModConst *__restrict__ mods, u32 n, u32 level,
                                                               u32 K, u32 L, u32 beta, u32 alpha, u32 logN,
                                                               u32 accumulate, u32 groups) {
    const u32 N = 1u << logN;
    // grid x = ((chunk of 8 coefficient runs) * groups + group of MR ciphertexts) * 8 + run within the chunk: the
    // groups of ciphertexts, which read the same key rows, follow each other at a distance of 8 workgroups, i.e. on
    // the same XCD at about the same time, so one of them fetches a key line and the others find it in that L2
    const u32 chunk = N / KS_THREADS < 8 ? N / KS_THREADS : 8;   // a power of two
    const u32 xg = blockIdx.x / chunk;
    const u32 k = ((xg / groups) * chunk + (blockIdx.x & (chunk - 1))) * KS_THREADS + threadIdx.x;
    const u32 t = blockIdx.y;
    const u32 r0 = (xg % groups) * MR;
    const u32 Wl = level + K, Wt = L + K;
    const u32 gl = t < level ? t : L + (t - level);
    const u32 own = t < level ? t / alpha : ~0u;                 // the digit whose own limb t is: read from c1
    const ModConst m = mods[gl];
    u128 a0[MR], a1[MR];
    u64 s0[MR], s1[MR], cs[MR];
#pragma unroll
    for (u32 r = 0; r < MR; ++r) {
        a0[r] = {0, 0};
        a1[r] = {0, 0};
        s0[r] = s1[r] = cs[r] = 0;
    }
    u32 terms = 0;
    for (u32 i = 0; i < rots.n_rot; ++i) {
        const u32 kp = galois_index(k, rots.galois_elt[i], logN);
        const u64 *key = rots.key[i];
        // the loads of up to MAX_BETA digits are issued before their products
        for (u32 j0 = 0; j0 < beta; j0 += MAX_BETA) {
            u64 k0[MAX_BETA], k1[MAX_BETA], d[MAX_BETA][MR];
#pragma unroll
            for (u32 jj = 0; jj < MAX_BETA; ++jj) {
                const u32 j = j0 + jj;
                if (j < beta) {
                    k0[jj] = key[(((size_t)j * 2 + 0) * Wt + gl) * N + k];
                    k1[jj] = key[(((size_t)j * 2 + 1) * Wt + gl) * N + k];
#pragma unroll
                    for (u32 r = 0; r < MR; ++r)
                        if (r0 + r < n)
                            d[jj][r] = own == j
                                           ? c0_base[(size_t)(r0 + r) * c0_stride_r + rots.c0_off[i] +
                                                     ((size_t)level + t) * N + kp]
                                           : digits[((size_t)i * n + r0 + r) * dig_w + ((size_t)j * Wl + t) * N + kp];
                }
            }
#pragma unroll
            for (u32 jj = 0; jj < MAX_BETA; ++jj)
                if (j0 + jj < beta) {
#pragma unroll
                    for (u32 r = 0; r < MR; ++r)
                        if (r0 + r < n) {
                            mac(a0[r], d[jj][r], k0[jj]);
                            mac(a1[r], d[jj][r], k1[jj]);
                        }
                }
        }
        if (t < level) {
#pragma unroll
            for (u32 r = 0; r < MR; ++r)
                if (r0 + r < n)
                    cs[r] = add_mod(cs[r], c0_base[(size_t)(r0 + r) * c0_stride_r + rots.c0_off[i] + (size_t)t * N + kp],
                                    m.q);
        }
        terms += beta;
        if (terms + beta > 16 || i + 1 == rots.n_rot) {
#pragma unroll
            for (u32 r = 0; r < MR; ++r) {
                s0[r] = add_mod(s0[r], redc_wide(a0[r], m), m.q);
                s1[r] = add_mod(s1[r], redc_wide(a1[r], m), m.q);
                a0[r] = {0, 0};
                a1[r] = {0, 0};
            }
            terms = 0;
        }
    }
#pragma unroll
    for (u32 r = 0; r < MR; ++r) {
        if (r0 + r < n) {
            u64 *u0 = u + (((size_t)(r0 + r) * 2 + 0) * Wl + t) * N + k;
            u64 *u1 = u + (((size_t)(r0 + r) * 2 + 1) * Wl + t) * N + k;
            u64 v0 = s0[r], v1 = s1[r];
            if (accumulate) {
                v0 = add_mod(v0, *u0, m.q);
                v1 = add_mod(v1, *u1, m.q);
            }
            *u0 = v0;
            *u1 = v1;
            if (t < level) {
                u64 *d = dst_base + (size_t)(r0 + r) * dst_stride + (size_t)t * N + k;
                *d = add_mod(*d, cs[r], m.q);
            }
        }
    }
}

// y holds, per (item, component), the K special-limb rows y_k = INTT(u_{p_k}) * (P/p_k)^-1 in the coefficient
// domain (the scaling comes out of the inverse transform); row (pc, k) starts at y + (pc*ystride + yoff + k)*N.
// w_i = sum_k y_k * (P/p_k mod q_i) mod q_i for a chunk of target limbs i.
template <u32 KMAX, bool FP>
__global__ __launch_bounds__(KS_THREADS) void moddown_conv_kernel(const u64 *__restrict__ y, u64 *__restrict__ w,
                                                                  const ModConst *__restrict__ mods,
                                                                  const ModFp *__restrict__ modf,
                                                                  const u64 *__restrict__ dn_mat,
                                                                  const double *__restrict__ dn_matf, u32 level,
                                                                  u32 K, u32 L, u32 N, u32 ystride, u32 yoff) {
    const u32 n = blockIdx.x * KS_THREADS + threadIdx.x;
    const u32 pc = blockIdx.y;   // (item, component)
    u64 yk[KMAX];
#pragma unroll
    for (u32 k = 0; k < KMAX; ++k) {
        yk[k] = 0;
        if (k < K) yk[k] = y[((size_t)pc * ystride + yoff + k) * N + n];
    }
    const u32 i0 = blockIdx.z * DN_CHUNK, i1 = min(i0 + DN_CHUNK, level);
    if (FP) {
        // Every target below 2^50 and every special prime below 2^60 (the launcher checks): each y_k is cut into
        // three 20-bit pieces and each factor (times 2^0, 2^20, 2^40, reduced) into two 25-bit halves, all held
        // as doubles.  The 45-bit products are summed exactly by FMAs into a low and a high sum (3*KMAX terms
        // each, below 2^53), and the result is (high * 2^25 + low) mod q: the 32-bit integer multiplier, four
        // times slower per product, stays out of it.
        double yp[KMAX][3];
#pragma unroll
        for (u32 k = 0; k < KMAX; ++k) {
            const u64 v = yk[k];
            yp[k][0] = __longlong_as_double((long long)(0x4330000000000000ull | (v & 0xFFFFFu))) - 4503599627370496.0;
            yp[k][1] =
                __longlong_as_double((long long)(0x4330000000000000ull | ((v >> 20) & 0xFFFFFu))) - 4503599627370496.0;
            yp[k][2] = __longlong_as_double((long long)(0x4330000000000000ull | (v >> 40))) - 4503599627370496.0;
        }
        for (u32 i = i0; i < i1; ++i) {
            const double q = modf[i].q, u = modf[i].u;
            const double *f = dn_matf + (size_t)i * K * 6;
            double lo = 0.0, hi = 0.0;
#pragma unroll
            for (u32 k = 0; k < KMAX; ++k)
                if (k < K) {
#pragma unroll
                    for (u32 a = 0; a < 3; ++a) {
                        lo = fma(yp[k][a], f[(k * 3 + a) * 2 + 0], lo);
                        hi = fma(yp[k][a], f[(k * 3 + a) * 2 + 1], hi);
                    }
                }
            const double t = hi * 33554432.0;                       // exact: a power of two
            double v = fma(-rint(t * u), q, t) + lo;                // |.| < 0.75 q, plus low < 2^51
            v = fma(-rint(v * u), q, v);
            if (v < 0) v += q;
            w[((size_t)pc * level + i) * N + n] = (u64)v;
        }
    } else {
        for (u32 i = i0; i < i1; ++i) {
            u128 acc = {0, 0};
#pragma unroll
            for (u32 k = 0; k < KMAX; ++k)
                if (k < K) mac(acc, yk[k], dn_mat[(size_t)k * L + i]);
            w[((size_t)pc * level + i) * N + n] = redc_wide(acc, mods[i]);   // up to 16 products below 2^62 * q each
        }
    }
}

// ModDown between the two tile passes at N = 2^16, one kernel instead of three.  The last 4 stages of the inverse
// transform of the special limbs, the base conversion P -> q_i and the first 4 stages of the forward transform of the
// correction w all work on columns (residues 4096 apart), so a workgroup that owns MID_COLS columns can do all
// three without leaving the CU:
//   1. thread (k, col): column col of special limb k, 16 rows in registers, last inverse round (which folds in
//      N^-1 (P/p_k)^-1) -> y_k in LDS;
//   2. thread (row pair, col): its two coefficients' y_k cut into 20-bit pieces once, then for each group of
//      MID_TG target limbs the exact fp64 sums of moddown_conv_kernel -> w in LDS;
//   3. thread (target, col): 16 rows of w_i from LDS, first forward round, out.
// y: rows (pc*ystride + yoff + k) hold the special limbs after the inverse tile pass; w [pc][level][N] receives the
// correction ready for the forward tile pass.  Needs K <= 8, every target below 2^50 and every special prime below
// 2^60 (the launcher checks).  grid: x = column tile, y = pc.
constexpr u32 MID_COLS = 32, MID_TG = 8, MID_MAX_LEVEL = 32;
// K8: exactly 8 special primes: no per-prime checks in the conversion loop, so a target's 48 factors arrive through the
// scalar cache in one burst (with the checks the wave waited for each prime's six in turn).  Staging the factors in
// LDS instead was measured slower: broadcast reads still take an LDS issue slot per pair of multiply-adds.
// w_i = sum_k y_k (P/p_k mod q_i) for the two coefficients of a thread, as doubles with |w| <= q/2: the exact fp64 sums
// of moddown_conv_kernel (20-bit pieces of y times 25-bit halves of the factors)
template <bool K8>
__device__ __forceinline__ double mid_convert(const double (&yp)[8][3], const double *__restrict__ f, u32 K, double q,
                                              double u) {
    double lo = 0.0, hi = 0.0;
#pragma unroll
    for (u32 k = 0; k < 8; ++k)
        if (K8 || k < K) {
#pragma unroll
            for (u32 a = 0; a < 3; ++a) {
                lo = fma(yp[k][a], f[(k * 3 + a) * 2 + 0], lo);
                hi = fma(yp[k][a], f[(k * 3 + a) * 2 + 1], hi);
            }
        }
    const double tt = hi * 33554432.0;                              // exact: a power of two
    const double x = fma(-rint(tt * u), q, tt) + lo;                // |.| < 0.75 q, plus low < 2^51
    return fma(-rint(x * u), q, x);                                 // |v| <= q/2
}

// the 20-bit pieces of the K special-limb values of one coefficient, as doubles
__device__ __forceinline__ void mid_pieces(const u64 (&yraw)[8], double (&yp)[8][3]) {
#pragma unroll
    for (u32 k = 0; k < 8; ++k) {
        const u64 v = yraw[k];
        yp[k][0] = __longlong_as_double((long long)(0x4330000000000000ull | (v & 0xFFFFFu))) - 4503599627370496.0;
        yp[k][1] = __longlong_as_double((long long)(0x4330000000000000ull | ((v >> 20) & 0xFFFFFu))) - 4503599627370496.0;
        yp[k][2] = __longlong_as_double((long long)(0x4330000000000000ull | (v >> 40))) - 4503599627370496.0;
    }
}

// RESC: ModDown and rescale in one (the merged giant step's last act).  The rescale needs the dropped limb of the
// brought-down ciphertext in the coefficient domain, r = INTT(z + u P^-1)[l-1] - w_{l-1} P^-1, with z the part of the
// ciphertext that needs no ModDown; t_rows holds INTT(z + u P^-1)[l-1] and w_{l-1} is computed here first.  With
// r' = r + floor(q_{l-1}/2) mod q_{l-1}, the correction of limb i < l-1 becomes w_i P^-1 + (r' mod q_i - floor(q_{l-1}/2)
// mod q_i): one forward transform per limb serves both the ModDown and the rescale, and the rows written are those of
// the l-1 remaining limbs.  Exact modular arithmetic throughout: the same residues as ModDown followed by rescale.
template <bool K8, bool RESC>
__global__ __launch_bounds__(256) void moddown_mid_kernel(const u64 *__restrict__ y, u64 *__restrict__ w,
                                                          const ModConst *__restrict__ mods,
                                                          const ModFp *__restrict__ modf,
                                                          const ModFp *__restrict__ modf_dn,
                                                          const u64 *__restrict__ tw_inv,
                                                          const double *__restrict__ twf_inv,
                                                          const u64 *__restrict__ ninv_dn,
                                                          const double *__restrict__ twf_fwd,
                                                          const double *__restrict__ dn_matf, u32 level, u32 K, u32 L,
                                                          u32 ystride, u32 yoff, const u64 *__restrict__ t_rows,
                                                          const double *__restrict__ pinvf) {
    constexpr u32 logN = 16, N = 1u << logN;
    static_assert(MID_TG == 8, "the correction tiles reuse the 8 rows of special-limb tiles");
    __shared__ u64 ylds[8 * 16 * MID_COLS];
    u64 *wlds = ylds;               // y lives in registers once step 2 has read it: the same 32 KiB
    const u32 tid = threadIdx.x, col = tid & (MID_COLS - 1), grp = tid / MID_COLS;   // grp < 8
    const u32 c0 = blockIdx.x * MID_COLS + col;
    const u32 pc = blockIdx.y;
    if (grp < K) {
        const u32 gl = L + grp;
        const u64 *src = y + ((size_t)pc * ystride + yoff + grp) * N;
        auto load = [&](u32 idx) { return src[idx]; };
        auto store = [&](u32 idx, u64 v) { ylds[(grp * 16 + (idx >> 12)) * MID_COLS + col] = v; };
        const ModFp mf = modf_dn[gl];
        if (mf.ok)
            pass_a16_body<true>(make_field_fp(mf, twf_inv, gl, logN), c0, load, store);
        else
            pass_a16_body<true>(make_field_int(mods, tw_inv, ninv_dn, gl, logN), c0, load, store);
    }
    __syncthreads();
    // the two coefficients of this thread (rows 2*grp, 2*grp + 1 of this column) leave LDS as they are
    u64 yraw[2][8];
#pragma unroll
    for (u32 e = 0; e < 2; ++e)
#pragma unroll
        for (u32 k = 0; k < 8; ++k) yraw[e][k] = (K8 || k < K) ? ylds[(k * 16 + 2 * grp + e) * MID_COLS + col] : 0;
    __syncthreads();                // every thread has its y: the tile may be overwritten
    // rescale: the dropped limb first
    double rp[2] = {0.0, 0.0}, hq = 0.0;
    const u32 n_out = RESC ? level - 1 : level;
    if (RESC) {
        const u32 il = level - 1;
        const ModFp ml = modf[il];
        FieldFp fl;
        fl.q = ml.q;
        fl.u = ml.u;
        fl.n0 = fl.n1 = 0.0;
        fl.tw = nullptr;
        hq = (double)(mods[il].q >> 1);
#pragma unroll
        for (u32 e = 0; e < 2; ++e) {
            double yp[8][3];
            mid_pieces(yraw[e], yp);
            const double wl = mid_convert<K8>(yp, dn_matf + (size_t)il * K * 6, K, ml.q, ml.u);
            const double t = fl.in(t_rows[(size_t)pc * N + (2 * grp + e) * 4096 + c0]);
            double r = t - fl.mul(wl, pinvf[il]);
            fl.norm(r);
            if (r < 0) r += ml.q;                                   // r in [0, q_last)
            r += hq;
            rp[e] = r >= ml.q ? r - ml.q : r;                       // r' = (r + h) mod q_last
        }
    }
    for (u32 i0 = 0; i0 < n_out; i0 += MID_TG) {
        // one coefficient at a time: its 24 pieces are rebuilt per group of targets (24 doubles live instead of 48,
        // which is what lets four waves share a SIMD)
#pragma unroll 1
        for (u32 e = 0; e < 2; ++e) {
            double yp[8][3];
            mid_pieces(e ? yraw[1] : yraw[0], yp);
            const double rpe = e ? rp[1] : rp[0];
            for (u32 t = 0; t < MID_TG && i0 + t < n_out; ++t) {
                const u32 i = i0 + t;
                const double q = modf[i].q, u = modf[i].u;
                double v = mid_convert<K8>(yp, dn_matf + (size_t)i * K * 6, K, q, u);
                if (RESC) {
                    FieldFp fi;
                    fi.q = q;
                    fi.u = u;
                    fi.n0 = fi.n1 = 0.0;
                    fi.tw = nullptr;
                    double hi_ = hq, ri = rpe;
                    fi.norm(hi_);                                   // floor(q_last / 2) mod q_i
                    fi.norm(ri);                                    // r' mod q_i
                    v = fi.mul(v, pinvf[i]) + (ri - hi_);           // |.| < 2q: the forward round normalises
                }
                wlds[(t * 16 + 2 * grp + e) * MID_COLS + col] = (u64)__double_as_longlong(v);
            }
        }
        __syncthreads();
        if (i0 + grp < n_out) {
            const u32 i = i0 + grp;
            const FieldFp ff = make_field_fp(modf[i], twf_fwd, i, logN);
            u64 *dst = w + ((size_t)pc * level + i) * N;
            double v[16];
#pragma unroll
            for (u32 j = 0; j < 16; ++j) v[j] = __longlong_as_double((long long)wlds[(grp * 16 + j) * MID_COLS + col]);
            radix16_fwd(ff, v, 0, 0);
#pragma unroll
            for (u32 j = 0; j < 16; ++j) dst[j * 4096 + c0] = ff.out(v[j]);
        }
        __syncthreads();
    }
}

// t[pc][k] = z[pc][l-1][k] + u[pc][l-1][k] P^-1 mod q_{l-1} (NTT domain): the dropped limb of the ciphertext before its
// special-limb correction.  z_r: component-major ciphertexts [2][level][N]; u [n][2][level+K][N].
__global__ __launch_bounds__(KS_THREADS) void rescale_last_row_kernel(PtrPack z, const u64 *__restrict__ u,
                                                                      u64 *__restrict__ t,
                                                                      const ModConst *__restrict__ mods,
                                                                      const u64 *__restrict__ pinv, u32 level, u32 K,
                                                                      u32 N) {
    const u32 k = blockIdx.x * KS_THREADS + threadIdx.x;
    const u32 pc = blockIdx.y, r = pc >> 1, comp = pc & 1, i = level - 1;
    const ModConst m = mods[i];
    const u64 zz = z.p[r][((size_t)comp * level + i) * N + k];
    const u64 uu = u[((size_t)pc * (level + K) + i) * N + k];
    t[(size_t)pc * N + k] = add_mod(zz, mont_mul(uu, pinv[i], m), m.q);
}

// out[r][comp][i][k] = (z[r][comp][i][k] + u P^-1 - NTT(w')[i][k]) q_{l-1}^-1 for the l-1 remaining limbs
__global__ __launch_bounds__(KS_THREADS) void moddown_rescale_final_kernel(PtrPack z, ItemPack out,
                                                                           const u64 *__restrict__ u,
                                                                           const u64 *__restrict__ w,
                                                                           const ModConst *__restrict__ mods,
                                                                           const u64 *__restrict__ pinv,
                                                                           const u64 *__restrict__ qlinv, u32 level,
                                                                           u32 K, u32 N) {
    typedef u64 vec_t __attribute__((ext_vector_type(2)));
    const u32 k = (blockIdx.x * KS_THREADS + threadIdx.x) * 2;
    const u32 i = blockIdx.y, pc = blockIdx.z, r = pc >> 1, comp = pc & 1;
    const ModConst m = mods[i];
    const vec_t zz = *reinterpret_cast<const vec_t *>(z.p[r] + ((size_t)comp * level + i) * N + k);
    const vec_t uu = *reinterpret_cast<const vec_t *>(u + ((size_t)pc * (level + K) + i) * N + k);
    const vec_t ww = *reinterpret_cast<const vec_t *>(w + ((size_t)pc * level + i) * N + k);
    vec_t o;
#pragma unroll
    for (u32 e = 0; e < 2; ++e) {
        const u64 y = add_mod(zz[e], mont_mul(uu[e], pinv[i], m), m.q);
        o[e] = mont_mul(sub_mod(y, ww[e], m.q), qlinv[i], m);
    }
    *reinterpret_cast<vec_t *>(out.it[r].dst + ((size_t)comp * (level - 1) + i) * N + k) = o;
}

// Whether the fused kernel applies to this parameter set at this level.
static bool moddown_mid_ok(const ckks_params *p, u32 level) {
    bool ok = p->logN == 16 && p->dn_fp && p->K <= 8 && level <= MID_MAX_LEVEL;
    for (u32 i = 0; i < level; ++i) ok = ok && (p->mod[i] >> 50) == 0;
    return ok;
}

static void launch_moddown_mid(const ckks_params *p, const u64 *y, u64 *w, u32 n, u32 level, u32 ystride, u32 yoff,
                               hipStream_t stream, const u64 *t_rows = nullptr) {
#define MID_LAUNCH(K8, RESC)                                                                                         \
    hipLaunchKernelGGL((moddown_mid_kernel<K8, RESC>), dim3(4096 / MID_COLS, n * 2), dim3(256), 0, stream, y, w,       \
                       p->d_mod, p->d_modf, p->d_modf_dn, p->d_tws_inv, p->d_twf_inv, p->d_ninvs_dn, p->d_twf_fwd,    \
                       p->d_dn_matf, level, p->K, p->L, ystride, yoff, t_rows, p->d_pinvf)
    if (p->K == 8) {
        if (t_rows) MID_LAUNCH(true, true); else MID_LAUNCH(true, false);
    } else {
        if (t_rows) MID_LAUNCH(false, true); else MID_LAUNCH(false, false);
    }
#undef MID_LAUNCH
}

// base conversion P -> q_i of n*2 polynomials; the rows of polynomial pc start at row pc * ystride + yoff of y
static void launch_moddown_conv(const ckks_params *p, const u64 *y, u64 *w, u32 n, u32 level, u32 ystride, u32 yoff,
                                hipStream_t stream) {
    const dim3 grid(p->N / KS_THREADS, n * 2, (level + DN_CHUNK - 1) / DN_CHUNK);
    bool fp = p->dn_fp;        // fp64 sums need every target below 2^50 and every special prime below 2^60
    for (u32 i = 0; i < level; ++i) fp = fp && (p->mod[i] >> 50) == 0;
#define CONV_LAUNCH(KM, FPK)                                                                                      \
    hipLaunchKernelGGL((moddown_conv_kernel<KM, FPK>), grid, dim3(KS_THREADS), 0, stream, y, w, p->d_mod, p->d_modf, \
                       p->d_dn_mat, p->d_dn_matf, level, p->K, p->L, p->N, ystride, yoff)
    if (p->K <= 8) {
        if (fp) CONV_LAUNCH(8, true); else CONV_LAUNCH(8, false);
    } else {
        if (fp) CONV_LAUNCH(MAX_DIGIT, true); else CONV_LAUNCH(MAX_DIGIT, false);
    }
#undef CONV_LAUNCH
}

// dst[comp][i][k] (+)= (u_{q_i} - NTT(w_i)) * P^-1  (+ sigma_g(c0)[i][k] for comp 0)
__global__ __launch_bounds__(KS_THREADS) void moddown_final_kernel(ItemPack pack, const u64 *__restrict__ u,
                                                                   const u64 *__restrict__ w,
                                                                   const ModConst *__restrict__ mods,
                                                                   const u64 *__restrict__ pinv, u32 level, u32 K,
                                                                   u32 logN) {
    const u32 N = 1u << logN;
    const u32 k = blockIdx.x * KS_THREADS + threadIdx.x;
    const u32 i = blockIdx.y, r = blockIdx.z >> 1, comp = blockIdx.z & 1;
    const u32 Wl = level + K;
    const SwitchItem &it = pack.it[r];
    const ModConst m = mods[i];
    const u64 uq = u[(((size_t)r * 2 + comp) * Wl + i) * N + k];
    const u64 wq = w[(((size_t)r * 2 + comp) * level + i) * N + k];
    u64 v = mont_mul(sub_mod(uq, wq, m.q), pinv[i], m);
    if (comp == 0 && it.c0) v = add_mod(v, it.c0[(size_t)i * N + galois_index(k, it.galois_elt, logN)], m.q);
    u64 *dst = it.dst + ((size_t)comp * level + i) * N + k;
    if (it.accumulate) v = add_mod(v, *dst, m.q);
    *dst = v;
}

// ---- fused kernels for N = 2^12 / 2^16 -------------------------------------------------------------
// Key inner product on the special limbs feeding straight into the first pass of their inverse transform:
// row (comp, k, r) of y = INTT-pass-B( sum_j sigma_g(d_j)[p_k] * key_j[comp][p_k] ).
// grid: x = tile of 4096, y = ((k*n + r)*2 + comp): the two components of an item (same digit reads) and the
// items of a batch that share a key sit next to each other and, with 16 tiles per row, on the same XCD.
// KEY_NT: key rows are read with non-temporal loads.  Right when every item has a key of its own (the rows are used
// once and would only push the digit rows, which every item re-reads, out of L2); wrong when neighbouring items share
// a key, where it is the cached line that lets the second and third reader skip HBM.
typedef u64 key_vec_t __attribute__((ext_vector_type(2)));
template <bool NT>
__device__ __forceinline__ key_vec_t load_key(const key_vec_t *p) {
    return NT ? __builtin_nontemporal_load(p) : *p;
}

template <bool KEY_NT>
__global__ __launch_bounds__(NTT_THREADS) void ip_intt_kernel(ItemPack pack, u64 *__restrict__ y,
                                                              const ModConst *__restrict__ mods,
                                                              const ModFp *__restrict__ modf,
                                                              const u64 *__restrict__ tw_inv,
                                                              const double *__restrict__ twf_inv,
                                                              const u64 *__restrict__ ninv, u32 n, u32 level, u32 K,
                                                              u32 L, u32 beta, u32 logN) {
    __shared__ u64 lds[FAST_LDS_WORDS];
    const u32 N = 1u << logN;
    const u32 comp = blockIdx.y & 1, r = (blockIdx.y >> 1) % n, k = (blockIdx.y >> 1) / n;
    const u32 gl = L + k, t = level + k, Wl = level + K, Wt = L + K;
    const SwitchItem &it = pack.it[r];
    const ModConst m = mods[gl];
    const u64 *dig = it.digits + (size_t)t * N;
    const u64 *key = it.key + ((size_t)comp * Wt + gl) * N;
    const u64 g = it.galois_elt;
    u64 *out = y + (((size_t)r * 2 + comp) * K + k) * N;
    auto store = [&](u32 idx, u64 v) { out[idx] = v; };
    // inner product into LDS on pairs of adjacent residues (16-byte key loads), two pairs at a time so that
    // their loads are in flight together
    typedef u64 vec_t __attribute__((ext_vector_type(2)));
    const u32 tid = threadIdx.x, base = blockIdx.x << 12;
    constexpr u32 EPP = EPI / 2;
    for (u32 i0 = 0; i0 < 8; i0 += EPP) {
        u64 dv[EPP][2][MAX_BETA];
        vec_t kv[EPP][MAX_BETA];
#pragma unroll
        for (u32 e = 0; e < EPP; ++e) {
            const u32 idx = base + 2 * (tid + 256 * (i0 + e));
            const u32 kp0 = galois_index(idx, g, logN), kp1 = galois_index(idx + 1, g, logN);
#pragma unroll
            for (u32 j = 0; j < MAX_BETA; ++j)
                if (j < beta) {
                    dv[e][0][j] = dig[(size_t)j * Wl * N + kp0];
                    dv[e][1][j] = dig[(size_t)j * Wl * N + kp1];
                    kv[e][j] = load_key<KEY_NT>(reinterpret_cast<const vec_t *>(key + (size_t)j * 2 * Wt * N + idx));
                }
        }
#pragma unroll
        for (u32 e = 0; e < EPP; ++e) {
            const u32 loc = 2 * (tid + 256 * (i0 + e));
#pragma unroll
            for (u32 z = 0; z < 2; ++z) {
                u128 acc = {0, 0};
#pragma unroll
                for (u32 j = 0; j < MAX_BETA; ++j)
                    if (j < beta) mac(acc, dv[e][z][j], kv[e][j][z]);
                lds[lds_pad(loc + z)] = redc_wide(acc, m);
            }
        }
    }
    __syncthreads();
    const ModFp mf = modf[gl];
    if (mf.ok)
        pass_b_inv_from_lds(make_field_fp(mf, twf_inv, gl, logN), logN, lds, store);
    else
        pass_b_inv_from_lds(make_field_int(mods, tw_inv, ninv, gl, logN), logN, lds, store);
}

// Last pass of the forward transform of w fused with the rest of the key switch on limb q_i:
//   dst[comp][i] (+)= ( sum_j sigma_g(d_j)[q_i] * key_j[comp][q_i] - NTT(w)[i] ) * P^-1  (+ sigma_g(c0)[i] if comp = 0)
// grid: x = tile of 4096, y = ((i*n + r)*2 + comp), neighbours share digit and key lines in L2 as above.
template <bool KEY_NT>
__global__ __launch_bounds__(NTT_THREADS) void passb_final_kernel(ItemPack pack, const u64 *__restrict__ w,
                                                                  const ModConst *__restrict__ mods,
                                                                  const ModFp *__restrict__ modf,
                                                                  const u64 *__restrict__ tw_fwd,
                                                                  const double *__restrict__ twf_fwd,
                                                                  const u64 *__restrict__ ninv,
                                                                  const u64 *__restrict__ pinv, u32 n, u32 level,
                                                                  u32 K, u32 L, u32 beta, u32 alpha, u32 logN) {
    __shared__ u64 lds[FAST_LDS_WORDS];
    const u32 N = 1u << logN;
    const u32 comp = blockIdx.y & 1, r = (blockIdx.y >> 1) % n, i = (blockIdx.y >> 1) / n;
    const u32 Wl = level + K, Wt = L + K;
    const SwitchItem &it = pack.it[r];
    const ModConst m = mods[i];
    const u64 *wrow = w + (((size_t)r * 2 + comp) * level + i) * N;
    // row of limb i in digit j; the digit that owns limb i is not stored: its row is the source's own
    const u64 *drow[MAX_BETA];
#pragma unroll
    for (u32 j = 0; j < MAX_BETA; ++j)
        drow[j] = j == i / alpha ? it.c1 + (size_t)i * N : it.digits + ((size_t)j * Wl + i) * N;
    const u64 *key = it.key + ((size_t)comp * Wt + i) * N;
    const u64 *c0 = it.c0 + (size_t)i * N;
    u64 *dst = it.dst + ((size_t)comp * level + i) * N;
    const u64 g = it.galois_elt, pi = pinv[i];
    const u32 accumulate = it.accumulate;
    auto load = [&](u32 idx) -> u64 { return __builtin_nontemporal_load(wrow + idx); };
    const ModFp mf = modf[i];
    if (mf.ok)   // the fp64 epilogue takes the transformed correction as doubles, |x| <= q/2
        pass_b_fwd_to_lds<true>(make_field_fp(mf, twf_fwd, i, logN), logN, lds, load);
    else
        pass_b_fwd_to_lds(make_field_int(mods, tw_fwd, ninv, i, logN), logN, lds, load);
    // epilogue on pairs of adjacent residues (16-byte accesses to the streamed operands), two pairs at a time so
    // that their loads are in flight together.  Keys, w and the output are streamed once: non-temporal, so that
    // they do not push the digit rows (re-read by every item of the batch) out of L2.
    typedef u64 vec_t __attribute__((ext_vector_type(2)));
    const u32 tid = threadIdx.x, base = blockIdx.x << 12;
    constexpr u32 EPP = EPI / 2;
    FieldFp ff;
    ff.q = mf.q;
    ff.u = mf.u;
    ff.n0 = ff.n1 = 0.0;
    ff.tw = nullptr;
    const u64 pinv_plain = mont_mul(pi, 1, m);                       // P^-1 (pi is its Montgomery form)
    const double c_w = ff.in(pinv_plain), c_sum = ff.in(mont_mul(pinv_plain, 1, m));
    for (u32 i0 = 0; i0 < 8; i0 += EPP) {
        u64 dv[EPP][2][MAX_BETA], cv[EPP][2];
        vec_t kv[EPP][MAX_BETA], ov[EPP];
#pragma unroll
        for (u32 e = 0; e < EPP; ++e) {
            const u32 idx = base + 2 * (tid + 256 * (i0 + e));
            const u32 kp0 = galois_index(idx, g, logN), kp1 = galois_index(idx + 1, g, logN);
#pragma unroll
            for (u32 j = 0; j < MAX_BETA; ++j)
                if (j < beta) {
                    dv[e][0][j] = drow[j][kp0];
                    dv[e][1][j] = drow[j][kp1];
                    kv[e][j] = load_key<KEY_NT>(reinterpret_cast<const vec_t *>(key + (size_t)j * 2 * Wt * N + idx));
                }
            const bool fold = comp == 0 && it.c0;
            cv[e][0] = fold ? c0[kp0] : 0;
            cv[e][1] = fold ? c0[kp1] : 0;
            if (accumulate)
                ov[e] = __builtin_nontemporal_load(reinterpret_cast<const vec_t *>(dst + idx));
            else
                ov[e] = vec_t{0, 0};
        }
#pragma unroll
        for (u32 e = 0; e < EPP; ++e) {
            const u32 loc = 2 * (tid + 256 * (i0 + e));
            vec_t out;
#pragma unroll
            for (u32 z = 0; z < 2; ++z) {
                if (mf.ok) {
                    // primes below 2^50: the same residues through exact fp64 products.  The keys are in
                    // Montgomery form (times 2^64), so the sum is multiplied by 2^-64 * P^-1 and w by P^-1.
                    double sum = 0.0;
#pragma unroll
                    for (u32 j = 0; j < MAX_BETA; ++j)
                        if (j < beta) sum += ff.mul(ff.in(dv[e][z][j]), ff.in(kv[e][j][z]));
                    const double t = ff.mul(sum, c_sum) - ff.mul(ff.from_bits(lds[lds_pad(loc + z)]), c_w) +
                                     (ff.in(cv[e][z]) + ff.in(ov[e][z]));
                    out[z] = ff.out(t);
                } else {
                    u128 acc = {0, 0};
#pragma unroll
                    for (u32 j = 0; j < MAX_BETA; ++j)
                        if (j < beta) mac(acc, dv[e][z][j], kv[e][j][z]);
                    u64 v = mont_mul(sub_mod(redc_wide(acc, m), lds[lds_pad(loc + z)], m.q), pi, m);
                    v = add_mod(v, cv[e][z], m.q);
                    out[z] = add_mod(v, ov[e][z], m.q);
                }
            }
            __builtin_nontemporal_store(out, reinterpret_cast<vec_t *>(dst + base + loc));
        }
    }
}

// (out0, out1, t2) = (a0*b0, a0*b1 + a1*b0, a1*b1), pointwise on limb blockIdx.y
__global__ __launch_bounds__(KS_THREADS) void tensor_kernel(const u64 *__restrict__ a, const u64 *__restrict__ b,
                                                            u64 *__restrict__ out, u64 *__restrict__ t2,
                                                            const ModConst *__restrict__ mods, u32 level, u32 N) {
    const u32 k = blockIdx.x * KS_THREADS + threadIdx.x;
    const u32 i = blockIdx.y;
    const ModConst m = mods[i];
    const size_t o0 = (size_t)i * N + k, o1 = ((size_t)level + i) * N + k;
    const u64 a0 = a[o0], a1 = a[o1];
    const u64 b0 = mont_mul(b[o0], m.r2, m), b1 = mont_mul(b[o1], m.r2, m);   // Montgomery form
    out[o0] = mont_mul(a0, b0, m);
    out[o1] = add_mod(mont_mul(a0, b1, m), mont_mul(a1, b0, m), m.q);
    t2[o0] = mont_mul(a1, b1, m);
}

size_t digits_words(const ckks_params *p, u32 level) {
    u32 beta = (level + p->alpha - 1) / p->alpha;
    return (size_t)beta * (level + p->K) * p->N;
}

size_t switch_scratch_words(const ckks_params *p, u32 level, u32 n_items) {
    return (size_t)n_items * 2 * ((size_t)(level + p->K) + level) * p->N;
}

// c1[r] [level][N] NTT domain (n <= ROT_BATCH device pointers) -> d_digits [n][beta][level+K][N] NTT domain;
// d_tmp [n][level][N] scratch.
int decompose(ckks_params *p, const u64 *const *c1, u32 n, u32 level, u64 *d_digits, u64 *d_tmp,
              hipStream_t stream) {
    if (n == 0) return CKKS_OK;
    const u32 N = p->N, K = p->K, L = p->L, Wl = level + K, alpha = p->alpha;
    const LevelTables *lt = nullptr;
    int rc = p->level_tables(level, &lt);
    if (rc) return rc;
    const u32 beta = lt->beta;
    PtrPack src;
    for (u32 r = 0; r < ROT_BATCH; ++r) src.p[r] = c1[r < n ? r : 0];
    LimbIds ids;
    for (u32 i = 0; i < level; ++i) ids.id[i] = (uint8_t)i;
    bool all_fp = true;
    for (u32 i = 0; i < level; ++i) all_fp = all_fp && (p->mod[i] >> 50) == 0;
    bool sp60 = true;
    for (u32 k = 0; k < K; ++k) sp60 = sp60 && (p->mod[L + k] >> 60) == 0;
    if (fast_ring(p)) {
        hipLaunchKernelGGL(gather_intt_kernel, dim3(N >> 12, n * level), dim3(NTT_THREADS), 0, stream, src, d_tmp,
                           p->d_mod, p->d_modf, p->d_tws_inv, p->d_twf_inv, p->d_ninvs, level, p->logN);
        CKKS_LAUNCH_CHECK("gather_intt_kernel");
        p->limb_ntts += (u64)n * level;
        if (p->logN == 16 && all_fp && sp60 && alpha <= 8 && K <= 8) {
            // the column passes of both transforms ride in the base conversion: c1 read once, digits written once
            const u32 tgroups = (Wl - std::min(alpha, level) + UP_TG - 1) / UP_TG;
            const u32 tsplit = n * beta * (4096 / UP_COLS) < 1024 ? std::max<u32>(1, tgroups) : 1;
            hipLaunchKernelGGL(modup_mid_kernel, dim3(4096 / UP_COLS * tsplit, beta, n), dim3(256), 0, stream, d_tmp,
                               d_digits, p->d_mod, p->d_modf, lt->d_modf_up, p->d_twf_inv, p->d_twf_fwd, p->d_tws_fwd,
                               p->d_ninvs, lt->d_up_ft, lt->d_up_mats, level, K, L, alpha, beta, tsplit);
            CKKS_LAUNCH_CHECK("modup_mid_kernel");
            p->limb_ntts += (u64)n * beta * Wl - (u64)n * level;
            auto row_id2 = [&](u32 j, u32 t) -> uint8_t {
                u32 lo = j * alpha, hi = std::min(lo + alpha, level);
                if (t >= lo && t < hi) return (uint8_t)SKIP_ROW;
                return (uint8_t)(t < level ? t : L + (t - level));
            };
            for (u32 j = 0; j < beta; ++j)
                for (u32 t = 0; t < Wl; ++t) ids.id[j * Wl + t] = row_id2(j, t);
            return launch_ntt(p, d_digits, ids, beta * Wl, n * beta * Wl, false, stream, 2);
        }
        rc = launch_ntt(p, d_tmp, ids, level, n * level, true, stream, 2);
    } else {
        hipLaunchKernelGGL(gather_c1_kernel, dim3(N / KS_THREADS, level, n), dim3(KS_THREADS), 0, stream, src, d_tmp,
                           level, N);
        CKKS_LAUNCH_CHECK("gather_c1_kernel");
        rc = launch_ntt(p, d_tmp, ids, level, n * level, true, stream);
    }
    if (rc) return rc;
    // two launches: the ciphertext-prime targets (fp64 arithmetic when every active prime is below 2^50) and the
    // special-prime targets (integer arithmetic); each keeps only its own form of y in registers
#define MODUP_LAUNCH(A, FPK, T0, T1)                                                                               \
    hipLaunchKernelGGL((modup_kernel<A, 2, FPK>), dim3(N / KS_THREADS / 2, beta, n), dim3(KS_THREADS), 0, stream,   \
                       d_tmp, d_digits, p->d_mod, p->d_modf, lt->d_up_inv, lt->d_up_mat, lt->d_up_matf, level, K,   \
                       L, alpha, N, beta, T0, T1)
    if (alpha <= 8) {
        if (all_fp)
            MODUP_LAUNCH(8, true, 0u, level);
        else
            MODUP_LAUNCH(8, false, 0u, level);
        MODUP_LAUNCH(8, false, level, Wl);
    } else {
        if (all_fp)
            MODUP_LAUNCH(MAX_DIGIT, true, 0u, level);
        else
            MODUP_LAUNCH(MAX_DIGIT, false, 0u, level);
        MODUP_LAUNCH(MAX_DIGIT, false, level, Wl);
    }
#undef MODUP_LAUNCH
    CKKS_LAUNCH_CHECK("modup_kernel");
    // forward NTT of the converted rows; the digit's own limbs were copied and are skipped
    auto row_id = [&](u32 j, u32 t) -> uint8_t {
        u32 lo = j * alpha, hi = std::min(lo + alpha, level);
        if (t >= lo && t < hi) return (uint8_t)SKIP_ROW;
        return (uint8_t)(t < level ? t : L + (t - level));
    };
    if (beta * Wl <= MAX_ROW_IDS) {
        for (u32 j = 0; j < beta; ++j)
            for (u32 t = 0; t < Wl; ++t) ids.id[j * Wl + t] = row_id(j, t);
        rc = launch_ntt(p, d_digits, ids, beta * Wl, n * beta * Wl, false, stream);
        if (rc) return rc;
    } else {
        for (u32 r = 0; r < n; ++r)
            for (u32 j = 0; j < beta; ++j) {
                for (u32 t = 0; t < Wl; ++t) ids.id[t] = row_id(j, t);
                rc = launch_ntt(p, d_digits + ((size_t)r * beta + j) * Wl * N, ids, Wl, Wl, false, stream);
                if (rc) return rc;
            }
    }
    return CKKS_OK;
}

static u32 build_pack(const SwitchItem *items, u32 n, ItemPack &pack) {
    for (u32 r = 0; r < ROT_BATCH; ++r) pack.it[r] = items[r < n ? r : 0];
    u32 n_groups = 0;
    for (u32 r = 0; r < n;) {
        u32 c = 1;
        while (r + c < n && c < KEY_GROUP && items[r + c].key == items[r].key &&
               items[r + c].galois_elt == items[r].galois_elt)
            ++c;
        pack.grp_first[n_groups] = (uint8_t)r;
        pack.grp_count[n_groups] = (uint8_t)c;
        ++n_groups;
        r += c;
    }
    for (u32 g = n_groups; g < ROT_BATCH; ++g) pack.grp_first[g] = pack.grp_count[g] = 0;
    return n_groups;
}

// Merged giant step, part 1: d_u[r] (+)= the key inner products of rots.n_rot rotations of ciphertext r over all
// level+K limbs (NTT domain), dst_r.c0 += the rotated c0 parts.  d_u [n][2][level+K][N].
int switch_accumulate_merged(ckks_params *p, u32 level, const MergedRot &rots, u32 n, const u64 *d_digits,
                             const u64 *c0_base, size_t c0_stride_r, u64 *dst_base, size_t dst_stride, u64 *d_u,
                             bool accumulate, hipStream_t stream) {
    if (n == 0 || rots.n_rot == 0) return CKKS_OK;
    if (n > ROT_BATCH || rots.n_rot > MERGE_GROUP) {
        set_error("switch_accumulate_merged: %u ciphertexts x %u rotations exceed one launch", n, rots.n_rot);
        return CKKS_E_INVAL;
    }
    const u32 N = p->N, K = p->K, L = p->L, Wl = level + K;
    const u32 beta = (level + p->alpha - 1) / p->alpha;
    const u32 groups = (n + MR - 1) / MR;
    hipLaunchKernelGGL(merged_ip_kernel, dim3(N / KS_THREADS * groups, Wl), dim3(KS_THREADS), 0, stream, rots,
                       d_digits, digits_words(p, level), c0_base, c0_stride_r, dst_base, dst_stride, d_u, p->d_mod, n,
                       level, K, L, beta, p->alpha, p->logN, accumulate ? 1u : 0u, groups);
    CKKS_LAUNCH_CHECK("merged_ip_kernel");
    return CKKS_OK;
}

// Merged giant step, part 2: dst_r += ModDown(d_u[r]) for n <= ROT_BATCH ciphertexts; d_u is consumed.
// d_w: n*2*level*N words of scratch.
int moddown_add(ckks_params *p, u32 level, u64 *d_u, u64 *const *dst, u32 n, u64 *d_w, hipStream_t stream) {
    if (n == 0) return CKKS_OK;
    const u32 N = p->N, K = p->K, L = p->L, Wl = level + K;
    ItemPack pack;
    for (u32 r = 0; r < ROT_BATCH; ++r) {
        SwitchItem &it = pack.it[r];
        it.digits = nullptr;
        it.c1 = nullptr;
        it.c0 = nullptr;                       // already folded in by switch_accumulate_merged
        it.key = nullptr;
        it.dst = dst[r < n ? r : 0];
        it.galois_elt = 1;
        it.accumulate = 1;
    }
    LimbIds ids;
    for (u32 t = 0; t < Wl; ++t) ids.id[t] = (uint8_t)(t < level ? SKIP_ROW : L + (t - level));
    const bool mid = moddown_mid_ok(p, level);      // the column passes of both transforms ride in the conversion
    int rc = launch_ntt(p, d_u, ids, Wl, n * 2 * Wl, true, stream, mid ? 1 : 3, true);
    if (rc) return rc;
    if (mid) {
        launch_moddown_mid(p, d_u, d_w, n, level, Wl, level, stream);
        CKKS_LAUNCH_CHECK("moddown_mid_kernel");
        p->limb_ntts += (u64)n * 2 * level;
    } else {
        launch_moddown_conv(p, d_u, d_w, n, level, Wl, level, stream);
        CKKS_LAUNCH_CHECK("moddown_conv_kernel");
    }
    for (u32 i = 0; i < level; ++i) ids.id[i] = (uint8_t)i;
    rc = launch_ntt(p, d_w, ids, level, n * 2 * level, false, stream, mid ? 2 : 3);
    if (rc) return rc;
    hipLaunchKernelGGL(moddown_final_kernel, dim3(N / KS_THREADS, level, n * 2), dim3(KS_THREADS), 0, stream, pack,
                       d_u, d_w, p->d_mod, p->d_pinv, level, K, p->logN);
    CKKS_LAUNCH_CHECK("moddown_final_kernel");
    return CKKS_OK;
}

// ModDown and rescale in one pass over the correction (merged giant step with CKKS_MATMUL_RESCALE):
//   out_r = rescale( z_r + ModDown(d_u[r]) ),   z_r [2][level][N] -> out_r [2][level-1][N],   n <= ROT_BATCH.
// d_u is consumed; d_w: n*2*level*N words, d_t: n*2*N words of scratch.  Returns CKKS_E_INVAL if the fused kernels do
// not apply to this parameter set (the caller then brings down and rescales in two steps).
int moddown_rescale(ckks_params *p, u32 level, u64 *d_u, const u64 *const *z, u64 *const *out, u32 n, u64 *d_w,
                    u64 *d_t, hipStream_t stream) {
    if (n == 0) return CKKS_OK;
    if (!moddown_mid_ok(p, level) || level < 2) return CKKS_E_INVAL;
    const u32 N = p->N, K = p->K, L = p->L, Wl = level + K;
    PtrPack zp;
    ItemPack op;
    for (u32 r = 0; r < ROT_BATCH; ++r) {
        zp.p[r] = z[r < n ? r : 0];
        SwitchItem &it = op.it[r];
        it.digits = it.c1 = it.c0 = it.key = nullptr;
        it.dst = out[r < n ? r : 0];
        it.galois_elt = 1;
        it.accumulate = 0;
    }
    LimbIds ids;
    for (u32 t = 0; t < Wl; ++t) ids.id[t] = (uint8_t)(t < level ? SKIP_ROW : L + (t - level));
    int rc = launch_ntt(p, d_u, ids, Wl, n * 2 * Wl, true, stream, 1, true);     // special limbs: inverse tile pass
    if (rc) return rc;
    hipLaunchKernelGGL(rescale_last_row_kernel, dim3(N / KS_THREADS, n * 2), dim3(KS_THREADS), 0, stream, zp, d_u, d_t,
                       p->d_mod, p->d_pinv, level, K, N);
    CKKS_LAUNCH_CHECK("rescale_last_row_kernel");
    ids.id[0] = (uint8_t)(level - 1);
    rc = launch_ntt(p, d_t, ids, 1, n * 2, true, stream);
    if (rc) return rc;
    launch_moddown_mid(p, d_u, d_w, n, level, Wl, level, stream, d_t);
    CKKS_LAUNCH_CHECK("moddown_mid_kernel");
    p->limb_ntts += (u64)n * 2 * (level - 1);
    for (u32 i = 0; i < level; ++i) ids.id[i] = (uint8_t)(i + 1 < level ? i : SKIP_ROW);
    rc = launch_ntt(p, d_w, ids, level, n * 2 * level, false, stream, 2);
    if (rc) return rc;
    hipLaunchKernelGGL(moddown_rescale_final_kernel, dim3(N / KS_THREADS / 2, level - 1, n * 2), dim3(KS_THREADS), 0,
                       stream, zp, op, d_u, d_w, p->d_mod, p->d_pinv, p->d_qlinv + (size_t)(level - 1) * L, level, K, N);
    CKKS_LAUNCH_CHECK("moddown_rescale_final_kernel");
    return CKKS_OK;
}

// n <= ROT_BATCH key switches from ready digits.  d_work: switch_scratch_words(level, n).
int switch_batch(ckks_params *p, u32 level, const SwitchItem *items, u32 n, u64 *d_work, hipStream_t stream) {
    if (n == 0) return CKKS_OK;
    if (n > ROT_BATCH) {
        set_error("switch_batch: %u items exceed one batch", n);
        return CKKS_E_INVAL;
    }
    const u32 N = p->N, K = p->K, L = p->L, Wl = level + K;
    const u32 beta = (level + p->alpha - 1) / p->alpha;
    ItemPack pack;
    const u32 n_groups = build_pack(items, n, pack);
    LimbIds ids;
    if (fast_ring(p) && beta <= MAX_BETA) {
        // inner product fused into the transforms on both sides of the base conversion
        u64 *y = d_work;                                   // [n][2][K][N]
        u64 *w = d_work + (size_t)n * 2 * K * N;           // [n][2][level][N]
        const u32 tiles = N >> 12;
        // at N = 2^12 the tile pass is the whole inverse transform and carries the (P/p_k)^-1 scaling itself
        const bool whole = p->logN == 12;
        const bool own_keys = n_groups == n;               // no two neighbouring items share a key
        hipLaunchKernelGGL(own_keys ? ip_intt_kernel<true> : ip_intt_kernel<false>, dim3(tiles, n * 2 * K),
                           dim3(NTT_THREADS), 0, stream, pack, y, p->d_mod, whole ? p->d_modf_dn : p->d_modf,
                           p->d_tws_inv, p->d_twf_inv, whole ? p->d_ninvs_dn : p->d_ninvs, n, level, K, L, beta,
                           p->logN);
        CKKS_LAUNCH_CHECK("ip_intt_kernel");
        p->limb_ntts += (u64)n * 2 * K;
        int rc;
        if (moddown_mid_ok(p, level)) {
            // column passes of the inverse transform (special limbs) and of the forward one (correction) inside the
            // base conversion: one kernel, y read once, w written once
            launch_moddown_mid(p, y, w, n, level, K, 0u, stream);
            CKKS_LAUNCH_CHECK("moddown_mid_kernel");
            p->limb_ntts += (u64)n * 2 * level;
        } else {
            for (u32 k = 0; k < K; ++k) ids.id[k] = (uint8_t)(L + k);
            rc = launch_ntt(p, y, ids, K, n * 2 * K, true, stream, 2, true);
            if (rc) return rc;
            launch_moddown_conv(p, y, w, n, level, K, 0u, stream);
            CKKS_LAUNCH_CHECK("moddown_conv_kernel");
            for (u32 i = 0; i < level; ++i) ids.id[i] = (uint8_t)i;
            rc = launch_ntt(p, w, ids, level, n * 2 * level, false, stream, 1, false);
            if (rc) return rc;
        }
        hipLaunchKernelGGL(own_keys ? passb_final_kernel<true> : passb_final_kernel<false>, dim3(tiles, n * 2 * level),
                           dim3(NTT_THREADS), 0, stream, pack, w, p->d_mod, p->d_modf, p->d_tws_fwd, p->d_twf_fwd,
                           p->d_ninvs, p->d_pinv, n, level, K, L, beta, p->alpha, p->logN);
        CKKS_LAUNCH_CHECK("passb_final_kernel");
        return CKKS_OK;
    }
    u64 *u = d_work;
    u64 *w = d_work + (size_t)n * 2 * Wl * N;
    hipLaunchKernelGGL(inner_product_kernel, dim3(N / KS_THREADS, Wl, n_groups), dim3(KS_THREADS), 0, stream, pack, u,
                       p->d_mod, level, K, L, beta, p->alpha, p->logN);
    CKKS_LAUNCH_CHECK("inner_product_kernel");
    for (u32 t = 0; t < Wl; ++t) ids.id[t] = (uint8_t)(t < level ? SKIP_ROW : L + (t - level));
    int rc = launch_ntt(p, u, ids, Wl, n * 2 * Wl, true, stream, 3, true);
    if (rc) return rc;
    launch_moddown_conv(p, u, w, n, level, Wl, level, stream);
    CKKS_LAUNCH_CHECK("moddown_conv_kernel");
    for (u32 i = 0; i < level; ++i) ids.id[i] = (uint8_t)i;
    rc = launch_ntt(p, w, ids, level, n * 2 * level, false, stream);
    if (rc) return rc;
    hipLaunchKernelGGL(moddown_final_kernel, dim3(N / KS_THREADS, level, n * 2), dim3(KS_THREADS), 0, stream, pack,
                       u, w, p->d_mod, p->d_pinv, level, K, p->logN);
    CKKS_LAUNCH_CHECK("moddown_final_kernel");
    return CKKS_OK;
}

}  // namespace ckks

namespace ckks {

size_t rotate_hoisted_scratch_words(const ckks_params *P, u32 level, u32 n_steps) {
    const u32 batch = std::max<u32>(1, std::min<u32>(ROT_BATCH, n_steps));
    return digits_words(P, level) + (size_t)level * P->N + switch_scratch_words(P, level, batch);
}

int rotate_hoisted(ckks_params *P, const u64 *d_ct_in, u32 level, const int32_t *steps, u32 n_steps,
                   const ckks_gkey *const *keys, u64 *d_ct_out, size_t reserve_words, hipStream_t stream) {
    if (!P || !d_ct_in || (n_steps && (!steps || !d_ct_out))) {
        set_error("ckks_rotate_hoisted: null argument");
        return CKKS_E_INVAL;
    }
    if (level == 0 || level > P->L) {
        set_error("ckks_rotate_hoisted: level %u outside [1,%u]", level, P->L);
        return CKKS_E_LEVEL;
    }
    const u32 N = P->N;
    const size_t ctw = (size_t)2 * level * N;
    if (words_overlap(d_ct_in, ctw, d_ct_out, (size_t)n_steps * ctw)) {   // the switches gather from the input
        set_error("ckks_rotate_hoisted: d_ct_out overlaps d_ct_in");
        return CKKS_E_INVAL;
    }
    std::vector<SwitchItem> items;
    std::vector<u32> copies;
    for (u32 r = 0; r < n_steps; ++r) {
        u64 g;
        ckks_galois_elt(P, steps[r], &g);
        if (g == 1) {
            copies.push_back(r);
            continue;
        }
        if (P->K == 0) {
            set_error("ckks_rotate_hoisted: parameter set has no special primes");
            return CKKS_E_INVAL;
        }
        if (!keys || !keys[r]) {
            set_error("ckks_rotate_hoisted: step %d (index %u) has no key", steps[r], r);
            return CKKS_E_NOKEY;
        }
        if (keys[r]->params != P || keys[r]->galois_elt != g) {
            set_error("ckks_rotate_hoisted: key %u is for Galois element %llu, step %d needs %llu", r,
                      (unsigned long long)keys[r]->galois_elt, steps[r], (unsigned long long)g);
            return CKKS_E_INVAL;
        }
        SwitchItem it;
        it.digits = nullptr;
        it.c1 = d_ct_in + (size_t)level * N;
        it.c0 = d_ct_in;
        it.key = keys[r]->d_key;
        it.dst = d_ct_out + (size_t)r * ctw;
        it.galois_elt = g;
        it.accumulate = 0;
        items.push_back(it);
    }
    for (u32 r : copies)
        CKKS_HIP(hipMemcpyAsync(d_ct_out + (size_t)r * ctw, d_ct_in, ctw * sizeof(u64), hipMemcpyDeviceToDevice,
                                stream));
    if (items.empty()) return CKKS_OK;
    const u32 batch = std::min<u32>(ROT_BATCH, (u32)items.size());
    const size_t dig_w = digits_words(P, level), tmp_w = (size_t)level * N;
    int rc = P->ensure_scratch((reserve_words + dig_w + tmp_w + switch_scratch_words(P, level, batch)) * sizeof(u64),
                               stream);
    if (rc) return rc;
    u64 *d_digits = (u64 *)P->d_scratch + reserve_words, *d_tmp = d_digits + dig_w, *d_work = d_tmp + tmp_w;
    const u64 *c1 = d_ct_in + (size_t)level * N;
    rc = decompose(P, &c1, 1, level, d_digits, d_tmp, stream);
    if (rc) return rc;
    for (auto &it : items) it.digits = d_digits;
    for (size_t done = 0; done < items.size(); done += batch) {
        u32 n = (u32)std::min<size_t>(batch, items.size() - done);
        rc = switch_batch(P, level, items.data() + done, n, d_work, stream);
        if (rc) return rc;
    }
    return CKKS_OK;
}

}  // namespace ckks

using namespace ckks;

extern "C" {

int ckks_galois_key_load(const ckks_params_t *P, uint64_t galois_elt, const uint64_t *d_key, void *stream,
                         ckks_gkey_t **out) {
    if (!out) {
        set_error("ckks_galois_key_load: out is null");
        return CKKS_E_INVAL;
    }
    *out = nullptr;
    if (!P || !d_key) {
        set_error("ckks_galois_key_load: null argument");
        return CKKS_E_INVAL;
    }
    if (P->K == 0) {
        set_error("ckks_galois_key_load: parameter set has no special primes");
        return CKKS_E_INVAL;
    }
    if (!(galois_elt & 1) || galois_elt >= 2ull * P->N || galois_elt == 1) {
        set_error("ckks_galois_key_load: %llu is not a non-trivial Galois element", (unsigned long long)galois_elt);
        return CKKS_E_INVAL;
    }
    ckks_gkey *k = new ckks_gkey();
    k->params = P;
    k->galois_elt = galois_elt;
    size_t rows = (size_t)P->dnum * 2 * P->W;
    hipError_t e = hipMalloc((void **)&k->d_key, rows * P->N * sizeof(u64));
    if (e != hipSuccess) {
        delete k;
        return hip_fail(e, "hipMalloc(key)");
    }
    hipLaunchKernelGGL(to_mont_kernel, dim3(P->N / KS_THREADS, (u32)rows), dim3(KS_THREADS), 0, (hipStream_t)stream,
                       d_key, k->d_key, P->d_mod, P->W, P->N);
    e = hipGetLastError();
    if (e != hipSuccess) {
        hipFree(k->d_key);
        delete k;
        return hip_fail(e, "to_mont_kernel");
    }
    *out = k;
    return CKKS_OK;
}

int ckks_galois_key_adopt(const ckks_params_t *P, uint64_t galois_elt, uint64_t *d_key, void *stream,
                          ckks_gkey_t **out) {
    if (!out) {
        set_error("ckks_galois_key_adopt: out is null");
        return CKKS_E_INVAL;
    }
    *out = nullptr;
    if (!P || !d_key || P->K == 0) {
        set_error("ckks_galois_key_adopt: null argument or no special primes");
        return CKKS_E_INVAL;
    }
    if (!(galois_elt & 1) || galois_elt >= 2ull * P->N || galois_elt == 1) {
        set_error("ckks_galois_key_adopt: %llu is not a non-trivial Galois element", (unsigned long long)galois_elt);
        return CKKS_E_INVAL;
    }
    const size_t rows = (size_t)P->dnum * 2 * P->W;
    // elementwise, each thread reads and writes its own word: in place is safe
    hipLaunchKernelGGL(to_mont_kernel, dim3(P->N / KS_THREADS, (u32)rows), dim3(KS_THREADS), 0, (hipStream_t)stream,
                       d_key, d_key, P->d_mod, P->W, P->N);
    CKKS_LAUNCH_CHECK("to_mont_kernel");
    ckks_gkey *k = new ckks_gkey();
    k->params = P;
    k->galois_elt = galois_elt;
    k->d_key = d_key;
    k->owned = false;
    *out = k;
    return CKKS_OK;
}

int ckks_relin_key_load(const ckks_params_t *P, const uint64_t *d_key, void *stream, ckks_gkey_t **out) {
    if (!out) {
        set_error("ckks_relin_key_load: out is null");
        return CKKS_E_INVAL;
    }
    *out = nullptr;
    if (!P || !d_key || P->K == 0) {
        set_error("ckks_relin_key_load: null argument or no special primes");
        return CKKS_E_INVAL;
    }
    ckks_gkey *k = new ckks_gkey();
    k->params = P;
    k->galois_elt = 1;   // no automorphism: the key switches from s^2
    size_t rows = (size_t)P->dnum * 2 * P->W;
    hipError_t e = hipMalloc((void **)&k->d_key, rows * P->N * sizeof(u64));
    if (e != hipSuccess) {
        delete k;
        return hip_fail(e, "hipMalloc(key)");
    }
    hipLaunchKernelGGL(to_mont_kernel, dim3(P->N / KS_THREADS, (u32)rows), dim3(KS_THREADS), 0, (hipStream_t)stream,
                       d_key, k->d_key, P->d_mod, P->W, P->N);
    e = hipGetLastError();
    if (e != hipSuccess) {
        hipFree(k->d_key);
        delete k;
        return hip_fail(e, "to_mont_kernel");
    }
    *out = k;
    return CKKS_OK;
}

int ckks_ctmul(ckks_params_t *P, const uint64_t *d_ct_a, const uint64_t *d_ct_b, uint32_t level,
               const ckks_gkey_t *relin_key, uint64_t *d_ct_out, void *stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    if (!P || !d_ct_a || !d_ct_b || !d_ct_out) {
        set_error("ckks_ctmul: null argument");
        return CKKS_E_INVAL;
    }
    if (level == 0 || level > P->L) {
        set_error("ckks_ctmul: level %u outside [1,%u]", level, P->L);
        return CKKS_E_LEVEL;
    }
    if (!relin_key) {
        set_error("ckks_ctmul: no relinearisation key");
        return CKKS_E_NOKEY;
    }
    if (relin_key->params != P || relin_key->galois_elt != 1) {
        set_error("ckks_ctmul: the key is not a relinearisation key of this parameter set");
        return CKKS_E_INVAL;
    }
    const u32 N = P->N;
    if (words_overlap(d_ct_out, (size_t)2 * level * N, d_ct_a, (size_t)2 * level * N) ||
        words_overlap(d_ct_out, (size_t)2 * level * N, d_ct_b, (size_t)2 * level * N)) {
        set_error("ckks_ctmul: d_ct_out overlaps an input");
        return CKKS_E_INVAL;
    }
    const size_t dig_w = digits_words(P, level), lim_w = (size_t)level * N;
    int rc = P->ensure_scratch((dig_w + 2 * lim_w + switch_scratch_words(P, level, 1)) * sizeof(u64), stream);
    if (rc) return rc;
    u64 *d_digits = (u64 *)P->d_scratch, *d_tmp = d_digits + dig_w, *d_t2 = d_tmp + lim_w, *d_work = d_t2 + lim_w;
    hipLaunchKernelGGL(tensor_kernel, dim3(N / KS_THREADS, level), dim3(KS_THREADS), 0, stream, d_ct_a, d_ct_b,
                       d_ct_out, d_t2, P->d_mod, level, N);
    CKKS_LAUNCH_CHECK("tensor_kernel");
    const u64 *c1 = d_t2;
    rc = decompose(P, &c1, 1, level, d_digits, d_tmp, stream);
    if (rc) return rc;
    SwitchItem it;
    it.digits = d_digits;
    it.c1 = d_t2;
    it.c0 = nullptr;            // (t0, t1) are already in the output: the switch only adds ModDown(...)
    it.key = relin_key->d_key;
    it.dst = d_ct_out;
    it.galois_elt = 1;
    it.accumulate = 1;
    return switch_batch(P, level, &it, 1, d_work, stream);
}

void ckks_galois_key_destroy(ckks_gkey_t *key) {
    if (!key) return;
    if (key->owned) hipFree(key->d_key);
    delete key;
}

int ckks_rotate_hoisted(ckks_params_t *P, const uint64_t *d_ct_in, uint32_t level, const int32_t *steps,
                        uint32_t n_steps, const ckks_gkey_t *const *keys, uint64_t *d_ct_out, void *stream_) {
    return rotate_hoisted(P, d_ct_in, level, steps, n_steps, keys, d_ct_out, 0, (hipStream_t)stream_);
}

}  // extern "C"
