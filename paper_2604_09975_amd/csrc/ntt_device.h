// Device-side building blocks of the radix-16 NTT (N = 2^12 and 2^16), shared by the transform kernels
// and by the key-switch kernels that fuse other work into a transform pass.
#pragma once
#include "ckks_internal.h"

namespace ckks {

constexpr u32 NTT_THREADS = 256;

// LDS slot of tile element i: one padding word after every 16 elements.  The three access patterns of the tile pass
// (residues 256 apart, 16 apart, and 16 consecutive ones per thread) then fall on distinct banks, and, unlike an
// XOR fold, every slot a thread touches is its base slot plus a compile-time offset: no address registers, which is
// what brings the pass from 130 to under 100 vector registers.  A tile takes 34 KiB; four fit a CU.
__device__ __forceinline__ u32 lds_pad(u32 i) { return i + (i >> 4); }
constexpr u32 FAST_LDS_WORDS = 4096 + 256;

// Integer butterflies for primes that do not fit the fp64 scheme (the 60-bit special primes): lazy values and
// twiddles with a precomputed quotient.  A twiddle is the pair (w, w') with w' = floor(w * 2^64 / q); for any 64-bit
// y, y*w - floor(y*w' / 2^64) * q lies in [0, 2q) and is congruent to y*w: one high product and two low products,
// no correction step.  Forward values live in [0, 4q), inverse values in [0, 2q) (q < 2^62 keeps 4q in a word);
// out() brings a value back to [0, q).
struct TwInt {
    u64 w, ws;
};

struct FieldInt {
    typedef u64 T;
    typedef TwInt W;
    u64 q, q2;
    const ulonglong2 *tw;
    TwInt n0, n1;
    __device__ __forceinline__ T in(u64 x) const { return x; }
    __device__ __forceinline__ u64 out(T x) const {
        if (x >= q2) x -= q2;
        if (x >= q) x -= q;
        return x;
    }
    __device__ __forceinline__ u64 bits(T x) const { return x; }
    __device__ __forceinline__ T from_bits(u64 x) const { return x; }
    __device__ __forceinline__ W twid(u32 idx) const {
        const ulonglong2 t = tw[idx];
        return TwInt{t.x, t.y};
    }
    __device__ __forceinline__ void norm(T &) const {}
    __device__ __forceinline__ T mul(T y, const W &w) const { return y * w.w - mul_hi(y, w.ws) * q; }   // [0, 2q)
    __device__ __forceinline__ void fwd(T &x, T &y, const W &w) const {
        if (x >= q2) x -= q2;
        const T v = mul(y, w);
        y = x - v + q2;
        x = x + v;
    }
    __device__ __forceinline__ void inv(T &x, T &y, const W &w) const {
        T s = x + y;
        if (s >= q2) s -= q2;
        y = mul(x - y + q2, w);
        x = s;
    }
    __device__ __forceinline__ void inv_last(T &x, T &y) const {
        const T s = x + y, d = x - y + q2;
        x = mul(s, n0);
        y = mul(d, n1);
    }
};

// Exact integer arithmetic in doubles for q < 2^50.  mul(a, w) returns r = a*w - c*q with
// c = rint(a*w/q) computed in floating point: |r| <= (1/2 + 3|a|/2^53) q, exact as long as
// |a| <= 2^52.  Sums stay exact below 2^53.  norm() brings a value back to |x| <= q/2.
struct FieldFp {
    typedef double T;
    typedef double W;
    double q, u, n0, n1;
    const double *tw;
    __device__ __forceinline__ T in(u64 x) const {
        return __longlong_as_double((long long)(x | 0x4330000000000000ull)) - 4503599627370496.0;
    }
    __device__ __forceinline__ void norm(T &x) const {
        const double c = rint(x * u);
        x = fma(-c, q, x);
    }
    __device__ __forceinline__ u64 out(T x) const {
        norm(x);
        if (x < 0) x += q;
        return (u64)__double_as_longlong(x + 4503599627370496.0) & 0x000fffffffffffffull;
    }
    __device__ __forceinline__ u64 bits(T x) const { return (u64)__double_as_longlong(x); }
    __device__ __forceinline__ T from_bits(u64 x) const { return __longlong_as_double((long long)x); }
    __device__ __forceinline__ T twid(u32 idx) const { return tw[idx]; }
    __device__ __forceinline__ T mul(T a, T w) const {
        const double h = a * w;
        const double l = fma(a, w, -h);
        const double c = rint(h * u);
        const double d = fma(-c, q, h);
        return d + l;
    }
    __device__ __forceinline__ void fwd(T &x, T &y, T w) const {
        const T v = mul(y, w);
        y = x - v;
        x = x + v;
    }
    __device__ __forceinline__ void inv(T &x, T &y, T w) const {
        const T s = x + y;
        y = mul(x - y, w);
        x = s;
    }
    __device__ __forceinline__ void inv_last(T &x, T &y) const {
        const T s = x + y, d = x - y;
        x = mul(s, n0);
        y = mul(d, n1);
    }
};

// Four stages on the 16 values a thread holds.  The group is node `nb` of stage s0; at stage
// s0 + t it covers nodes (nb << t) + k, k < 2^t, and values j, j + (8 >> t) pair up.
template <class F>
__device__ __forceinline__ void radix16_fwd(const F &f, typename F::T (&v)[16], u32 s0, u32 nb) {
#pragma unroll
    for (u32 j = 0; j < 16; ++j) f.norm(v[j]);
#pragma unroll
    for (u32 t = 0; t < 4; ++t) {
        const u32 g = 8u >> t;
#pragma unroll
        for (u32 k = 0; k < (1u << t); ++k) {
            const typename F::W w = f.twid((1u << (s0 + t)) + (nb << t) + k);
#pragma unroll
            for (u32 i = 0; i < g; ++i) f.fwd(v[k * 2 * g + i], v[k * 2 * g + i + g], w);
        }
    }
}

template <class F>
__device__ __forceinline__ void radix16_inv(const F &f, typename F::T (&v)[16], u32 s0, u32 nb, bool last) {
#pragma unroll
    for (u32 j = 0; j < 16; ++j) f.norm(v[j]);
#pragma unroll
    for (int t = 3; t >= 0; --t) {
        const u32 g = 8u >> t;
        if (t == 1) {
#pragma unroll
            for (u32 j = 0; j < 16; ++j) f.norm(v[j]);
        }
        if (t == 0 && last) {
#pragma unroll
            for (u32 i = 0; i < 8; ++i) f.inv_last(v[i], v[i + 8]);
        } else {
#pragma unroll
            for (u32 k = 0; k < (1u << t); ++k) {
                const typename F::W w = f.twid((1u << (s0 + t)) + (nb << t) + k);
#pragma unroll
                for (u32 i = 0; i < g; ++i) f.inv(v[k * 2 * g + i], v[k * 2 * g + i + g], w);
            }
        }
    }
}

// pass B: the last 12 stages act inside aligned runs of 4096 consecutive residues, one workgroup per run, in three
// radix-16 rounds with an LDS exchange between them:
//   round 1 (stages logN-12 .. logN-9): thread t holds residues j*256 + t          (2 KiB runs in global memory)
//   round 2 (stages logN-8  .. logN-5): thread (blk, c) holds blk*256 + c + 16*j
//   round 3 (stages logN-4  .. logN-1): thread (blk, c) holds blk*256 + 16*c + j
// For N = 2^12 this is the whole transform.  The passes come in halves so that callers can put their own code
// between global memory and LDS.  LDS slot of residue e of the tile: lds[lds_pad(e)].
//
// forward: load(idx) gives the canonical residue at index idx of the polynomial (round-1 pattern: coalesced); on
// return the tile's transformed, canonical residues are in LDS and the workgroup is synced.  RAW: the residues are
// left in the field's own form instead (f.bits of a value brought back by f.norm: for the fp64 field a double with
// |x| <= q/2), for a caller that goes on computing in that field and would only convert them back.
template <bool RAW = false, class F, class Load>
__device__ __forceinline__ void pass_b_fwd_to_lds(const F &f, u32 logN, u64 *lds, Load load) {
    const u32 tid = threadIdx.x, blk = tid >> 4, c = tid & 15;
    const u32 base = blockIdx.x << 12;
    const u32 run = (base >> 8) + blk;              // which run of 256 in the polynomial
    const u32 strided = blk * 256 + c, contig = blk * 256 + c * 16;
    typename F::T v[16];
#pragma unroll
    for (u32 j = 0; j < 16; ++j) v[j] = f.in(load(base + j * 256 + tid));
    radix16_fwd(f, v, logN - 12, blockIdx.x);
#pragma unroll
    for (u32 j = 0; j < 16; ++j) lds[lds_pad(j * 256 + tid)] = f.bits(v[j]);
    __syncthreads();
#pragma unroll
    for (u32 j = 0; j < 16; ++j) v[j] = f.from_bits(lds[lds_pad(strided + j * 16)]);
    radix16_fwd(f, v, logN - 8, run);
#pragma unroll
    for (u32 j = 0; j < 16; ++j) lds[lds_pad(strided + j * 16)] = f.bits(v[j]);   // a thread's own slots
    __syncthreads();
#pragma unroll
    for (u32 j = 0; j < 16; ++j) v[j] = f.from_bits(lds[lds_pad(contig + j)]);
    radix16_fwd(f, v, logN - 4, run * 16 + c);
#pragma unroll
    for (u32 j = 0; j < 16; ++j) {                                          // a thread's own slots
        if (RAW) {
            f.norm(v[j]);
            lds[lds_pad(contig + j)] = f.bits(v[j]);
        } else {
            lds[lds_pad(contig + j)] = f.out(v[j]);
        }
    }
    __syncthreads();
}

// inverse: expects the tile's canonical residues in LDS (workgroup synced); store(idx, value) receives the
// canonical results in the round-1 pattern (coalesced).  whole: the tile is the whole polynomial (N = 2^12), so the
// last round ends the transform and folds in N^-1.
template <class F, class Store>
__device__ __forceinline__ void pass_b_inv_from_lds(const F &f, u32 logN, u64 *lds, Store store) {
    const u32 tid = threadIdx.x, blk = tid >> 4, c = tid & 15;
    const u32 base = blockIdx.x << 12;
    const u32 run = (base >> 8) + blk;
    const u32 strided = blk * 256 + c, contig = blk * 256 + c * 16;
    typename F::T v[16];
#pragma unroll
    for (u32 j = 0; j < 16; ++j) v[j] = f.in(lds[lds_pad(contig + j)]);
    radix16_inv(f, v, logN - 4, run * 16 + c, false);
#pragma unroll
    for (u32 j = 0; j < 16; ++j) lds[lds_pad(contig + j)] = f.bits(v[j]);   // a thread's own slots
    __syncthreads();
#pragma unroll
    for (u32 j = 0; j < 16; ++j) v[j] = f.from_bits(lds[lds_pad(strided + j * 16)]);
    radix16_inv(f, v, logN - 8, run, false);
#pragma unroll
    for (u32 j = 0; j < 16; ++j) lds[lds_pad(strided + j * 16)] = f.bits(v[j]);   // a thread's own slots
    __syncthreads();
#pragma unroll
    for (u32 j = 0; j < 16; ++j) v[j] = f.from_bits(lds[lds_pad(j * 256 + tid)]);
    radix16_inv(f, v, logN - 12, blockIdx.x, logN == 12);
#pragma unroll
    for (u32 j = 0; j < 16; ++j) store(base + j * 256 + tid, f.out(v[j]));
}

// Whole pass with coalesced stores (forward) / coalesced loads (inverse).
template <bool INV, class F, class Load, class Store>
__device__ __forceinline__ void pass_b_body(const F &f, u32 logN, u64 *lds, Load load, Store store) {
    const u32 tid = threadIdx.x, base = blockIdx.x << 12;
    if (!INV) {
        pass_b_fwd_to_lds(f, logN, lds, load);
#pragma unroll
        for (u32 i = 0; i < 16; ++i) store(base + tid + 256 * i, lds[lds_pad(tid + 256 * i)]);
    } else {
#pragma unroll
        for (u32 i = 0; i < 16; ++i) lds[lds_pad(tid + 256 * i)] = load(base + tid + 256 * i);
        __syncthreads();
        pass_b_inv_from_lds(f, logN, lds, store);
    }
}

// pass A for N = 2^16: the first 4 stages pair residues 4096 apart, so a thread that owns one of the 4096 columns
// holds its 16 rows in registers: no LDS, every access a run of consecutive residues.  col: the thread's column;
// load(idx) / store(idx, value) see canonical residues at index idx of the polynomial.
template <bool INV, class F, class Load, class Store>
__device__ __forceinline__ void pass_a16_body(const F &f, u32 col, Load load, Store store) {
    typename F::T v[16];
#pragma unroll
    for (u32 j = 0; j < 16; ++j) v[j] = f.in(load(j * 4096 + col));
    if (!INV)
        radix16_fwd(f, v, 0, 0);
    else
        radix16_inv(f, v, 0, 0, true);
#pragma unroll
    for (u32 j = 0; j < 16; ++j) store(j * 4096 + col, f.out(v[j]));
}

// Field objects for limb `limb` from the parameter tables.
__device__ __forceinline__ FieldFp make_field_fp(const ModFp &mf, const double *twf, u32 limb, u32 logN) {
    FieldFp f;
    f.q = mf.q;
    f.u = mf.u;
    f.n0 = mf.ninv;
    f.n1 = mf.ninv_w;
    f.tw = twf + ((size_t)limb << logN);
    return f;
}

// tws: [W][N] pairs (w, w') as consecutive words, ninvs: [W][4] = N^-1, its quotient, N^-1 psi^-(N/2), its quotient
__device__ __forceinline__ FieldInt make_field_int(const ModConst *mods, const u64 *tws, const u64 *ninvs, u32 limb,
                                                   u32 logN) {
    FieldInt f;
    f.q = mods[limb].q;
    f.q2 = 2 * f.q;
    f.tw = reinterpret_cast<const ulonglong2 *>(tws) + ((size_t)limb << logN);
    f.n0 = TwInt{ninvs[4 * limb], ninvs[4 * limb + 1]};
    f.n1 = TwInt{ninvs[4 * limb + 2], ninvs[4 * limb + 3]};
    return f;
}

}  // namespace ckks
