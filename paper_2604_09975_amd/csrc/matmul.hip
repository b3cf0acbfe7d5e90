// The projection kernel Y = XW on ciphertexts (Sec. 3.2, App. A.2) and rescale (Sec. 2.2).
//
//   bank     x_q^(g) = rot(x^(g); q*m), q < N1            one hoisted call per input group
//   diagonal acc_{b,p} = sum_g sum_q x_q^(g) (.) w_{b,p,g,q}  the byte mover: every weight limb is read once
//   giant    y_b = acc_{b,0} + sum_{p>=1} rot(acc_{b,p}; p*N1*m)
//   bias     y_b.c0 += bias_b
// Real packing: the imaginary half of the complex weights of App. A.2.1 is not used.
#include <algorithm>

#include "ckks_internal.h"
#include "common_kernels.h"

namespace ckks {

constexpr u32 MM_THREADS = 256;
constexpr u32 MM_TB = 8;   // (b,p) accumulators kept in registers per thread

// int64 coefficients [count][N] -> canonical residues [count][level][N]
__global__ __launch_bounds__(EW_THREADS) void expand_coeffs_kernel(const int64_t *__restrict__ coef,
                                                                   u64 *__restrict__ out,
                                                                   const ModConst *__restrict__ mods, u32 level,
                                                                   u32 N) {
    const u32 n = blockIdx.x * EW_THREADS + threadIdx.x;
    const u32 d = blockIdx.y;
    const int64_t v = coef[(size_t)d * N + n];
    for (u32 i = 0; i < level; ++i) out[((size_t)d * level + i) * N + n] = reduce_signed(v, mods[i]);
}

// rows [rows][N], row r modulo limb r % level: x <- x * c mod q (c canonical, any size)
__global__ __launch_bounds__(EW_THREADS) void scale_rows_kernel(u64 *data, const ModConst *__restrict__ mods,
                                                                u32 level, u32 N, u64 c) {
    const u32 n = blockIdx.x * EW_THREADS + threadIdx.x;
    const u32 row = blockIdx.y;
    const ModConst m = mods[row % level];
    const u64 cm = mont_mul(reduce_any(c, m), m.r2, m);
    const size_t idx = (size_t)row * N + n;
    data[idx] = mont_mul(data[idx], cm, m);
}

// acc[bp][comp][i][k] = sum_{gq} bank[gq][comp][i][k] * w[bp][gq][i][k]
// grid: x = tile of (b,p) pairs (fastest), y = run of coefficients, z = limb (slowest: one limb's bank slice
//       stays resident in the Infinity Cache while all its tiles run).  An XCD-aware remapping of x/y and a
//       variant whose four wavefronts share their bank loads were measured and did not help.
// Weight limbs are stored in the library's internal form: for a prime below 2^50 the residue as a
// double (products are then reduced with the exact FMA scheme of the NTT butterflies and summed as
// signed doubles, about 7 issue slots per product), otherwise in Montgomery form (128-bit lazy sums;
// flush = number of products that fit such a sum for the largest modulus).
// blockIdx.z indexes `limbs`, the list of limbs this launch covers (fp64 limbs and Montgomery limbs
// go to separate launches so that each kernel keeps its own register budget).
// Each thread owns VEC adjacent coefficients (16-byte loads for VEC = 2) and TB (b,p) accumulators.
// Packed weight records: 50 bits per residue instead of 64, in three parts: the low 32 bits, bits 32..47, and
// bits 48..49 four residues to a byte.  A half record holds the first N/2 residues of a limb (real diagonals,
// the rest is the mirror image), a whole-limb record all N.
__host__ __device__ inline size_t packed_record_bytes(u32 N) { return (size_t)3 * N + N / 8; }
// A record is a sequence of 800-byte chunks of 128 residues (what one wavefront reads per weight limb and step):
// 512 bytes of low words, 256 of middle halves, 32 of top bits, so that the three loads of a wavefront fall into
// one contiguous piece of memory.  Byte offsets of residue k's parts within the record:
__host__ __device__ inline u32 packed_lo(u32 k) { return (k >> 7) * 800u + 4u * (k & 127u); }
__host__ __device__ inline u32 packed_hi(u32 k) { return (k >> 7) * 800u + 512u + 2u * (k & 127u); }
__host__ __device__ inline u32 packed_top(u32 k) { return (k >> 7) * 800u + 768u + ((k & 127u) >> 2); }

// PACKED (VEC = 2): the weight limbs are whole-limb packed records.
// FULL: every tile of the launch has all its TB pairs (no per-pair guards: the loop body stays one basic block and the
// loaded registers are not copied around); tiles are numbered from tile0.
template <u32 TB, u32 VEC, bool PACKED, bool FULL>
__global__ __launch_bounds__(MM_THREADS) void diag_mac_kernel(const u64 *__restrict__ bank,
                                                              const u64 *__restrict__ w, u64 *__restrict__ acc,
                                                              const ModFp *__restrict__ modf, LimbIds limbs,
                                                              u32 level, u32 N, u32 GQ, u32 BP, u32 swizzle,
                                                              u32 gq0, u32 gq1, u32 accumulate, u32 tile0) {
    // steps gq0 .. gq1-1 of the GQ per pair are summed; accumulate: onto what acc already holds
    static_assert(!PACKED || VEC == 2, "packed weights are read in pairs");
    typedef u64 vec_t __attribute__((ext_vector_type(VEC)));
    // swizzle: one XCD walks all (b,p) tiles of a run of coefficients back to back (see diag_mac_sym_kernel)
    u32 tile = blockIdx.x, run = blockIdx.y;
    if (swizzle) {
        const u32 lin = blockIdx.y * gridDim.x + blockIdx.x;
        const u32 xcd = lin & 7, slot = lin >> 3;
        tile = slot % gridDim.x;
        run = (slot / gridDim.x) * 8 + xcd;
    }
    const u32 bp0 = (tile0 + tile) * TB;
    const u32 k = (run * MM_THREADS + threadIdx.x) * VEC;
    const u32 i = limbs.id[blockIdx.z];
    const size_t limb_off = (size_t)i * N + k;
    const size_t w_stride = (size_t)level * N;         // between consecutive gq of one (b,p)
    const ModFp mf = modf[i];
    const double q = mf.q, u = mf.u;
    double a0[TB][VEC], a1[TB][VEC];
#pragma unroll
    for (u32 t = 0; t < TB; ++t)
#pragma unroll
        for (u32 e = 0; e < VEC; ++e) a0[t][e] = a1[t][e] = 0.0;
    // loads of step gq+1 are issued before the arithmetic of step gq
    typedef u32 wvec_t __attribute__((ext_vector_type(4)));
    vec_t xb0, xb1;
    wvec_t wb[TB];
    const size_t rec = 2 * packed_record_bytes(N);
    const unsigned char *wbytes = reinterpret_cast<const unsigned char *>(w);
    const u32 off_lo = packed_lo(k), off_hi = packed_hi(k), off_top = packed_top(k);
    const u32 top_shift = (k & 2) * 2;
    auto fetch = [&](u32 gq) {
        xb0 = *reinterpret_cast<const vec_t *>(bank + ((size_t)gq * 2 + 0) * w_stride + limb_off);
        xb1 = *reinterpret_cast<const vec_t *>(bank + ((size_t)gq * 2 + 1) * w_stride + limb_off);
#pragma unroll
        for (u32 t = 0; t < TB; ++t)
            if (FULL || bp0 + t < BP) {
                if (PACKED) {
                    const unsigned char *r = wbytes + (((size_t)(bp0 + t) * GQ + gq) * level + i) * rec;
                    const __amdgpu_buffer_rsrc_t rs =
                        __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char *>(r), 0, (int)rec, 0x00020000);
                    typedef u32 u32x2 __attribute__((ext_vector_type(2)));
                    const u32x2 lo = __builtin_amdgcn_raw_buffer_load_b64(rs, (int)off_lo, 0, 0);
                    wb[t][0] = lo[0];
                    wb[t][1] = lo[1];
                    wb[t][2] = __builtin_amdgcn_raw_buffer_load_b32(rs, (int)off_hi, 0, 0);
                    wb[t][3] = __builtin_amdgcn_raw_buffer_load_b8(rs, (int)off_top, 0, 0);
                } else {
                    const vec_t v = *reinterpret_cast<const vec_t *>(w + ((size_t)(bp0 + t) * GQ + gq) * w_stride + limb_off);
#pragma unroll
                    for (u32 e = 0; e < VEC; ++e) {
                        wb[t][2 * e] = (u32)v[e];
                        wb[t][2 * e + 1] = (u32)(v[e] >> 32);
                    }
                }
            }
    };
    if (accumulate) {
#pragma unroll
        for (u32 t = 0; t < TB; ++t)
            if (FULL || bp0 + t < BP) {
                const vec_t p0 = *reinterpret_cast<const vec_t *>(acc + ((size_t)(bp0 + t) * 2 + 0) * w_stride + limb_off);
                const vec_t p1 = *reinterpret_cast<const vec_t *>(acc + ((size_t)(bp0 + t) * 2 + 1) * w_stride + limb_off);
#pragma unroll
                for (u32 e = 0; e < VEC; ++e) {
                    a0[t][e] = (double)p0[e];
                    a1[t][e] = (double)p1[e];
                }
            }
    }
    fetch(gq0);
    for (u32 gq = gq0; gq < gq1; ++gq) {
        double x0[VEC], x1[VEC];
#pragma unroll
        for (u32 e = 0; e < VEC; ++e) {
            x0[e] = __longlong_as_double((long long)(xb0[e] | 0x4330000000000000ull)) - 4503599627370496.0;
            x1[e] = __longlong_as_double((long long)(xb1[e] | 0x4330000000000000ull)) - 4503599627370496.0;
        }
        double wd[TB][VEC];
#pragma unroll
        for (u32 t = 0; t < TB; ++t) {
            if (PACKED) {
                const u32 top = wb[t][3] >> top_shift;
                const u32 h0 = 0x43300000u | ((top & 3u) << 16) | (wb[t][2] & 0xffffu);
                const u32 h1 = 0x43300000u | ((top & 12u) << 14) | (wb[t][2] >> 16);
                wd[t][0] = __hiloint2double((int)h0, (int)wb[t][0]) - 4503599627370496.0;
                wd[t][VEC - 1] = __hiloint2double((int)h1, (int)wb[t][1]) - 4503599627370496.0;
            } else {
#pragma unroll
                for (u32 e = 0; e < VEC; ++e) wd[t][e] = __hiloint2double((int)wb[t][2 * e + 1], (int)wb[t][2 * e]);
            }
        }
        if (gq + 1 < gq1) fetch(gq + 1);
#pragma unroll
        for (u32 t = 0; t < TB; ++t) {
            if (FULL || bp0 + t < BP) {
#pragma unroll
                for (u32 e = 0; e < VEC; ++e) {
                    const double wv = wd[t][e];
                    // x*w = h + l exactly; subtract the nearest multiple of q: |r| < 0.9 q
                    const double h0 = x0[e] * wv, h1 = x1[e] * wv;
                    const double l0 = fma(x0[e], wv, -h0), l1 = fma(x1[e], wv, -h1);
                    const double c0 = rint(h0 * u), c1 = rint(h1 * u);
                    a0[t][e] += fma(-c0, q, h0) + l0;
                    a1[t][e] += fma(-c1, q, h1) + l1;
                }
            }
        }
        if (((gq - gq0) & 7) == 7) {   // keep the signed sums far below 2^53
#pragma unroll
            for (u32 t = 0; t < TB; ++t)
#pragma unroll
                for (u32 e = 0; e < VEC; ++e) {
                    a0[t][e] = fma(-rint(a0[t][e] * u), q, a0[t][e]);
                    a1[t][e] = fma(-rint(a1[t][e] * u), q, a1[t][e]);
                }
        }
    }
#pragma unroll
    for (u32 t = 0; t < TB; ++t) {
        if (FULL || bp0 + t < BP) {
            vec_t o0, o1;
#pragma unroll
            for (u32 e = 0; e < VEC; ++e) {
                double v0 = fma(-rint(a0[t][e] * u), q, a0[t][e]), v1 = fma(-rint(a1[t][e] * u), q, a1[t][e]);
                if (v0 < 0) v0 += q;
                if (v1 < 0) v1 += q;
                o0[e] = (u64)__double_as_longlong(v0 + 4503599627370496.0) & 0x000fffffffffffffull;
                o1[e] = (u64)__double_as_longlong(v1 + 4503599627370496.0) & 0x000fffffffffffffull;
            }
            *reinterpret_cast<vec_t *>(acc + ((size_t)(bp0 + t) * 2 + 0) * w_stride + limb_off) = o0;
            *reinterpret_cast<vec_t *>(acc + ((size_t)(bp0 + t) * 2 + 1) * w_stride + limb_off) = o1;
        }
    }
}

// dst[z][0 .. words) = src[z * src_stride + 0 .. words), z = blockIdx.z; words is a multiple of 2 * EW_THREADS
__global__ __launch_bounds__(EW_THREADS) void copy_blocks_kernel(u64 *__restrict__ dst, const u64 *__restrict__ src,
                                                                 size_t words, size_t src_stride) {
    typedef u64 vec_t __attribute__((ext_vector_type(2)));
    const size_t k = ((size_t)blockIdx.x * EW_THREADS + threadIdx.x) * 2;
    *reinterpret_cast<vec_t *>(dst + blockIdx.z * words + k) =
        *reinterpret_cast<const vec_t *>(src + blockIdx.z * src_stride + k);
}

// c0 of block b (at y + b * y_stride) += bias[b]: blockIdx.y = limb, blockIdx.z = output block, two residues per thread
__global__ __launch_bounds__(EW_THREADS) void add_bias_kernel(u64 *__restrict__ y, size_t y_stride,
                                                              const u64 *__restrict__ bias,
                                                              const ModConst *__restrict__ mods, u32 level, u32 N) {
    typedef u64 vec_t __attribute__((ext_vector_type(2)));
    const u32 k = (blockIdx.x * EW_THREADS + threadIdx.x) * 2, i = blockIdx.y, b = blockIdx.z;
    const u64 q = mods[i].q;
    vec_t *dst = reinterpret_cast<vec_t *>(y + (size_t)b * y_stride + (size_t)i * N + k);
    const vec_t s = *reinterpret_cast<const vec_t *>(bias + ((size_t)b * level + i) * N + k);
    vec_t v = *dst;
    v[0] = add_mod(v[0], s[0], q);
    v[1] = add_mod(v[1], s[1], q);
    *dst = v;
}

// Same sum for plaintexts that encode REAL slot vectors.  Such a polynomial is fixed by X -> X^-1, so its
// transform is a palindrome: w[k] = w[N-1-k] (the exponents 2*bitrev(k)+1 and 2*bitrev(N-1-k)+1 are
// negatives of each other mod 2N).  Only the first half of every weight limb is read; each value serves
// coefficient k and its mirror.  A thread owns coefficients k, k+1 and N-2-k, N-1-k and TB (b,p) pairs.
// Workgroups go to the XCDs round-robin and each XCD has its own L2, so when the run count allows it the
// linear workgroup id is unfolded to let one XCD walk all (b,p) tiles of a run of coefficients back to
// back: the bank lines of that run are then fetched into one L2 once.
// PACKED: the half limb is stored in 50 bits per residue instead of 64 (packed_record_bytes) in three parts,
// the low 32 bits, bits 32..47, and bits 48..49 four residues to a byte.  The double is rebuilt as
// (2^52 + x) - 2^52 from the bit pattern, one addition per weight.
// FULL, tile0: as in diag_mac_kernel.
template <u32 TB, bool PACKED, bool FULL>
__global__ __launch_bounds__(MM_THREADS) void diag_mac_sym_kernel(const u64 *__restrict__ bank,
                                                                  const u64 *__restrict__ w, u64 *__restrict__ acc,
                                                                  const ModFp *__restrict__ modf, LimbIds limbs,
                                                                  u32 level, u32 N, u32 GQ, u32 BP, u32 swizzle,
                                                                  u32 gq0, u32 gq1, u32 accumulate, u32 tile0) {
    // steps gq0 .. gq1-1 of the GQ per pair are summed; accumulate: onto what acc already holds
    typedef u64 vec_t __attribute__((ext_vector_type(2)));
    typedef u32 wvec_t __attribute__((ext_vector_type(4)));      // one (b,p) pair's two weights as loaded
    u32 tile = blockIdx.x, run = blockIdx.y;
    if (swizzle) {
        const u32 lin = blockIdx.y * gridDim.x + blockIdx.x;
        const u32 xcd = lin & 7, slot = lin >> 3;
        tile = slot % gridDim.x;
        run = (slot / gridDim.x) * 8 + xcd;
    }
    const u32 bp0 = (tile0 + tile) * TB;
    const u32 k = (run * MM_THREADS + threadIdx.x) * 2;          // k < N/2
    const u32 km = N - 2 - k;                                    // mirrors of k+1, k
    const u32 i = limbs.id[blockIdx.z];
    const size_t row = (size_t)i * N;
    const size_t w_stride = (size_t)level * N;
    const ModFp mf = modf[i];
    const double q = mf.q, u = mf.u;
    double a[TB][2][4];                                          // [pair][component][k, k+1, N-2-k, N-1-k]
#pragma unroll
    for (u32 t = 0; t < TB; ++t)
#pragma unroll
        for (u32 e = 0; e < 4; ++e) a[t][0][e] = a[t][1][e] = 0.0;
    // loads of step gq+1 are issued before the arithmetic of step gq
    vec_t xb[2][2];
    wvec_t wb[TB];
    const size_t rec = packed_record_bytes(N);
    const unsigned char *wbytes = reinterpret_cast<const unsigned char *>(w);
    const u32 off_lo = packed_lo(k), off_hi = packed_hi(k), off_top = packed_top(k);
    auto fetch = [&](u32 gq) {
#pragma unroll
        for (u32 c = 0; c < 2; ++c) {
            const u64 *b = bank + ((size_t)gq * 2 + c) * w_stride + row;
            xb[c][0] = *reinterpret_cast<const vec_t *>(b + k);
            xb[c][1] = *reinterpret_cast<const vec_t *>(b + km);
        }
#pragma unroll
        for (u32 t = 0; t < TB; ++t)
            if (FULL || bp0 + t < BP) {
                if (PACKED) {
                    // buffer loads: the record's address is workgroup-uniform (scalar registers) and the lanes
                    // add 32-bit offsets, which keeps the 24 addresses of a step out of the vector registers
                    const unsigned char *r = wbytes + (((size_t)(bp0 + t) * GQ + gq) * level + i) * rec;
                    const __amdgpu_buffer_rsrc_t rs =
                        __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char *>(r), 0, (int)rec, 0x00020000);
                    typedef u32 u32x2 __attribute__((ext_vector_type(2)));
                    const u32x2 lo = __builtin_amdgcn_raw_buffer_load_b64(rs, (int)off_lo, 0, 0);
                    wb[t][0] = lo[0];
                    wb[t][1] = lo[1];
                    wb[t][2] = __builtin_amdgcn_raw_buffer_load_b32(rs, (int)off_hi, 0, 0);
                    wb[t][3] = __builtin_amdgcn_raw_buffer_load_b8(rs, (int)off_top, 0, 0);
                } else {
                    wb[t] = *reinterpret_cast<const wvec_t *>(w + ((size_t)(bp0 + t) * GQ + gq) * w_stride + row + k);
                }
            }
    };
    const u32 top_shift = (k & 2) * 2;                           // k is even: bits 0..3 or 4..7 of the byte
    if (accumulate) {
#pragma unroll
        for (u32 t = 0; t < TB; ++t)
            if (FULL || bp0 + t < BP) {
#pragma unroll
                for (u32 c = 0; c < 2; ++c) {
                    const u64 *src = acc + ((size_t)(bp0 + t) * 2 + c) * w_stride + row;
                    const vec_t lo = *reinterpret_cast<const vec_t *>(src + k);
                    const vec_t hi = *reinterpret_cast<const vec_t *>(src + km);
                    a[t][c][0] = (double)lo[0];
                    a[t][c][1] = (double)lo[1];
                    a[t][c][2] = (double)hi[0];
                    a[t][c][3] = (double)hi[1];
                }
            }
    }
    fetch(gq0);
    for (u32 gq = gq0; gq < gq1; ++gq) {
        double x[2][4];
#pragma unroll
        for (u32 c = 0; c < 2; ++c) {
            const u64 r[4] = {xb[c][0][0], xb[c][0][1], xb[c][1][0], xb[c][1][1]};
#pragma unroll
            for (u32 e = 0; e < 4; ++e)
                x[c][e] = __longlong_as_double((long long)(r[e] | 0x4330000000000000ull)) - 4503599627370496.0;
        }
        // the weights leave their load registers as doubles before the next step's loads are issued into them
        double wd[TB][2];
#pragma unroll
        for (u32 t = 0; t < TB; ++t) {
            if (PACKED) {
                const u32 top = wb[t][3] >> top_shift;
                const u32 h0 = 0x43300000u | ((top & 3u) << 16) | (wb[t][2] & 0xffffu);
                const u32 h1 = 0x43300000u | ((top & 12u) << 14) | (wb[t][2] >> 16);
                wd[t][0] = __hiloint2double((int)h0, (int)wb[t][0]) - 4503599627370496.0;
                wd[t][1] = __hiloint2double((int)h1, (int)wb[t][1]) - 4503599627370496.0;
            } else {
                wd[t][0] = __hiloint2double((int)wb[t][1], (int)wb[t][0]);
                wd[t][1] = __hiloint2double((int)wb[t][3], (int)wb[t][2]);
            }
        }
        if (gq + 1 < gq1) fetch(gq + 1);
#pragma unroll
        for (u32 t = 0; t < TB; ++t) {
            if (FULL || bp0 + t < BP) {
                // weight of k serves k and N-1-k; weight of k+1 serves k+1 and N-2-k
                const double wv[4] = {wd[t][0], wd[t][1], wd[t][1], wd[t][0]};
#pragma unroll
                for (u32 c = 0; c < 2; ++c)
#pragma unroll
                    for (u32 e = 0; e < 4; ++e) {
                        const double h = x[c][e] * wv[e];
                        const double l = fma(x[c][e], wv[e], -h);
                        a[t][c][e] += fma(-rint(h * u), q, h) + l;
                    }
            }
        }
        if (((gq - gq0) & 7) == 7) {
#pragma unroll
            for (u32 t = 0; t < TB; ++t)
#pragma unroll
                for (u32 c = 0; c < 2; ++c)
#pragma unroll
                    for (u32 e = 0; e < 4; ++e) a[t][c][e] = fma(-rint(a[t][c][e] * u), q, a[t][c][e]);
        }
    }
#pragma unroll
    for (u32 t = 0; t < TB; ++t) {
        if (FULL || bp0 + t < BP) {
#pragma unroll
            for (u32 c = 0; c < 2; ++c) {
                u64 o[4];
#pragma unroll
                for (u32 e = 0; e < 4; ++e) {
                    double v = fma(-rint(a[t][c][e] * u), q, a[t][c][e]);
                    if (v < 0) v += q;
                    o[e] = (u64)__double_as_longlong(v + 4503599627370496.0) & 0x000fffffffffffffull;
                }
                u64 *dst = acc + ((size_t)(bp0 + t) * 2 + c) * w_stride + row;
                vec_t lo, hi;
                lo[0] = o[0];
                lo[1] = o[1];
                hi[0] = o[2];
                hi[1] = o[3];
                *reinterpret_cast<vec_t *>(dst + k) = lo;
                *reinterpret_cast<vec_t *>(dst + km) = hi;
            }
        }
    }
}

// sym[d] is cleared if polynomial d of the chunk is not fixed by X -> X^-1, i.e. breaks
// c[N-j] == -c[j] for 0 < j < N (which also forces c[N/2] == 0)
__global__ __launch_bounds__(EW_THREADS) void check_real_kernel(const int64_t *__restrict__ coef, u32 *sym, u32 N) {
    const u32 n = blockIdx.x * EW_THREADS + threadIdx.x;
    const int64_t *c = coef + (size_t)blockIdx.y * N;
    if (n == 0) return;
    if (c[N - n] != -c[n]) sym[blockIdx.y] = 0;
}

// rows [rows][N] of canonical residues below 2^50 -> packed half-limb records (first N/2 residues of each row);
// a thread packs four residues
__global__ __launch_bounds__(EW_THREADS) void pack_half_kernel(const u64 *__restrict__ in,
                                                               unsigned char *__restrict__ out, u32 N, u32 cnt) {
    // cnt = N/2 (half records of real diagonals) or N (whole limbs of general ones)
    const u32 k = (blockIdx.x * EW_THREADS + threadIdx.x) * 4;
    if (k >= cnt) return;
    const u64 *src = in + (size_t)blockIdx.y * N + k;
    unsigned char *r = out + (size_t)blockIdx.y * (cnt == N ? 2 : 1) * packed_record_bytes(N);
    uint4 lo;
    uint2 hi;
    const u64 x0 = src[0], x1 = src[1], x2 = src[2], x3 = src[3];
    lo.x = (u32)x0;
    lo.y = (u32)x1;
    lo.z = (u32)x2;
    lo.w = (u32)x3;
    hi.x = (u32)((x0 >> 32) & 0xffff) | ((u32)((x1 >> 32) & 0xffff) << 16);
    hi.y = (u32)((x2 >> 32) & 0xffff) | ((u32)((x3 >> 32) & 0xffff) << 16);
    *reinterpret_cast<uint4 *>(r + packed_lo(k)) = lo;
    *reinterpret_cast<uint2 *>(r + packed_hi(k)) = hi;
    r[packed_top(k)] =
        (unsigned char)(((x0 >> 48) & 3) | (((x1 >> 48) & 3) << 2) | (((x2 >> 48) & 3) << 4) | (((x3 >> 48) & 3) << 6));
}

// half records [rows] -> whole-limb records [rows]: residue k of the second half is residue N-1-k of the first
__global__ __launch_bounds__(EW_THREADS) void widen_half_kernel(const unsigned char *__restrict__ in,
                                                                unsigned char *__restrict__ out, u32 N) {
    const u32 k = (blockIdx.x * EW_THREADS + threadIdx.x) * 4;
    if (k >= N) return;
    const unsigned char *r = in + (size_t)blockIdx.y * packed_record_bytes(N);
    unsigned char *o = out + (size_t)blockIdx.y * 2 * packed_record_bytes(N);
    u32 lo[4], hi[4], top = 0;
#pragma unroll
    for (u32 e = 0; e < 4; ++e) {
        const u32 s = k + e < N / 2 ? k + e : N - 1 - (k + e);
        lo[e] = *reinterpret_cast<const u32 *>(r + packed_lo(s));
        hi[e] = *reinterpret_cast<const unsigned short *>(r + packed_hi(s));
        top |= ((r[packed_top(s)] >> ((s & 3) * 2)) & 3u) << (2 * e);
    }
    *reinterpret_cast<uint4 *>(o + packed_lo(k)) = make_uint4(lo[0], lo[1], lo[2], lo[3]);
    *reinterpret_cast<uint2 *>(o + packed_hi(k)) = make_uint2(hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16));
    o[packed_top(k)] = (unsigned char)top;
}

__global__ __launch_bounds__(EW_THREADS) void fill_u32_kernel(u32 *p, u32 v, u32 n) {
    const u32 i = blockIdx.x * EW_THREADS + threadIdx.x;
    if (i < n) p[i] = v;
}

// the fp64 multiply-accumulate kernels by weight store, FULL left open
template <bool FULL> constexpr auto sym_packed = diag_mac_sym_kernel<MM_TB, true, FULL>;
template <bool FULL> constexpr auto sym_plain = diag_mac_sym_kernel<MM_TB, false, FULL>;
template <bool FULL> constexpr auto gen_packed = diag_mac_kernel<MM_TB, 2, true, FULL>;
template <bool FULL> constexpr auto gen_plain = diag_mac_kernel<MM_TB, 2, false, FULL>;

__global__ __launch_bounds__(MM_THREADS) void diag_mac_int_kernel(const u64 *__restrict__ bank,
                                                                  const u64 *__restrict__ w, u64 *__restrict__ acc,
                                                                  const ModConst *__restrict__ mods, LimbIds limbs,
                                                                  u32 level, u32 N, u32 GQ, u32 BP, u32 flush) {
    const u32 bp0 = blockIdx.x * MM_TB;
    const u32 k = blockIdx.y * MM_THREADS + threadIdx.x;
    const u32 i = limbs.id[blockIdx.z];
    const size_t limb_off = (size_t)i * N + k;
    const size_t w_stride = (size_t)level * N;
    const ModConst m = mods[i];
    u128 a0[MM_TB], a1[MM_TB];
    u64 s0[MM_TB], s1[MM_TB];
#pragma unroll
    for (u32 t = 0; t < MM_TB; ++t) {
        a0[t] = {0, 0};
        a1[t] = {0, 0};
        s0[t] = 0;
        s1[t] = 0;
    }
    u32 pending = 0;
    for (u32 gq = 0; gq < GQ; ++gq) {
        const u64 x0 = bank[((size_t)gq * 2 + 0) * w_stride + limb_off];
        const u64 x1 = bank[((size_t)gq * 2 + 1) * w_stride + limb_off];
#pragma unroll
        for (u32 t = 0; t < MM_TB; ++t) {
            if (bp0 + t < BP) {
                const u64 wv = w[((size_t)(bp0 + t) * GQ + gq) * w_stride + limb_off];
                mac(a0[t], x0, wv);
                mac(a1[t], x1, wv);
            }
        }
        if (++pending == flush) {
#pragma unroll
            for (u32 t = 0; t < MM_TB; ++t) {
                s0[t] = add_mod(s0[t], redc(a0[t], m), m.q);
                s1[t] = add_mod(s1[t], redc(a1[t], m), m.q);
                a0[t] = {0, 0};
                a1[t] = {0, 0};
            }
            pending = 0;
        }
    }
#pragma unroll
    for (u32 t = 0; t < MM_TB; ++t) {
        if (bp0 + t < BP) {
            acc[((size_t)(bp0 + t) * 2 + 0) * w_stride + limb_off] = add_mod(s0[t], redc(a0[t], m), m.q);
            acc[((size_t)(bp0 + t) * 2 + 1) * w_stride + limb_off] = add_mod(s1[t], redc(a1[t], m), m.q);
        }
    }
}

// canonical residues -> the internal form diag_mac_kernel reads (rows [rows][N], limb = row % period)
__global__ __launch_bounds__(EW_THREADS) void to_weight_form_kernel(u64 *data, const ModConst *__restrict__ mods,
                                                                    const ModFp *__restrict__ modf, u32 period,
                                                                    u32 N) {
    const u32 n = blockIdx.x * EW_THREADS + threadIdx.x;
    const u32 row = blockIdx.y;
    const u32 limb = row % period;
    const size_t idx = (size_t)row * N + n;
    const u64 x = data[idx];
    if (modf[limb].ok) {
        data[idx] = (u64)__double_as_longlong((double)x);   // exact: x < 2^50
    } else {
        const ModConst m = mods[limb];
        data[idx] = mont_mul(x, m.r2, m);
    }
}

// delta[pc][i][n] = ((r + h) mod q_l) mod q_i - h mod q_i, r = coefficient-domain last limb, h = floor(q_l/2)
__global__ __launch_bounds__(EW_THREADS) void rescale_delta_kernel(const u64 *__restrict__ r, u64 *__restrict__ out,
                                                                   const ModConst *__restrict__ mods, u32 level,
                                                                   u32 N) {
    const u32 n = blockIdx.x * EW_THREADS + threadIdx.x;
    const u32 pc = blockIdx.y;
    const u64 ql = mods[level - 1].q, h = ql >> 1;
    const u64 rp = add_mod(r[(size_t)pc * N + n], h, ql);
    for (u32 i = 0; i + 1 < level; ++i) {
        const ModConst m = mods[i];
        out[((size_t)pc * (level - 1) + i) * N + n] = sub_mod(reduce_any(rp, m), reduce_any(h, m), m.q);
    }
}

// out[pc][i][k] = (in[pc][i][k] - out[pc][i][k]) * q_l^-1 mod q_i   (out holds NTT(delta) on entry)
__global__ __launch_bounds__(EW_THREADS) void rescale_final_kernel(const u64 *__restrict__ in, u64 *out,
                                                                   const ModConst *__restrict__ mods,
                                                                   const u64 *__restrict__ qlinv, u32 level, u32 N) {
    const u32 k = blockIdx.x * EW_THREADS + threadIdx.x;
    const u32 i = blockIdx.y, pc = blockIdx.z;
    const ModConst m = mods[i];
    const size_t o = ((size_t)pc * (level - 1) + i) * N + k;
    out[o] = mont_mul(sub_mod(in[((size_t)pc * level + i) * N + k], out[o], m.q), qlinv[i], m);
}

// gather rows: dst[pc][n] = src[pc][level-1][n]
__global__ __launch_bounds__(EW_THREADS) void take_last_limb_kernel(const u64 *__restrict__ in, u64 *__restrict__ r,
                                                                    u32 level, u32 N) {
    const u32 n = blockIdx.x * EW_THREADS + threadIdx.x;
    const u32 pc = blockIdx.y;
    r[(size_t)pc * N + n] = in[((size_t)pc * level + level - 1) * N + n];
}

// Arena layout of one ckks_ctpt_matmul call, in words: [key-switch scratch | bank | accumulators | merged sums |
// merged digits].
struct MatmulLayout {
    u32 in_chunk, batch, mg_rots;
    size_t dig_w, tmp_w, ks_w, bank_w, acc_w, u_w, mg_w, yfull_w, t_w;
    size_t total() const { return ks_w + bank_w + acc_w + u_w + mg_w + yfull_w + t_w; }
};

constexpr u32 RESCALE_CHUNK = 64;
static int rescale_rows(ckks_params *P, const u64 *d_in, u32 level, u32 rows, u64 *d_out, u64 *d_r, hipStream_t stream);

static MatmulLayout matmul_layout(const ckks_params *P, const ckks_weights *w, bool merged, bool rescale = true) {
    MatmulLayout l;
    const u32 N = P->N, level = w->level, G = w->G, B = w->B_out, N2 = w->N2;
    const size_t ctw = (size_t)2 * level * N;
    merged = merged && N2 > 1;
    l.in_chunk = std::min<u32>(ROT_BATCH, G);                    // inputs decomposed together
    l.batch = std::min<u32>(ROT_BATCH, std::max(l.in_chunk, B));
    l.dig_w = digits_words(P, level);
    l.tmp_w = (size_t)level * N;
    l.ks_w = l.batch * (l.dig_w + l.tmp_w) + switch_scratch_words(P, level, ROT_BATCH);
    l.bank_w = (size_t)G * w->N1 * ctw;
    l.acc_w = (size_t)B * N2 * ctw;
    l.u_w = merged ? (size_t)B * 2 * (level + P->K) * N : 0;    // extended-basis sums of the giant step
    // merged giant step: the digits of up to MERGE_GROUP rotations of one batch of blocks are held together
    l.mg_rots = merged ? std::min<u32>(MERGE_GROUP, N2 - 1) : 0;
    l.mg_w = (size_t)l.mg_rots * std::min(l.batch, B) * l.dig_w;
    // CKKS_MATMUL_RESCALE: the unrescaled blocks and the dropped limbs in the coefficient domain
    l.yfull_w = rescale ? (size_t)B * ctw : 0;
    l.t_w = rescale ? (size_t)std::max<u32>(l.batch, RESCALE_CHUNK) * 2 * N : 0;
    return l;
}

size_t matmul_scratch_words(const ckks_params *P, const ckks_weights *w, bool merged) {
    return matmul_layout(P, w, merged).total();
}

int expand_plain(const ckks_params *P, u32 level, const int64_t *d_coeffs, u32 count, u64 *d_out, bool mont,
                        hipStream_t stream) {
    const u32 N = P->N;
    LimbIds ids;
    for (u32 i = 0; i < level; ++i) ids.id[i] = (uint8_t)i;
    const u32 per = std::max<u32>(1, 16384 / level);
    for (u32 done = 0; done < count; done += per) {
        const u32 c = std::min(per, count - done);
        u64 *o = d_out + (size_t)done * level * N;
        hipLaunchKernelGGL(expand_coeffs_kernel, dim3(N / EW_THREADS, c), dim3(EW_THREADS), 0, stream,
                           d_coeffs + (size_t)done * N, o, P->d_mod, level, N);
        CKKS_LAUNCH_CHECK("expand_coeffs_kernel");
        int rc = launch_ntt(P, o, ids, level, c * level, false, stream);
        if (rc) return rc;
        if (mont) {
            hipLaunchKernelGGL(to_weight_form_kernel, dim3(N / EW_THREADS, c * level), dim3(EW_THREADS), 0, stream, o,
                               P->d_mod, P->d_modf, level, N);
            CKKS_LAUNCH_CHECK("to_weight_form_kernel");
        }
    }
    return CKKS_OK;
}

}  // namespace ckks

using namespace ckks;

extern "C" {

int ckks_weights_create(const ckks_params_t *P, uint32_t level, uint32_t m, uint32_t C, uint32_t G, uint32_t B_out,
                        uint32_t N1, ckks_weights_t **out) {
    if (!out) {
        set_error("ckks_weights_create: out is null");
        return CKKS_E_INVAL;
    }
    *out = nullptr;
    if (!P) {
        set_error("ckks_weights_create: params is null");
        return CKKS_E_INVAL;
    }
    if (level == 0 || level > P->L) {
        set_error("ckks_weights_create: level %u outside [1,%u]", level, P->L);
        return CKKS_E_LEVEL;
    }
    const u32 n = P->N / 2;
    if (!m || !C || !G || !B_out || !N1 || n % m || (n / m) % C || C % N1) {
        set_error("ckks_weights_create: plan m=%u C=%u G=%u B_out=%u N1=%u does not tile %u slots", m, C, G, B_out, N1,
                  n);
        return CKKS_E_INVAL;
    }
    ckks_weights *w = new ckks_weights();
    w->params = P;
    w->level = level;
    w->m = m;
    w->C = C;
    w->G = G;
    w->B_out = B_out;
    w->N1 = N1;
    w->N2 = C / N1;
    w->block_real.assign((size_t)B_out * G, 1);
    w->block_packed.assign((size_t)B_out * G, 0);
    w->loaded.assign((size_t)B_out * w->N2 * G * N1, 0);
    w->packable = P->N >= 4 * MM_THREADS;
    for (u32 i = 0; i < level; ++i)
        if (P->mod[i] >> 50) w->packable = false;
    // the projection's scratch (bank, accumulators, key-switch workspace) is sized here, in either giant-step
    // order, so that ckks_ctpt_matmul itself neither allocates nor synchronises
    ckks_params *Pm = const_cast<ckks_params *>(P);
    CKKS_HIP(hipDeviceSynchronize());
    int rc = Pm->ensure_scratch(std::max(matmul_scratch_words(P, w, false), matmul_scratch_words(P, w, true)) *
                                    sizeof(u64), nullptr);
    if (rc) {
        delete w;
        return rc;
    }
    *out = w;
    return CKKS_OK;
}

namespace {

constexpr u32 STAGE_DIAGS = 32;

int ensure_full_store(ckks_weights *w) {
    if (w->d_w) return CKKS_OK;
    const size_t words = (size_t)w->B_out * w->N2 * w->G * w->N1 * w->level * w->params->N;
    CKKS_HIP(hipMalloc((void **)&w->d_w, words * sizeof(u64)));
    return CKKS_OK;
}

// whole: the store of whole-limb records (general diagonals) instead of the store of half records (real ones)
int ensure_packed_store(ckks_weights *w, bool whole) {
    const u32 N = w->params->N;
    const size_t recs = (size_t)w->B_out * w->N2 * w->G * w->N1 * w->level;
    if (!whole && !w->d_wp) CKKS_HIP(hipMalloc((void **)&w->d_wp, recs * packed_record_bytes(N)));
    if (whole && !w->d_wpf) CKKS_HIP(hipMalloc((void **)&w->d_wpf, recs * 2 * packed_record_bytes(N)));
    if (!w->d_stage) CKKS_HIP(hipMalloc((void **)&w->d_stage, (size_t)STAGE_DIAGS * w->level * N * sizeof(u64)));
    return CKKS_OK;
}

// A group (b, g) of half records receives a diagonal that is not real: its diagonals move to the whole-limb store.
int widen_group(ckks_weights *w, u32 b, u32 g, hipStream_t stream) {
    int rc = ensure_packed_store(w, true);
    if (rc) return rc;
    const u32 N = w->params->N;
    const size_t rows = (size_t)w->N1 * w->level;            // the records of one (b, p, g)
    for (u32 p = 0; p < w->N2; ++p) {
        const size_t first = ((((size_t)b * w->N2 + p) * w->G + g) * w->N1) * w->level;
        hipLaunchKernelGGL(widen_half_kernel, dim3((N / 4 + EW_THREADS - 1) / EW_THREADS, (u32)rows), dim3(EW_THREADS),
                           0, stream, w->d_wp + first * packed_record_bytes(N),
                           w->d_wpf + first * 2 * packed_record_bytes(N), N);
        CKKS_LAUNCH_CHECK("widen_half_kernel");
    }
    w->block_packed[(size_t)b * w->G + g] = 2;
    return CKKS_OK;
}

}  // namespace

int ckks_weights_set_diagonals(ckks_weights_t *w, uint32_t first, uint32_t count, const int64_t *d_coeffs,
                               void *stream) {
    if (!w || !d_coeffs) {
        set_error("ckks_weights_set_diagonals: null argument");
        return CKKS_E_INVAL;
    }
    const u64 total = (u64)w->B_out * w->N2 * w->G * w->N1;
    if ((u64)first + count > total) {
        set_error("ckks_weights_set_diagonals: [%u,%u) exceeds %llu diagonals", first, first + count,
                  (unsigned long long)total);
        return CKKS_E_INVAL;
    }
    const ckks_params *P = w->params;
    if (count) {
        // real slot vectors are recognised by their coefficients (c[N-j] = -c[j]); an (output block, input group)
        // pair whose diagonals all pass is read through the palindrome kernel.  One host read per chunk: this call is
        // the offline weight-loading step.
        if (w->flag_cap < count) {
            hipFree(w->d_flag);
            w->d_flag = nullptr;
            CKKS_HIP(hipMalloc((void **)&w->d_flag, count * sizeof(u32)));
            w->flag_cap = count;
        }
        hipLaunchKernelGGL(fill_u32_kernel, dim3((count + EW_THREADS - 1) / EW_THREADS), dim3(EW_THREADS), 0,
                           (hipStream_t)stream, w->d_flag, 1u, count);
        hipLaunchKernelGGL(check_real_kernel, dim3(P->N / EW_THREADS, count), dim3(EW_THREADS), 0, (hipStream_t)stream,
                           d_coeffs, w->d_flag, P->N);
        CKKS_LAUNCH_CHECK("check_real_kernel");
        std::vector<u32> flags(count);
        CKKS_HIP(hipMemcpyAsync(flags.data(), w->d_flag, count * sizeof(u32), hipMemcpyDeviceToHost,
                                (hipStream_t)stream));
        CKKS_HIP(hipStreamSynchronize((hipStream_t)stream));
        const u32 N = P->N, level = w->level, N1 = w->N1, G = w->G;
        // the chunk is stored one (b, p, g) run of baby steps at a time; the kind of store is a property of the
        // (output block, input group) pair: packed half records while the pair has seen real diagonals only,
        // packed whole limbs otherwise (chains with a prime of 50 bits or more keep 8-byte words)
        for (u32 lo = first; lo < first + count;) {
            const u32 run = lo / N1;                                   // (b*N2 + p)*G + g
            const u32 g = run % G, b = run / G / w->N2;
            const u32 hi = std::min<u32>(first + count, (run + 1) * N1);
            const size_t grp = (size_t)b * G + g;
            if (w->N1 > 65535 / level) {
                set_error("ckks_weights_set_diagonals: N1 * level = %u exceeds one launch", w->N1 * level);
                return CKKS_E_INVAL;
            }
            bool all_real = true;
            for (u32 d = lo; d < hi; ++d) all_real = all_real && flags[d - first];
            if (!all_real) w->block_real[grp] = 0;
            int rc;
            if (w->packable) {
                const bool whole = !w->block_real[grp];
                if (whole && w->block_packed[grp] == 1 && (rc = widen_group(w, b, g, (hipStream_t)stream))) return rc;
                if ((rc = ensure_packed_store(w, whole))) return rc;
                w->block_packed[grp] = whole ? 2 : 1;
                const size_t recb = (whole ? 2 : 1) * packed_record_bytes(N);
                unsigned char *store = whole ? w->d_wpf : w->d_wp;
                const u32 cnt = whole ? N : N / 2;
                for (u32 d = lo; d < hi; d += STAGE_DIAGS) {
                    const u32 c = std::min(STAGE_DIAGS, hi - d);
                    rc = expand_plain(P, level, d_coeffs + (size_t)(d - first) * N, c, w->d_stage, false,
                                      (hipStream_t)stream);
                    if (rc) return rc;
                    hipLaunchKernelGGL(pack_half_kernel, dim3((cnt / 4 + EW_THREADS - 1) / EW_THREADS, c * level),
                                       dim3(EW_THREADS), 0, (hipStream_t)stream, w->d_stage,
                                       store + (size_t)d * level * recb, N, cnt);
                    CKKS_LAUNCH_CHECK("pack_half_kernel");
                }
            } else {
                if ((rc = ensure_full_store(w))) return rc;
                rc = expand_plain(P, level, d_coeffs + (size_t)(lo - first) * N, hi - lo,
                                  w->d_w + (size_t)lo * level * N, true, (hipStream_t)stream);
                if (rc) return rc;
            }
            std::fill(w->loaded.begin() + lo, w->loaded.begin() + hi, (uint8_t)1);
            lo = hi;
        }
    }
    return CKKS_OK;
}

int ckks_weights_set_bias(ckks_weights_t *w, const int64_t *d_bias_coeffs, uint64_t bias_mul, void *stream) {
    if (!w || !d_bias_coeffs) {
        set_error("ckks_weights_set_bias: null argument");
        return CKKS_E_INVAL;
    }
    const ckks_params *P = w->params;
    if (!w->d_bias) CKKS_HIP(hipMalloc((void **)&w->d_bias, (size_t)w->B_out * w->level * P->N * sizeof(u64)));
    int rc = expand_plain(P, w->level, d_bias_coeffs, w->B_out, w->d_bias, false, (hipStream_t)stream);
    if (rc) return rc;
    hipLaunchKernelGGL(scale_rows_kernel, dim3(P->N / EW_THREADS, w->B_out * w->level), dim3(EW_THREADS), 0,
                       (hipStream_t)stream, w->d_bias, P->d_mod, w->level, P->N, bias_mul);
    CKKS_LAUNCH_CHECK("scale_rows_kernel");
    return CKKS_OK;
}

int ckks_weights_load(const ckks_params_t *P, uint32_t level, uint32_t m, uint32_t C, uint32_t G, uint32_t B_out,
                      uint32_t N1, const int64_t *d_coeffs, const int64_t *d_bias_coeffs, uint64_t bias_mul,
                      void *stream, ckks_weights_t **out) {
    if (!d_coeffs || !out) {
        set_error("ckks_weights_load: null argument");
        return CKKS_E_INVAL;
    }
    ckks_weights_t *w = nullptr;
    int rc = ckks_weights_create(P, level, m, C, G, B_out, N1, &w);
    if (rc) return rc;
    const uint64_t total = (uint64_t)B_out * w->N2 * G * N1;
    // in pieces of whole (b, p) runs, so that one call's device-side checks stay small
    const uint32_t piece = G * N1 * std::max<uint32_t>(1u, 4096u / (G * N1));
    for (uint64_t first = 0; first < total && rc == CKKS_OK; first += piece)
        rc = ckks_weights_set_diagonals(w, (uint32_t)first, (uint32_t)std::min<uint64_t>(piece, total - first),
                                        d_coeffs + first * P->N, stream);
    if (rc == CKKS_OK && d_bias_coeffs) rc = ckks_weights_set_bias(w, d_bias_coeffs, bias_mul, stream);
    if (rc) {
        ckks_weights_destroy(w);
        return rc;
    }
    *out = w;
    return CKKS_OK;
}

void ckks_weights_destroy(ckks_weights_t *w) {
    if (!w) return;
    hipFree(w->d_w);
    hipFree(w->d_wp);
    hipFree(w->d_wpf);
    hipFree(w->d_stage);
    hipFree(w->d_bias);
    hipFree(w->d_flag);
    delete w;
}

int ckks_ctpt_matmul(ckks_params_t *P, const ckks_weights_t *w, const uint64_t *d_ct_x,
                     const ckks_gkey_t *const *baby_keys, const ckks_gkey_t *const *giant_keys,
                     const ckks_gkey_t *conj_key, uint32_t flags, uint64_t *d_ct_y, ckks_counters_t *counters,
                     void *stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    if (!P || !w || !d_ct_x || !d_ct_y) {
        set_error("ckks_ctpt_matmul: null argument");
        return CKKS_E_INVAL;
    }
    if (w->params != P) {
        set_error("ckks_ctpt_matmul: weights belong to another parameter set");
        return CKKS_E_INVAL;
    }
    const u32 N = P->N, level = w->level, G = w->G, B = w->B_out, N1 = w->N1, N2 = w->N2, m = w->m;
    if ((N1 > 1 && !baby_keys) || (N2 > 1 && !giant_keys)) {
        set_error("ckks_ctpt_matmul: key list missing (N1=%u, N2=%u)", N1, N2);
        return CKKS_E_NOKEY;
    }
    // every key is checked before any work is enqueued
    std::vector<int32_t> baby_steps(N1), giant_steps(N2);
    for (u32 q = 0; q < N1; ++q) baby_steps[q] = (int32_t)(q * m);
    for (u32 p = 0; p < N2; ++p) giant_steps[p] = (int32_t)(p * N1 * m);
    std::vector<const ckks_gkey_t *> bk(N1, nullptr);
    for (u32 q = 1; q < N1; ++q) {
        u64 g;
        ckks_galois_elt(P, baby_steps[q], &g);
        bk[q] = baby_keys[q - 1];
        if (g != 1 && (!bk[q] || bk[q]->params != P || bk[q]->galois_elt != g)) {
            set_error("ckks_ctpt_matmul: baby key %u missing or for the wrong Galois element", q);
            return bk[q] ? CKKS_E_INVAL : CKKS_E_NOKEY;
        }
    }
    std::vector<u64> giant_g(N2, 1);
    for (u32 p = 1; p < N2; ++p) {
        ckks_galois_elt(P, giant_steps[p], &giant_g[p]);
        const ckks_gkey_t *k = giant_keys[p - 1];
        if (giant_g[p] != 1 && (!k || k->params != P || k->galois_elt != giant_g[p])) {
            set_error("ckks_ctpt_matmul: giant key %u missing or for the wrong Galois element", p);
            return k ? CKKS_E_INVAL : CKKS_E_NOKEY;
        }
    }
    if (conj_key && (conj_key->params != P || conj_key->galois_elt != 2ull * P->N - 1)) {
        set_error("ckks_ctpt_matmul: conj_key is not a key for conjugation");
        return CKKS_E_INVAL;
    }
    if (flags & ~(uint32_t)(CKKS_MATMUL_MERGED_GIANT | CKKS_MATMUL_RESCALE | CKKS_MATMUL_CONJ_PER_ACC)) {
        set_error("ckks_ctpt_matmul: unknown flags 0x%x", flags);
        return CKKS_E_INVAL;
    }
    const bool conj_per_acc = (flags & CKKS_MATMUL_CONJ_PER_ACC) != 0;
    if (conj_per_acc && !conj_key) {
        set_error("ckks_ctpt_matmul: CKKS_MATMUL_CONJ_PER_ACC needs conj_key");
        return CKKS_E_NOKEY;
    }
    for (size_t d = 0; d < w->loaded.size(); ++d)
        if (!w->loaded[d]) {
            set_error("ckks_ctpt_matmul: diagonal %zu of %zu was never loaded (ckks_weights_set_diagonals)", d,
                      w->loaded.size());
            return CKKS_E_INVAL;
        }
    const uint64_t ntt0 = P->limb_ntts;
    const size_t ctw = (size_t)2 * level * N;
    const bool rescale = (flags & CKKS_MATMUL_RESCALE) != 0;
    if (rescale && level < 2) {
        set_error("ckks_ctpt_matmul: CKKS_MATMUL_RESCALE needs weights at level 2 or above");
        return CKKS_E_LEVEL;
    }
    if (words_overlap(d_ct_x, (size_t)G * ctw, d_ct_y, (size_t)B * (rescale ? ctw - 2 * N : ctw))) {
        set_error("ckks_ctpt_matmul: d_ct_y overlaps d_ct_x");
        return CKKS_E_INVAL;
    }
    const u32 BP = B * N2, GQ = G * N1;
    // persistent buffers of this call live behind the key-switch scratch
    const bool merged = (flags & CKKS_MATMUL_MERGED_GIANT) && N2 > 1;
    const MatmulLayout lay = matmul_layout(P, w, merged, rescale);
    const u32 in_chunk = lay.in_chunk, batch = lay.batch, mg_rots = lay.mg_rots;
    const size_t dig_w = lay.dig_w, tmp_w = lay.tmp_w, ks_w = lay.ks_w, bank_w = lay.bank_w, acc_w = lay.acc_w,
                 u_w = lay.u_w;
    int rc = P->ensure_scratch(lay.total() * sizeof(u64), stream);   // reserved by ckks_weights_create: no-op
    if (rc) return rc;
    u64 *d_digits = (u64 *)P->d_scratch, *d_tmp = d_digits + batch * dig_w, *d_work = d_tmp + batch * tmp_w;
    u64 *d_bank = (u64 *)P->d_scratch + ks_w, *d_acc = d_bank + bank_w;
    // with CKKS_MATMUL_RESCALE the blocks are assembled at the input level in scratch and leave one limb shorter
    u64 *d_out_final = d_ct_y;
    u64 *d_yfull = d_acc + acc_w + u_w + lay.mg_w, *d_t = d_yfull + lay.yfull_w;
    if (rescale) d_ct_y = d_yfull;
    // ModDown and rescale of the merged giant step in one pass, where the fused kernels apply
    const bool fused_rescale = rescale && merged && !conj_key && P->logN == 16 && P->K <= 8 && P->dn_fp &&
                               [&] {
                                   for (u32 i = 0; i < level; ++i)
                                       if (P->mod[i] >> 50) return false;
                                   return level <= 32;
                               }();

    // 1. baby-step bank: the inputs are decomposed once (hoisting); the switches are issued step by step
    //    with the G inputs of one step next to each other, so that they share the reads of that step's key
    std::vector<u64> baby_g(N1, 1);
    for (u32 q = 1; q < N1; ++q) ckks_galois_elt(P, baby_steps[q], &baby_g[q]);
    for (u32 g0 = 0; g0 < G; g0 += in_chunk) {
        const u32 ng = std::min(in_chunk, G - g0);
        const u64 *c1s[ROT_BATCH];
        for (u32 r = 0; r < ng; ++r) c1s[r] = d_ct_x + (size_t)(g0 + r) * ctw + (size_t)level * N;
        rc = decompose(P, c1s, ng, level, d_digits, d_tmp, stream);
        if (rc) return rc;
        SwitchItem items[ROT_BATCH];
        u32 n_it = 0;
        // the inputs of one step stay in one batch; the steps are spread evenly over the batches they need
        u32 n_rot = 0;
        for (u32 q = 0; q < N1; ++q) n_rot += baby_g[q] != 1;
        const u32 per_max = ROT_BATCH / ng, n_batches = (n_rot + per_max - 1) / per_max;
        const u32 per = n_batches ? (n_rot + n_batches - 1) / n_batches : per_max;
        for (u32 q = 0; q < N1; ++q) {
            if (n_it + ng > per * ng) {
                rc = switch_batch(P, level, items, n_it, d_work, stream);
                if (rc) return rc;
                n_it = 0;
            }
            for (u32 r = 0; r < ng; ++r) {
                const u64 *src = d_ct_x + (size_t)(g0 + r) * ctw;
                u64 *dst = d_bank + ((size_t)(g0 + r) * N1 + q) * ctw;
                if (baby_g[q] == 1) {
                    CKKS_HIP(hipMemcpyAsync(dst, src, ctw * sizeof(u64), hipMemcpyDeviceToDevice, stream));
                    continue;
                }
                SwitchItem &it = items[n_it++];
                it.digits = d_digits + (size_t)r * dig_w;
                it.c1 = src + (size_t)level * N;
                it.c0 = src;
                it.key = bk[q]->d_key;
                it.dst = dst;
                it.galois_elt = baby_g[q];
                it.accumulate = 0;
            }
        }
        rc = switch_batch(P, level, items, n_it, d_work, stream);
        if (rc) return rc;
    }
    // 2. diagonal multiply-accumulate
    u64 maxq = 0;
    for (u32 i = 0; i < level; ++i) maxq = std::max(maxq, P->mod[i]);
    const u32 flush = (u32)std::min<u64>(1u << 30, (~0ull) / maxq);
    if (P->prof_on) {
        while (P->prof_ev.size() < P->prof_used + 2) {
            hipEvent_t ev;
            CKKS_HIP(hipEventCreate(&ev));
            P->prof_ev.push_back(ev);
        }
        CKKS_HIP(hipEventRecord(P->prof_ev[P->prof_used], stream));
    }
    {
        LimbIds fp_limbs, int_limbs;
        u32 n_fp = 0, n_int = 0;
        for (u32 i = 0; i < level; ++i) {
            if ((P->mod[i] >> 50) == 0)
                fp_limbs.id[n_fp++] = (uint8_t)i;
            else
                int_limbs.id[n_int++] = (uint8_t)i;
        }
        const dim3 tiles((BP + MM_TB - 1) / MM_TB, N / MM_THREADS);
        // Runs of output blocks whose input groups have the same kinds of store; within a run, one launch per
        // range of input groups of one kind (real diagonals: palindrome kernel on half records; general ones:
        // whole limbs), the later launches adding onto the accumulators of the earlier ones.  Real packing gives
        // one launch; complexified inputs with an odd last group give a general and a real one.
        auto same_kinds = [&](u32 ba, u32 bb) {
            for (u32 g = 0; g < G; ++g)
                if (w->block_real[(size_t)ba * G + g] != w->block_real[(size_t)bb * G + g] ||
                    w->block_packed[(size_t)ba * G + g] != w->block_packed[(size_t)bb * G + g])
                    return false;
            return true;
        };
        for (u32 b0 = 0; n_fp && b0 < B;) {
            u32 b1 = b0 + 1;
            while (b1 < B && same_kinds(b0, b1)) ++b1;
            const u32 bp_first = b0 * N2, bp_count = (b1 - b0) * N2;
            const u64 *wp = w->d_w ? w->d_w + (size_t)bp_first * GQ * level * N : nullptr;
            u64 *ap = d_acc + (size_t)bp_first * ctw;
            const u32 runs = N / (4 * MM_THREADS), gen_runs = N / MM_THREADS / 2;
            // full tiles of MM_TB pairs go to the unguarded kernels, a ragged last tile to the guarded ones
            const u32 full_tiles = bp_count / MM_TB, rag = bp_count % MM_TB ? 1u : 0u;
            for (u32 g0 = 0; g0 < G;) {
                const size_t grp = (size_t)b0 * G + g0;
                u32 g1 = g0 + 1;
                while (g1 < G && w->block_real[grp + (g1 - g0)] == w->block_real[grp] &&
                       w->block_packed[grp + (g1 - g0)] == w->block_packed[grp])
                    ++g1;
                const u32 q0 = g0 * N1, q1 = g1 * N1, add = g0 ? 1u : 0u;
                // 8 (b,p) pairs x 4 coefficients per thread with the next step's loads in flight measured best
#define MM_LAUNCH(KERNEL, RUNS, WPTR)                                                                              \
    do {                                                                                                           \
        if (full_tiles)                                                                                            \
            hipLaunchKernelGGL((KERNEL<true>), dim3(full_tiles, RUNS, n_fp), dim3(MM_THREADS), 0, stream, d_bank,  \
                               WPTR, ap, P->d_modf, fp_limbs, level, N, GQ, bp_count, (RUNS) % 8 == 0 ? 1u : 0u,   \
                               q0, q1, add, 0u);                                                                   \
        if (rag)                                                                                                   \
            hipLaunchKernelGGL((KERNEL<false>), dim3(1, RUNS, n_fp), dim3(MM_THREADS), 0, stream, d_bank, WPTR,    \
                               ap, P->d_modf, fp_limbs, level, N, GQ, bp_count, (RUNS) % 8 == 0 ? 1u : 0u, q0, q1, \
                               add, full_tiles);                                                                   \
    } while (0)
                if (w->block_packed[grp] == 1) {
                    const u64 *pp = reinterpret_cast<const u64 *>(w->d_wp + (size_t)bp_first * GQ * level *
                                                                                packed_record_bytes(N));
                    MM_LAUNCH(sym_packed, runs, pp);
                } else if (w->block_packed[grp] == 2) {
                    const u64 *pp = reinterpret_cast<const u64 *>(w->d_wpf + (size_t)bp_first * GQ * level * 2 *
                                                                                 packed_record_bytes(N));
                    MM_LAUNCH(gen_packed, gen_runs, pp);
                } else if (w->block_real[grp] && N >= 4 * MM_THREADS) {
                    MM_LAUNCH(sym_plain, runs, wp);
                } else {   // 8 accumulators x 2 coefficients per thread (16-byte loads)
                    MM_LAUNCH(gen_plain, gen_runs, wp);
                }
#undef MM_LAUNCH
                g0 = g1;
            }
            b0 = b1;
        }
        if (n_int)
            hipLaunchKernelGGL(diag_mac_int_kernel, dim3(tiles.x, tiles.y, n_int), dim3(MM_THREADS), 0, stream, d_bank,
                               w->d_w, d_acc, P->d_mod, int_limbs, level, N, GQ, BP, flush);
        CKKS_LAUNCH_CHECK("diag_mac_kernel");
    }
    if (P->prof_on) {
        CKKS_HIP(hipEventRecord(P->prof_ev[P->prof_used + 1], stream));
        P->prof_used += 2;
    }
    // 2b. decomplexification in the order Sec. 3.2 displays it: acc_{b,p} += conj(acc_{b,p}) for every accumulator,
    //     before the fold over p.  The switch gathers from its source while it writes, so it goes to the output
    //     area (not yet in use) first.
    if (conj_per_acc) {
        const u32 step = std::min(batch, B);
        for (u32 a0 = 0; a0 < BP; a0 += step) {
            const u32 na = std::min(step, BP - a0);
            SwitchItem items[ROT_BATCH];
            const u64 *c1s[ROT_BATCH];
            for (u32 r = 0; r < na; ++r) c1s[r] = d_acc + (size_t)(a0 + r) * ctw + (size_t)level * N;
            rc = decompose(P, c1s, na, level, d_digits, d_tmp, stream);
            if (rc) return rc;
            for (u32 r = 0; r < na; ++r) {
                items[r].digits = d_digits + (size_t)r * dig_w;
                items[r].c1 = c1s[r];
                items[r].c0 = d_acc + (size_t)(a0 + r) * ctw;
                items[r].key = conj_key->d_key;
                items[r].dst = d_ct_y + (size_t)r * ctw;
                items[r].galois_elt = conj_key->galois_elt;
                items[r].accumulate = 0;
            }
            rc = switch_batch(P, level, items, na, d_work, stream);
            if (rc) return rc;
            hipLaunchKernelGGL(add_rows_kernel, dim3(N / EW_THREADS, na * 2 * level), dim3(EW_THREADS), 0, stream,
                               d_acc + (size_t)a0 * ctw, d_ct_y, P->d_mod, level, N);
            CKKS_LAUNCH_CHECK("add_rows_kernel");
        }
    }
    // 3. giant steps: y_b = acc_{b,0} + sum_p rot(acc_{b,p}).  Where ModDown and rescale are one pass and at least one
    //    rotation needs a key, that pass writes the caller's buffer itself and y_b is assembled where acc_{b,0} lies;
    //    otherwise y_b starts as a copy of acc_{b,0} in the output (or its full-level stand-in).
    std::vector<u32> ps;                                      // giant rotations that are not a full turn
    for (u32 p = 1; p < N2; ++p)
        if (giant_g[p] != 1) ps.push_back(p);
    const bool in_place = fused_rescale && !ps.empty();
    u64 *y_base = in_place ? d_acc : d_ct_y;
    const size_t y_stride = in_place ? (size_t)N2 * ctw : ctw;
    for (u32 b0 = 0; !in_place && b0 < B; b0 += 65535) {
        hipLaunchKernelGGL(copy_blocks_kernel, dim3((u32)(ctw / (2 * EW_THREADS)), 1, std::min<u32>(B - b0, 65535)),
                           dim3(EW_THREADS), 0, stream, d_ct_y + (size_t)b0 * ctw, d_acc + (size_t)b0 * N2 * ctw, ctw,
                           (size_t)N2 * ctw);
        CKKS_LAUNCH_CHECK("copy_blocks_kernel");
    }
    auto add_bias = [&]() -> int {
        for (u32 b0 = 0; w->d_bias && b0 < B; b0 += 65535) {
            hipLaunchKernelGGL(add_bias_kernel, dim3(N / (2 * EW_THREADS), level, std::min<u32>(B - b0, 65535)),
                               dim3(EW_THREADS), 0, stream, y_base + (size_t)b0 * y_stride, y_stride,
                               w->d_bias + (size_t)b0 * level * N, P->d_mod, level, N);
            CKKS_LAUNCH_CHECK("add_bias_kernel");
        }
        return CKKS_OK;
    };
    if (fused_rescale && (rc = add_bias())) return rc;      // the rescale needs the complete dropped limb
    bool any_giant = false;
    u64 *d_u = d_acc + acc_w, *d_mdig = d_u + u_w;
    if (merged) {
        // rotations that are a full turn are plain additions; the others are grouped: the accumulators of a
        // group are decomposed, then one pass sums their switched forms over the extended basis; one ModDown
        // per block follows
        for (u32 p = 1; p < N2; ++p) {
            if (giant_g[p] != 1) continue;
            for (u32 b = 0; b < B; ++b) {
                hipLaunchKernelGGL(add_rows_kernel, dim3(N / EW_THREADS, 2 * level), dim3(EW_THREADS), 0, stream,
                                   y_base + (size_t)b * y_stride, d_acc + ((size_t)b * N2 + p) * ctw, P->d_mod, level, N);
                CKKS_LAUNCH_CHECK("add_rows_kernel");
            }
        }
        for (u32 b0 = 0; !ps.empty() && b0 < B; b0 += batch) {
            const u32 nb = std::min(batch, B - b0);
            u64 *u_b = d_u + (size_t)b0 * 2 * (level + P->K) * N;
            for (size_t i0 = 0; i0 < ps.size(); i0 += mg_rots) {
                MergedRot rots;
                rots.n_rot = (u32)std::min<size_t>(mg_rots, ps.size() - i0);
                // the group's accumulators, rotation-major, are decomposed in as few launches as the batch size
                // allows (their digits fill d_mdig in the same order); the key-switch scratch is idle until the
                // ModDown and holds the coefficient-domain c1 of a whole batch
                const u32 n_dec = rots.n_rot * nb;
                for (u32 c0 = 0; c0 < n_dec; c0 += ROT_BATCH) {
                    const u32 cn = std::min(ROT_BATCH, n_dec - c0);
                    const u64 *c1s[ROT_BATCH];
                    for (u32 c = 0; c < cn; ++c) {
                        const u32 i = (c0 + c) / nb, r = (c0 + c) % nb;
                        c1s[c] = d_acc + ((size_t)(b0 + r) * N2 + ps[i0 + i]) * ctw + (size_t)level * N;
                    }
                    rc = decompose(P, c1s, cn, level, d_mdig + (size_t)c0 * dig_w, d_work, stream);
                    if (rc) return rc;
                }
                for (u32 i = 0; i < rots.n_rot; ++i) {
                    const u32 p = ps[i0 + i];
                    rots.key[i] = giant_keys[p - 1]->d_key;
                    rots.galois_elt[i] = giant_g[p];
                    rots.c0_off[i] = (size_t)p * ctw;
                }
                rc = switch_accumulate_merged(P, level, rots, nb, d_mdig, d_acc + (size_t)b0 * N2 * ctw,
                                              (size_t)N2 * ctw, y_base + (size_t)b0 * y_stride, y_stride, u_b, i0 > 0,
                                              stream);
                if (rc) return rc;
            }
            u64 *dsts[ROT_BATCH];
            for (u32 r = 0; r < nb; ++r) dsts[r] = y_base + (size_t)(b0 + r) * y_stride;
            any_giant = true;
            if (fused_rescale) {
                u64 *outs[ROT_BATCH];
                for (u32 r = 0; r < nb; ++r) outs[r] = d_out_final + (size_t)(b0 + r) * (ctw - 2 * N);
                rc = moddown_rescale(P, level, u_b, dsts, outs, nb, d_work, d_t, stream);
            } else {
                rc = moddown_add(P, level, u_b, dsts, nb, d_work, stream);
            }
            if (rc) return rc;
        }
    }
    for (u32 p = 1; !merged && p < N2; ++p) {
        for (u32 b0 = 0; b0 < B; b0 += batch) {
            const u32 nb = std::min(batch, B - b0);
            if (giant_g[p] == 1) {   // a full turn: plain addition
                for (u32 r = 0; r < nb; ++r) {
                    hipLaunchKernelGGL(add_rows_kernel, dim3(N / EW_THREADS, 2 * level), dim3(EW_THREADS), 0, stream,
                                       d_ct_y + (size_t)(b0 + r) * ctw, d_acc + ((size_t)(b0 + r) * N2 + p) * ctw,
                                       P->d_mod, level, N);
                    CKKS_LAUNCH_CHECK("add_rows_kernel");
                }
                continue;
            }
            SwitchItem items[ROT_BATCH];
            const u64 *c1s[ROT_BATCH];
            for (u32 r = 0; r < nb; ++r) c1s[r] = d_acc + ((size_t)(b0 + r) * N2 + p) * ctw + (size_t)level * N;
            rc = decompose(P, c1s, nb, level, d_digits, d_tmp, stream);
            if (rc) return rc;
            for (u32 r = 0; r < nb; ++r) {
                const u64 *src = d_acc + ((size_t)(b0 + r) * N2 + p) * ctw;
                items[r].digits = d_digits + (size_t)r * dig_w;
                items[r].c1 = src + (size_t)level * N;
                items[r].c0 = src;
                items[r].key = giant_keys[p - 1]->d_key;
                items[r].dst = d_ct_y + (size_t)(b0 + r) * ctw;   // distinct b within a batch: no two items share dst
                items[r].galois_elt = giant_g[p];
                items[r].accumulate = 1;
            }
            rc = switch_batch(P, level, items, nb, d_work, stream);
            if (rc) return rc;
        }
    }
    // 3b. decomplexification: y_b += conj(y_b), one key switch per output block.  The switch gathers from
    //     y_b while it writes, so it goes to the (now free) accumulator area first.
    if (conj_key && !conj_per_acc) {
        for (u32 b0 = 0; b0 < B; b0 += batch) {
            const u32 nb = std::min(batch, B - b0);
            SwitchItem items[ROT_BATCH];
            const u64 *c1s[ROT_BATCH];
            for (u32 r = 0; r < nb; ++r) c1s[r] = d_ct_y + (size_t)(b0 + r) * ctw + (size_t)level * N;
            rc = decompose(P, c1s, nb, level, d_digits, d_tmp, stream);
            if (rc) return rc;
            for (u32 r = 0; r < nb; ++r) {
                items[r].digits = d_digits + (size_t)r * dig_w;
                items[r].c1 = d_ct_y + (size_t)(b0 + r) * ctw + (size_t)level * N;
                items[r].c0 = d_ct_y + (size_t)(b0 + r) * ctw;
                items[r].key = conj_key->d_key;
                items[r].dst = d_acc + (size_t)r * ctw;
                items[r].galois_elt = conj_key->galois_elt;
                items[r].accumulate = 0;
            }
            rc = switch_batch(P, level, items, nb, d_work, stream);
            if (rc) return rc;
            hipLaunchKernelGGL(add_rows_kernel, dim3(N / EW_THREADS, nb * 2 * level), dim3(EW_THREADS), 0, stream,
                               d_ct_y + (size_t)b0 * ctw, d_acc, P->d_mod, level, N);
            CKKS_LAUNCH_CHECK("add_rows_kernel");
        }
    }
    // 4. bias into c0 of every block; 5. rescale, unless the giant step's ModDown already did both
    const bool rescaled = fused_rescale && any_giant;
    if (!fused_rescale && (rc = add_bias())) return rc;
    if (rescale && !rescaled) {
        for (u32 b0 = 0; b0 < B; b0 += RESCALE_CHUNK) {
            const u32 c = std::min(RESCALE_CHUNK, B - b0);
            rc = rescale_rows(P, d_ct_y + (size_t)b0 * ctw, level, 2 * c, d_out_final + (size_t)b0 * (ctw - 2 * N), d_t,
                              stream);
            if (rc) return rc;
        }
    }
    if (counters) {
        u64 ks = 0;
        for (u32 q = 1; q < N1; ++q) {
            u64 g;
            ckks_galois_elt(P, baby_steps[q], &g);
            ks += (g != 1) ? G : 0;
        }
        for (u32 p = 1; p < N2; ++p) ks += (giant_g[p] != 1) ? B : 0;
        if (conj_key) ks += conj_per_acc ? BP : B;
        counters->key_switches = ks;
        counters->ptmuls = (u64)GQ * BP;
        counters->limb_ntts = P->limb_ntts - ntt0;
    }
    return CKKS_OK;
}

}  // extern "C"

namespace ckks {

// rescale of `rows` polynomials (rows = 2 x ciphertexts): d_in [rows][level][N] -> d_out [rows][level-1][N];
// d_r: rows*N words of scratch (the last limbs in the coefficient domain)
static int rescale_rows(ckks_params *P, const u64 *d_in, u32 level, u32 rows, u64 *d_out, u64 *d_r,
                        hipStream_t stream) {
    const u32 N = P->N;
    hipLaunchKernelGGL(take_last_limb_kernel, dim3(N / EW_THREADS, rows), dim3(EW_THREADS), 0, stream, d_in, d_r,
                       level, N);
    CKKS_LAUNCH_CHECK("take_last_limb_kernel");
    LimbIds ids;
    ids.id[0] = (uint8_t)(level - 1);
    int rc = launch_ntt(P, d_r, ids, 1, rows, true, stream);
    if (rc) return rc;
    hipLaunchKernelGGL(rescale_delta_kernel, dim3(N / EW_THREADS, rows), dim3(EW_THREADS), 0, stream, d_r, d_out,
                       P->d_mod, level, N);
    CKKS_LAUNCH_CHECK("rescale_delta_kernel");
    for (u32 i = 0; i + 1 < level; ++i) ids.id[i] = (uint8_t)i;
    rc = launch_ntt(P, d_out, ids, level - 1, rows * (level - 1), false, stream);
    if (rc) return rc;
    hipLaunchKernelGGL(rescale_final_kernel, dim3(N / EW_THREADS, level - 1, rows), dim3(EW_THREADS), 0, stream, d_in,
                       d_out, P->d_mod, P->d_qlinv + (size_t)(level - 1) * P->L, level, N);
    CKKS_LAUNCH_CHECK("rescale_final_kernel");
    return CKKS_OK;
}

// Scratch of ckks_rescale_static: device memory that exists from load time on every GPU the library runs on, so
// that the entry point never allocates.  In host code the array's name is only a stand-in: its device address is
// looked up once per device (static_scratch_ptr) and that pointer is what kernels and copies receive.
constexpr size_t STATIC_SCRATCH_WORDS = (size_t)1 << 20;          // 8 MiB: 16 limb polynomials at N = 2^16
static __device__ __align__(256) u64 scratch[STATIC_SCRATCH_WORDS];
constexpr int MAX_DEVICES = 64;
static u64 *g_static_ptr[MAX_DEVICES] = {};

static int static_scratch_ptr(int device, u64 **out) {
    if (device < 0 || device >= MAX_DEVICES) {
        set_error("ckks_rescale_static: device %d outside [0,%d)", device, MAX_DEVICES);
        return CKKS_E_INVAL;
    }
    if (!g_static_ptr[device]) {
        u64 *ptr = nullptr;
        CKKS_HIP(hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)));
        g_static_ptr[device] = ptr;
    }
    *out = g_static_ptr[device];
    return CKKS_OK;
}

}  // namespace ckks

extern "C" {

int ckks_profile_begin(ckks_params_t *P) {
    if (!P) {
        set_error("ckks_profile_begin: params is null");
        return CKKS_E_INVAL;
    }
    P->prof_on = true;
    P->prof_used = 0;
    return CKKS_OK;
}

int ckks_profile_end(ckks_params_t *P, void *stream, double *total_ms, uint32_t *launches) {
    if (!P || !total_ms || !launches) {
        set_error("ckks_profile_end: null argument");
        return CKKS_E_INVAL;
    }
    CKKS_HIP(hipStreamSynchronize((hipStream_t)stream));
    double sum = 0;
    for (size_t i = 0; i + 1 < P->prof_used; i += 2) {
        float ms = 0;
        CKKS_HIP(hipEventElapsedTime(&ms, P->prof_ev[i], P->prof_ev[i + 1]));
        sum += ms;
    }
    *total_ms = sum;
    *launches = (uint32_t)(P->prof_used / 2);
    P->prof_on = false;
    P->prof_used = 0;
    return CKKS_OK;
}

int ckks_rescale(ckks_params_t *P, const uint64_t *d_ct_in, uint32_t level_in, uint32_t n_ct, uint64_t *d_ct_out,
                 void *stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    if (!P || !d_ct_in || !d_ct_out) {
        set_error("ckks_rescale: null argument");
        return CKKS_E_INVAL;
    }
    if (level_in < 2 || level_in > P->L) {
        set_error("ckks_rescale: level %u outside [2,%u]", level_in, P->L);
        return CKKS_E_LEVEL;
    }
    if (n_ct == 0) return CKKS_OK;
    const u32 N = P->N, level = level_in;
    if (words_overlap(d_ct_in, (size_t)n_ct * 2 * level * N, d_ct_out, (size_t)n_ct * 2 * (level - 1) * N)) {
        set_error("ckks_rescale: d_ct_out overlaps d_ct_in");
        return CKKS_E_INVAL;
    }
    // in slices of RESCALE_CHUNK ciphertexts: the scratch need (one limb polynomial per component) stays within what
    // ckks_params_create reserved
    int rc = P->ensure_scratch((size_t)2 * std::min(n_ct, RESCALE_CHUNK) * N * sizeof(u64), stream);
    if (rc) return rc;
    for (u32 done = 0; done < n_ct; done += RESCALE_CHUNK) {
        const u32 c = std::min(RESCALE_CHUNK, n_ct - done);
        rc = rescale_rows(P, d_ct_in + (size_t)done * 2 * level * N, level, 2 * c,
                          d_ct_out + (size_t)done * 2 * (level - 1) * N, (u64 *)P->d_scratch, stream);
        if (rc) return rc;
    }
    return CKKS_OK;
}

int ckks_rescale_static(ckks_params_t *P, const uint64_t *d_ct_in, uint32_t level_in, uint32_t n_ct,
                        uint64_t *d_ct_out, void *stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    if (!P || !d_ct_in || !d_ct_out) {
        set_error("ckks_rescale_static: null argument");
        return CKKS_E_INVAL;
    }
    if (level_in < 2 || level_in > P->L) {
        set_error("ckks_rescale_static: level %u outside [2,%u]", level_in, P->L);
        return CKKS_E_LEVEL;
    }
    if (n_ct == 0) return CKKS_OK;
    const u32 N = P->N, level = level_in;
    if ((size_t)2 * n_ct * N > STATIC_SCRATCH_WORDS) {
        set_error("ckks_rescale_static: %u ciphertexts of N = %u need %zu words of scratch, the static buffer holds %zu "
                  "(use ckks_rescale)", n_ct, N, (size_t)2 * n_ct * N, STATIC_SCRATCH_WORDS);
        return CKKS_E_INVAL;
    }
    if (words_overlap(d_ct_in, (size_t)n_ct * 2 * level * N, d_ct_out, (size_t)n_ct * 2 * (level - 1) * N)) {
        set_error("ckks_rescale_static: d_ct_out overlaps d_ct_in");
        return CKKS_E_INVAL;
    }
    int device = -1;
    CKKS_HIP(hipGetDevice(&device));
    if (device != P->device) {
        set_error("ckks_rescale_static: current device %d is not the parameter set's device %d", device, P->device);
        return CKKS_E_INVAL;
    }
    u64 *d_r = nullptr;
    int rc = static_scratch_ptr(device, &d_r);
    if (rc) return rc;
    // every word of the buffer this call reads is written first (take_last_limb_kernel): nothing to clear
    return rescale_rows(P, d_ct_in, level, 2 * n_ct, d_ct_out, d_r, stream);
}

}  // extern "C"
