// Complex-slot encode / decode on the device (Sec. 2.1 Encode / Decode, Sec. 3.1 slot order).
// Slot j of a plaintext m(X) is m(zeta^(5^j)), zeta = exp(i*pi/N).  With e_j = 5^j mod 2N and bin t_j = (e_j - 1)/2,
//   z_j = sum_k (m_k * zeta^k) * exp(+2*pi*i*t_j*k/N)                                  (decode)
//   m_k = (1/N) * Re( zeta^(-k) * sum_t v_t * exp(-2*pi*i*t*k/N) ),  v[t_j] = z_j,  v[N-1-t_j] = conj(z_j)   (encode)
// so both directions are one N-point complex FFT in fp64 plus a twist by the 2N-th roots.  The FFT is
// decimation-in-frequency (natural order in, bit-reversed order out) in one or two passes over LDS tiles; the
// kernels after it read their inputs at bit-reversed positions.  Off the server's hot path.
#include <cmath>

#include "ckks_internal.h"
#include "common_kernels.h"

namespace ckks {

constexpr u32 FFT_THREADS = 256;
constexpr u32 FFT_TILE_LOG = 12;      // 4096 complex doubles = 64 KiB of LDS per workgroup
constexpr u32 ENC_CHUNK = 64;         // vectors transformed per scratch chunk (N = 2^16: 64 MiB)

__device__ __forceinline__ double2 cmul(double2 a, double2 b) {
    return make_double2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x);
}

// Stages whose butterfly partner differs in bit position [lo, lo+c) of the element index, highest bit first.
// A workgroup owns 2^tl elements: the c butterfly bits and tl-c "column" bits, which are the lowest index bits
// (lo >= tl-c; contiguous runs of 2^(tl-c) elements), or, for lo == 0, the bits just above the butterfly bits
// (one contiguous run of 2^tl elements).  w[e] = exp(-2*pi*i*e/N), e < N/2; conj != 0 uses the conjugates.
__global__ __launch_bounds__(FFT_THREADS) void fft_pass_kernel(double2 *__restrict__ data,
                                                               const double2 *__restrict__ w, u32 logN, u32 lo,
                                                               u32 c, u32 tl, u32 conj) {
    __shared__ double2 tile[1u << FFT_TILE_LOG];
    const u32 T = 1u << tl, cb = tl - c, outer = blockIdx.x;
    double2 *v = data + ((size_t)blockIdx.y << logN);
    const u32 ob = lo ? lo - cb : 0;                      // outer bits that sit below the butterfly bits
    const u32 ol = outer & ((1u << ob) - 1u), oh = outer >> ob;
    auto gidx = [&](u32 l) -> u32 {
        if (lo == 0) return (outer << tl) | l;
        const u32 col = l & ((1u << cb) - 1u), a = l >> cb;
        return (((((oh << c) | a) << ob) | ol) << cb) | col;
    };
    for (u32 l = threadIdx.x; l < T; l += FFT_THREADS) tile[l] = v[gidx(l)];
    __syncthreads();
    const u32 ab = lo ? cb : 0;                           // local position of the lowest butterfly bit
    for (u32 t = 0; t < c; ++t) {
        const u32 bp = ab + c - 1 - t, gbp = lo + c - 1 - t, s = logN - 1 - gbp;
        for (u32 u = threadIdx.x; u < T / 2; u += FFT_THREADS) {
            const u32 i0 = ((u >> bp) << (bp + 1)) | (u & ((1u << bp) - 1u)), i1 = i0 | (1u << bp);
            const u32 j = gidx(i0) & ((1u << gbp) - 1u);
            double2 tw = w[(size_t)j << s];
            if (conj) tw.y = -tw.y;
            const double2 a = tile[i0], b = tile[i1];
            tile[i0] = make_double2(a.x + b.x, a.y + b.y);
            tile[i1] = cmul(make_double2(a.x - b.x, a.y - b.y), tw);
        }
        __syncthreads();
    }
    for (u32 l = threadIdx.x; l < T; l += FFT_THREADS) v[gidx(l)] = tile[l];
}

// v[bin_j] = z_j, v[N-1-bin_j] = conj(z_j); real != 0 takes the imaginary parts as zero
__global__ __launch_bounds__(EW_THREADS) void slots_scatter_kernel(const double2 *__restrict__ slots,
                                                                   double2 *__restrict__ v,
                                                                   const u32 *__restrict__ bin, u32 N, u32 real) {
    const u32 j = blockIdx.x * EW_THREADS + threadIdx.x, n = N / 2;
    double2 z = slots[(size_t)blockIdx.y * n + j];
    if (real) z.y = 0.0;
    const u32 t = bin[j];
    double2 *row = v + (size_t)blockIdx.y * N;
    row[t] = z;
    row[N - 1 - t] = make_double2(z.x, -z.y);
}

__device__ __forceinline__ double encode_coeff(const double2 *__restrict__ row, const double2 *__restrict__ twist,
                                               u32 k, u32 logN, double mul) {
    const double2 x = row[__brev(k) >> (32 - logN)], tw = twist[k];
    return rint((x.x * tw.x - x.y * tw.y) * mul);
}

// coefficient k = nearest integer to (scale/N) * Re(zeta^(-k) * X_k).  A real slot vector is fixed by conjugation,
// so its polynomial satisfies m[N-k] = -m[k] and m[N/2] = 0 exactly; real != 0 imposes that on the rounded values
// (the transform gives it only up to rounding).
__global__ __launch_bounds__(EW_THREADS) void encode_final_kernel(const double2 *__restrict__ v,
                                                                  const double2 *__restrict__ twist,
                                                                  int64_t *__restrict__ out, u32 logN, double mul,
                                                                  u32 real) {
    const u32 N = 1u << logN, k = blockIdx.x * EW_THREADS + threadIdx.x;
    const double2 *row = v + ((size_t)blockIdx.y << logN);
    double c;
    if (real && k >= N / 2)
        c = k == N / 2 ? 0.0 : -encode_coeff(row, twist, N - k, logN, mul);
    else
        c = encode_coeff(row, twist, k, logN, mul);
    out[((size_t)blockIdx.y << logN) + k] = (int64_t)c;
}

// centred lift of the residues on one or two primes, times zeta^k
__global__ __launch_bounds__(EW_THREADS) void decode_lift_kernel(const u64 *__restrict__ res,
                                                                 const double2 *__restrict__ twist,
                                                                 double2 *__restrict__ v, u32 N, u32 nlimbs, u64 q0,
                                                                 u64 q1, u64 q0inv_mont, ModConst m1) {
    const u32 k = blockIdx.x * EW_THREADS + threadIdx.x;
    const u64 *r = res + (size_t)blockIdx.y * nlimbs * N;
    const u64 r0 = r[k];
    double x;
    if (nlimbs == 1) {
        x = r0 > q0 / 2 ? -(double)(q0 - r0) : (double)r0;
    } else {
        // x = r0 + q0 * ((r1 - r0) * q0^-1 mod q1), then centred modulo q0*q1
        const u64 d = sub_mod(r[N + k], r0 % q1, q1);
        const u64 t = mont_mul(d, q0inv_mont, m1);
        const unsigned __int128 Q = (unsigned __int128)q0 * q1;
        unsigned __int128 y = (unsigned __int128)q0 * t + r0;
        const bool neg = y > Q / 2;
        if (neg) y = Q - y;
        x = (double)(u64)(y >> 64) * 18446744073709551616.0 + (double)(u64)y;
        if (neg) x = -x;
    }
    const double2 tw = twist[k];
    v[(size_t)blockIdx.y * N + k] = make_double2(x * tw.x, -x * tw.y);
}

__global__ __launch_bounds__(EW_THREADS) void decode_gather_kernel(const double2 *__restrict__ v,
                                                                   const u32 *__restrict__ bin,
                                                                   double2 *__restrict__ slots, u32 logN,
                                                                   double inv_scale) {
    const u32 j = blockIdx.x * EW_THREADS + threadIdx.x, n = 1u << (logN - 1);
    const double2 x = v[((size_t)blockIdx.y << logN) + (__brev(bin[j]) >> (32 - logN))];
    slots[(size_t)blockIdx.y * n + j] = make_double2(x.x * inv_scale, x.y * inv_scale);
}

static int fft_tables(ckks_params *P) {
    if (P->d_fft_w) return CKKS_OK;
    const u32 N = P->N, n = N / 2;
    std::vector<double> w(2 * (size_t)n), tw(2 * (size_t)N);
    const long double pi = 3.14159265358979323846264338327950288L;
    for (u32 e = 0; e < n; ++e) {
        w[2 * e] = (double)cosl(2 * pi * e / N);
        w[2 * e + 1] = (double)-sinl(2 * pi * e / N);
    }
    for (u32 k = 0; k < N; ++k) {
        tw[2 * k] = (double)cosl(pi * k / N);
        tw[2 * k + 1] = (double)-sinl(pi * k / N);
    }
    std::vector<u32> bin(n);
    u64 e = 1;
    for (u32 j = 0; j < n; ++j) {
        bin[j] = (u32)((e - 1) >> 1);
        e = e * 5 % (2ull * N);
    }
    // d_fft_w is set last: it marks the tables as complete
    if (!P->d_fft_twist) CKKS_HIP(hipMalloc(&P->d_fft_twist, tw.size() * sizeof(double)));
    if (!P->d_slot_bin) CKKS_HIP(hipMalloc(&P->d_slot_bin, bin.size() * sizeof(u32)));
    CKKS_HIP(hipMemcpy(P->d_fft_twist, tw.data(), tw.size() * sizeof(double), hipMemcpyHostToDevice));
    CKKS_HIP(hipMemcpy(P->d_slot_bin, bin.data(), bin.size() * sizeof(u32), hipMemcpyHostToDevice));
    double *d_w = nullptr;
    CKKS_HIP(hipMalloc(&d_w, w.size() * sizeof(double)));
    hipError_t e_w = hipMemcpy(d_w, w.data(), w.size() * sizeof(double), hipMemcpyHostToDevice);
    if (e_w != hipSuccess) {
        hipFree(d_w);
        return hip_fail(e_w, "hipMemcpy (transform roots)");
    }
    P->d_fft_w = d_w;
    return CKKS_OK;
}

// in-place transform of `count` vectors of N complex doubles
static int launch_fft(const ckks_params *P, double2 *d_v, u32 count, bool conj, hipStream_t stream) {
    const u32 logN = P->logN;
    const double2 *w = (const double2 *)P->d_fft_w;
    if (logN <= FFT_TILE_LOG) {
        hipLaunchKernelGGL(fft_pass_kernel, dim3(1, count), dim3(FFT_THREADS), 0, stream, d_v, w,
                           logN, 0u, logN, logN, (u32)conj);
        CKKS_LAUNCH_CHECK("fft_pass_kernel");
        return CKKS_OK;
    }
    const u32 tl = FFT_TILE_LOG, tiles = 1u << (logN - tl);
    hipLaunchKernelGGL(fft_pass_kernel, dim3(tiles, count), dim3(FFT_THREADS), 0, stream, d_v, w,
                       logN, 8u, logN - 8, tl, (u32)conj);
    CKKS_LAUNCH_CHECK("fft_pass_kernel (first pass)");
    hipLaunchKernelGGL(fft_pass_kernel, dim3(tiles, count), dim3(FFT_THREADS), 0, stream, d_v, w,
                       logN, 0u, 8u, tl, (u32)conj);
    CKKS_LAUNCH_CHECK("fft_pass_kernel (second pass)");
    return CKKS_OK;
}

static u64 inv_mod_host(u64 a, u64 q) {   // q prime
    unsigned __int128 r = 1, b = a % q;
    for (u64 e = q - 2; e; e >>= 1) {
        if (e & 1) r = r * b % q;
        b = b * b % q;
    }
    return (u64)r;
}

}  // namespace ckks

using namespace ckks;

extern "C" {

int ckks_encode(ckks_params_t *P, const double *d_slots, uint32_t count, double scale, uint32_t flags,
                int64_t *d_coeffs, void *stream_) {
    if (!P || (count && (!d_slots || !d_coeffs))) {
        set_error("ckks_encode: null argument");
        return CKKS_E_INVAL;
    }
    if (!(scale > 0.0) || !std::isfinite(scale) || (flags & ~(uint32_t)CKKS_ENCODE_REAL)) {
        set_error("ckks_encode: scale %g must be positive and finite, flags 0x%x must be known", scale, flags);
        return CKKS_E_INVAL;
    }
    if (count == 0) return CKKS_OK;
    hipStream_t stream = (hipStream_t)stream_;
    int rc = fft_tables(P);
    if (rc) return rc;
    const u32 N = P->N, chunk = std::min<u32>(count, ENC_CHUNK), real = flags & CKKS_ENCODE_REAL;
    rc = P->ensure_scratch((size_t)chunk * N * sizeof(double2), stream);
    if (rc) return rc;
    double2 *v = (double2 *)P->d_scratch;
    for (u32 done = 0; done < count; done += chunk) {
        const u32 c = std::min(chunk, count - done);
        hipLaunchKernelGGL(slots_scatter_kernel, dim3(N / 2 / EW_THREADS, c), dim3(EW_THREADS), 0, stream,
                           (const double2 *)d_slots + (size_t)done * (N / 2), v, P->d_slot_bin, N, real);
        CKKS_LAUNCH_CHECK("slots_scatter_kernel");
        rc = launch_fft(P, v, c, false, stream);
        if (rc) return rc;
        hipLaunchKernelGGL(encode_final_kernel, dim3(N / EW_THREADS, c), dim3(EW_THREADS), 0, stream, v,
                           (const double2 *)P->d_fft_twist, d_coeffs + (size_t)done * N, P->logN, scale / N, real);
        CKKS_LAUNCH_CHECK("encode_final_kernel");
    }
    return CKKS_OK;
}

int ckks_decode(ckks_params_t *P, const uint64_t *d_res, uint32_t nlimbs, uint32_t count, double scale,
                double *d_slots, void *stream_) {
    if (!P || (count && (!d_res || !d_slots))) {
        set_error("ckks_decode: null argument");
        return CKKS_E_INVAL;
    }
    if (nlimbs < 1 || nlimbs > 2 || nlimbs > P->L) {
        set_error("ckks_decode: nlimbs = %u, must be 1 or 2 and at most L = %u", nlimbs, P->L);
        return CKKS_E_INVAL;
    }
    if (!(scale > 0.0) || !std::isfinite(scale)) {
        set_error("ckks_decode: scale %g must be positive and finite", scale);
        return CKKS_E_INVAL;
    }
    if (count == 0) return CKKS_OK;
    hipStream_t stream = (hipStream_t)stream_;
    int rc = fft_tables(P);
    if (rc) return rc;
    const u32 N = P->N, chunk = std::min<u32>(count, ENC_CHUNK);
    rc = P->ensure_scratch((size_t)chunk * N * sizeof(double2), stream);
    if (rc) return rc;
    double2 *v = (double2 *)P->d_scratch;
    const u64 q0 = P->mod[0], q1 = nlimbs > 1 ? P->mod[1] : 0;
    ModConst m1 = nlimbs > 1 ? P->hmod[1] : P->hmod[0];
    u64 q0inv = 0;
    if (nlimbs > 1) {
        const unsigned __int128 inv = inv_mod_host(q0 % q1, q1);
        q0inv = (u64)((inv << 64) % q1);                 // Montgomery form: times 2^64 mod q1
    }
    for (u32 done = 0; done < count; done += chunk) {
        const u32 c = std::min(chunk, count - done);
        hipLaunchKernelGGL(decode_lift_kernel, dim3(N / EW_THREADS, c), dim3(EW_THREADS), 0, stream,
                           d_res + (size_t)done * nlimbs * N, (const double2 *)P->d_fft_twist, v, N, nlimbs, q0, q1,
                           q0inv, m1);
        CKKS_LAUNCH_CHECK("decode_lift_kernel");
        rc = launch_fft(P, v, c, true, stream);
        if (rc) return rc;
        hipLaunchKernelGGL(decode_gather_kernel, dim3(N / 2 / EW_THREADS, c), dim3(EW_THREADS), 0, stream, v,
                           P->d_slot_bin, (double2 *)d_slots + (size_t)done * (N / 2), P->logN, 1.0 / scale);
        CKKS_LAUNCH_CHECK("decode_gather_kernel");
    }
    return CKKS_OK;
}

}  // extern "C"
