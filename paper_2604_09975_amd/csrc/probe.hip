// Measured ceilings of the machine the library runs on: streaming rates of plain copy / read / write kernels and
// the issue rate of the two modular multiplications the kernels are built from.  The benchmark reports its
// roofline fractions against the published peaks and, beside them, against these.
#include "ckks_internal.h"
#include "ntt_device.h"

namespace ckks {

constexpr u32 PROBE_THREADS = 256;

__global__ __launch_bounds__(PROBE_THREADS) void probe_copy_kernel(const ulonglong2 *__restrict__ src,
                                                                   ulonglong2 *__restrict__ dst, size_t n) {
    const size_t stride = (size_t)gridDim.x * PROBE_THREADS;
    for (size_t i = (size_t)blockIdx.x * PROBE_THREADS + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

// every word is read and folded into a sum that is stored only if it hits one fixed value, so the loads stay
__global__ __launch_bounds__(PROBE_THREADS) void probe_read_kernel(const ulonglong2 *__restrict__ src,
                                                                   u64 *__restrict__ sink, size_t n) {
    const size_t stride = (size_t)gridDim.x * PROBE_THREADS;
    u64 s = 0;
    for (size_t i = (size_t)blockIdx.x * PROBE_THREADS + threadIdx.x; i < n; i += stride) {
        const ulonglong2 v = src[i];
        s += v.x ^ v.y;
    }
    if (s == 0x9e3779b97f4a7c15ull) sink[0] = s;
}

__global__ __launch_bounds__(PROBE_THREADS) void probe_write_kernel(ulonglong2 *__restrict__ dst, size_t n) {
    const size_t stride = (size_t)gridDim.x * PROBE_THREADS;
    for (size_t i = (size_t)blockIdx.x * PROBE_THREADS + threadIdx.x; i < n; i += stride)
        dst[i] = make_ulonglong2(i, ~i);
}

// four independent chains of dependent products per lane
__global__ __launch_bounds__(PROBE_THREADS) void probe_mulmod_int_kernel(u64 *__restrict__ out, ModConst m, u64 w,
                                                                         u32 iters) {
    const u32 t = blockIdx.x * PROBE_THREADS + threadIdx.x;
    u64 x[4];
    for (u32 c = 0; c < 4; ++c) x[c] = (t * 4ull + c + 1) % (1u << 20);
    for (u32 i = 0; i < iters; ++i)
#pragma unroll
        for (u32 c = 0; c < 4; ++c) x[c] = mont_mul(x[c], w, m);
    out[t] = x[0] ^ x[1] ^ x[2] ^ x[3];
}

// the product of the integer butterflies: x * w - floor(x * w' / 2^64) * q with w' = floor(w * 2^64 / q), in [0, 2q)
__global__ __launch_bounds__(PROBE_THREADS) void probe_mulmod_lazy_kernel(u64 *__restrict__ out, u64 q, u64 w, u64 ws,
                                                                          u32 iters) {
    const u32 t = blockIdx.x * PROBE_THREADS + threadIdx.x;
    FieldInt f;
    f.q = q;
    f.q2 = 2 * q;
    f.tw = nullptr;
    f.n0 = f.n1 = TwInt{0, 0};
    const TwInt tw{w, ws};
    u64 x[4];
    for (u32 c = 0; c < 4; ++c) x[c] = (t * 4ull + c + 1) % (1u << 20);
    for (u32 i = 0; i < iters; ++i)
#pragma unroll
        for (u32 c = 0; c < 4; ++c) x[c] = f.mul(x[c], tw);
    out[t] = f.out(x[0]) ^ f.out(x[1]) ^ f.out(x[2]) ^ f.out(x[3]);
}

__global__ __launch_bounds__(PROBE_THREADS) void probe_mulmod_fp_kernel(u64 *__restrict__ out, ModFp mf, double w,
                                                                        u32 iters) {
    const u32 t = blockIdx.x * PROBE_THREADS + threadIdx.x;
    FieldFp f;
    f.q = mf.q;
    f.u = mf.u;
    f.n0 = f.n1 = 0.0;
    f.tw = nullptr;
    double x[4];
    for (u32 c = 0; c < 4; ++c) x[c] = (double)((t * 4ull + c + 1) % (1u << 20));
    for (u32 i = 0; i < iters; ++i)
#pragma unroll
        for (u32 c = 0; c < 4; ++c) x[c] = f.mul(x[c], w);     // |result| <= q/2 + small: stays a valid operand
    out[t] = f.out(x[0]) ^ f.out(x[1]) ^ f.out(x[2]) ^ f.out(x[3]);
}

}  // namespace ckks

using namespace ckks;

extern "C" {

int ckks_probe_stream(uint64_t *d_dst, const uint64_t *d_src, uint64_t n_words, uint32_t mode, void *stream) {
    if (mode > CKKS_PROBE_WRITE || (mode != CKKS_PROBE_WRITE && !d_src) || !d_dst || n_words % 2) {
        set_error("ckks_probe_stream: null buffer, odd word count or unknown mode %u", mode);
        return CKKS_E_INVAL;
    }
    if (n_words == 0) return CKKS_OK;
    const size_t n = n_words / 2;
    const u32 grid = (u32)std::min<size_t>((n + PROBE_THREADS - 1) / PROBE_THREADS, 256 * 64);
    if (mode == CKKS_PROBE_COPY)
        hipLaunchKernelGGL(probe_copy_kernel, dim3(grid), dim3(PROBE_THREADS), 0, (hipStream_t)stream,
                           (const ulonglong2 *)d_src, (ulonglong2 *)d_dst, n);
    else if (mode == CKKS_PROBE_READ)
        hipLaunchKernelGGL(probe_read_kernel, dim3(grid), dim3(PROBE_THREADS), 0, (hipStream_t)stream,
                           (const ulonglong2 *)d_src, d_dst, n);
    else
        hipLaunchKernelGGL(probe_write_kernel, dim3(grid), dim3(PROBE_THREADS), 0, (hipStream_t)stream,
                           (ulonglong2 *)d_dst, n);
    CKKS_LAUNCH_CHECK("probe stream kernel");
    return CKKS_OK;
}

int ckks_probe_mulmod(const ckks_params_t *P, uint32_t limb, uint32_t kind, uint32_t n_threads, uint32_t iters,
                      uint64_t *d_out, void *stream) {
    if (!P || !d_out || limb >= P->W || kind > CKKS_PROBE_INT64_LAZY || n_threads == 0 || n_threads % PROBE_THREADS) {
        set_error("ckks_probe_mulmod: bad arguments (limb %u, kind %u, %u threads: a positive multiple of %u)", limb,
                  kind, n_threads, PROBE_THREADS);
        return CKKS_E_INVAL;
    }
    const u64 q = P->mod[limb], w = P->psi[limb];
    if (kind == CKKS_PROBE_FP64) {
        if (q >> 50) {
            set_error("ckks_probe_mulmod: the fp64 product needs a prime below 2^50 (limb %u is not)", limb);
            return CKKS_E_INVAL;
        }
        ModFp mf{};
        mf.q = (double)q;
        mf.u = 1.0 / (double)q;
        const double wc = (double)(w > q / 2 ? (int64_t)w - (int64_t)q : (int64_t)w);
        hipLaunchKernelGGL(probe_mulmod_fp_kernel, dim3(n_threads / PROBE_THREADS), dim3(PROBE_THREADS), 0,
                           (hipStream_t)stream, d_out, mf, wc, iters);
    } else if (kind == CKKS_PROBE_INT64_LAZY) {
        if (q >> 62) {
            set_error("ckks_probe_mulmod: the lazy integer product needs a prime below 2^62 (limb %u is not)", limb);
            return CKKS_E_INVAL;
        }
        const u64 ws = (u64)(((unsigned __int128)w << 64) / q);
        hipLaunchKernelGGL(probe_mulmod_lazy_kernel, dim3(n_threads / PROBE_THREADS), dim3(PROBE_THREADS), 0,
                           (hipStream_t)stream, d_out, q, w, ws, iters);
    } else {
        const ModConst &m = P->hmod[limb];
        const u64 wm = (u64)(((unsigned __int128)w << 64) % q);
        hipLaunchKernelGGL(probe_mulmod_int_kernel, dim3(n_threads / PROBE_THREADS), dim3(PROBE_THREADS), 0,
                           (hipStream_t)stream, d_out, m, wm, iters);
    }
    CKKS_LAUNCH_CHECK("probe mulmod kernel");
    return CKKS_OK;
}

}  // extern "C"
