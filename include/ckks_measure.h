/*
 * Measurement interface of libckks_hip.so: NOT part of the product ABI in ckks.h.
 *
 * Benchmarks use these calls to time the byte-moving kernel of the projection in
 * place and to measure what plain streaming kernels and bare modular-product
 * chains reach on the same machine (the ceilings that roofline fractions are
 * also reported against).  Nothing on the path of Sec. 3.2 calls them.
 */
#ifndef CKKS_MEASURE_H
#define CKKS_MEASURE_H

#include "ckks.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Timing of the diagonal multiply-accumulate kernel inside ckks_ctpt_matmul (the kernel that streams
 * the weights, i.e. the path's byte mover): between begin and end every launch is bracketed by HIP
 * events on the call's stream.  end synchronises `stream` and returns the summed kernel time in ms
 * and the number of launches. */
int ckks_profile_begin(ckks_params_t *params);
int ckks_profile_end(ckks_params_t *params, void *stream, double *total_ms, uint32_t *launches);

/* ---- measured ceilings of the machine (what roofline fractions are also reported against) ----
 * Plain streaming kernels and chains of the two modular products the kernels are built from; the caller times
 * them with events on `stream`. */

#define CKKS_PROBE_COPY 0u  /* d_dst[i] = d_src[i]: n_words read and n_words written */
#define CKKS_PROBE_READ 1u  /* n_words of d_src read, at most one word of d_dst written */
#define CKKS_PROBE_WRITE 2u /* n_words of d_dst written (d_src unused) */
int ckks_probe_stream(uint64_t *d_dst, const uint64_t *d_src, uint64_t n_words /* even */, uint32_t mode,
                      void *stream);

#define CKKS_PROBE_INT64 0u /* 64-bit Montgomery product (any prime of the chain) */
#define CKKS_PROBE_FP64 1u  /* exact product in doubles (primes below 2^50) */
#define CKKS_PROBE_INT64_LAZY 2u /* the transforms' integer product: constant factor w stored with floor(w 2^64 / q),
                                    result kept in [0, 2q) along the chain (primes below 2^62) */
/* Every one of n_threads lanes (a multiple of 256) runs four independent chains of `iters` dependent products
 * x <- x * psi mod q, q = prime `limb` (ciphertext primes first, then special), psi its 2N-th root
 * (ckks_params_root), chain c of lane t starting from (4t + c + 1) mod 2^20; d_out[t] (device, n_threads words) is
 * the XOR of the four canonical results, so the caller can check the arithmetic it timed:
 * 4 * n_threads * iters products per launch. */
int ckks_probe_mulmod(const ckks_params_t *params, uint32_t limb, uint32_t kind, uint32_t n_threads, uint32_t iters,
                      uint64_t *d_out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* CKKS_MEASURE_H */
