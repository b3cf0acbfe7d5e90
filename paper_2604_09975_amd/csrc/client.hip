// Key holder's side: secret key upload, Galois key generation, symmetric
// encryption and decryption (Sec. 2.1 KeyGen / Enc / Dec, Sec. 2.3 key
// distribution).  Randomness comes from the caller.  Off the server's hot path.
#include "ckks_internal.h"
#include "common_kernels.h"

struct ckks_secret {
    const ckks_params *params = nullptr;
    ckks::u64 *d_s = nullptr;   // [L+K][N] NTT(s), canonical
};

namespace ckks {

__device__ __forceinline__ u32 galois_index_c(u32 k, u64 g, u32 logN) {
    u32 e = 2u * (__brev(k) >> (32 - logN)) + 1u;
    u32 e2 = (u32)(((u64)e * g) & ((2ull << logN) - 1));
    return __brev((e2 - 1u) >> 1) >> (32 - logN);
}

// int8/int64 coefficients -> residues on the listed limbs; rows [n_rows][N], row r uses limb ids.id[r % period]
template <typename T>
__global__ __launch_bounds__(EW_THREADS) void small_to_residues_kernel(const T *__restrict__ src, u64 *__restrict__ dst,
                                                                       const ModConst *__restrict__ mods, LimbIds ids,
                                                                       u32 period, u32 N) {
    const u32 n = blockIdx.x * EW_THREADS + threadIdx.x;
    const u32 row = blockIdx.y;
    const ModConst m = mods[ids.id[row % period]];
    dst[(size_t)row * N + n] = reduce_signed((int64_t)src[(size_t)(row / period) * N + n], m);
}

// key[j][0][t] = e_hat[j][t] - a[j][t]*s[t] + f(j,t) * target[t],  key[j][1][t] = a[j][t]
// target = sigma_g(s) (Galois key) or s^2 (relin != 0: relinearisation key)
__global__ __launch_bounds__(EW_THREADS) void keygen_kernel(const u64 *__restrict__ s, const u64 *__restrict__ a,
                                                            const u64 *__restrict__ e_hat, u64 *__restrict__ key,
                                                            const ModConst *__restrict__ mods,
                                                            const u64 *__restrict__ pmod, u64 g, u32 W, u32 L,
                                                            u32 alpha, u32 logN, u32 relin) {
    const u32 N = 1u << logN;
    const u32 k = blockIdx.x * EW_THREADS + threadIdx.x;
    const u32 t = blockIdx.y, j = blockIdx.z;
    const ModConst m = mods[t];
    const size_t jt = ((size_t)j * W + t) * N + k;
    const u64 av = a[jt], sv = s[(size_t)t * N + k];
    const u64 as = mont_mul(av, mont_mul(sv, m.r2, m), m);
    u64 v = sub_mod(e_hat[jt], as, m.q);
    if (t < L && t / alpha == j) {
        const u64 sg = relin ? mont_mul(sv, mont_mul(sv, m.r2, m), m) : s[(size_t)t * N + galois_index_c(k, g, logN)];
        v = add_mod(v, mont_mul(sg, pmod[t], m), m.q);   // pmod: P mod q_t in Montgomery form
    }
    key[(((size_t)j * 2 + 0) * W + t) * N + k] = v;
    key[(((size_t)j * 2 + 1) * W + t) * N + k] = av;
}

// ct[0][i] = me_hat[i] - a[i]*s[i], ct[1][i] = a[i]
__global__ __launch_bounds__(EW_THREADS) void encrypt_kernel(const u64 *__restrict__ s, const u64 *__restrict__ a,
                                                             const u64 *__restrict__ me_hat, u64 *__restrict__ ct,
                                                             const ModConst *__restrict__ mods, u32 level, u32 N) {
    const u32 k = blockIdx.x * EW_THREADS + threadIdx.x;
    const u32 i = blockIdx.y;
    const ModConst m = mods[i];
    const size_t o = (size_t)i * N + k;
    const u64 as = mont_mul(a[o], mont_mul(s[o], m.r2, m), m);
    ct[o] = sub_mod(me_hat[o], as, m.q);
    ct[(size_t)level * N + o] = a[o];
}

// out[i] = c0[i] + c1[i]*s[i]
__global__ __launch_bounds__(EW_THREADS) void decrypt_kernel(const u64 *__restrict__ s, const u64 *__restrict__ ct,
                                                             u64 *__restrict__ out, const ModConst *__restrict__ mods,
                                                             u32 level, u32 N) {
    const u32 k = blockIdx.x * EW_THREADS + threadIdx.x;
    const u32 i = blockIdx.y;
    const ModConst m = mods[i];
    const size_t o = (size_t)i * N + k;
    const u64 cs = mont_mul(ct[(size_t)level * N + o], mont_mul(s[o], m.r2, m), m);
    out[o] = add_mod(ct[o], cs, m.q);
}

// m + e as int64 (both small)
__global__ __launch_bounds__(EW_THREADS) void add_i64_kernel(const int64_t *a, const int64_t *b, int64_t *o) {
    const size_t n = (size_t)blockIdx.x * EW_THREADS + threadIdx.x;
    o[n] = a[n] + b[n];
}

}  // namespace ckks

using namespace ckks;

extern "C" {

int ckks_client_secret_load(const ckks_params_t *P, const int8_t *s, void *stream_, ckks_secret_t **out) {
    hipStream_t stream = (hipStream_t)stream_;
    if (!out) {
        set_error("ckks_client_secret_load: out is null");
        return CKKS_E_INVAL;
    }
    *out = nullptr;
    if (!P || !s) {
        set_error("ckks_client_secret_load: null argument");
        return CKKS_E_INVAL;
    }
    for (u32 i = 0; i < P->N; ++i)
        if (s[i] < -1 || s[i] > 1) {
            set_error("ckks_client_secret_load: coefficient %u is not ternary", i);
            return CKKS_E_INVAL;
        }
    int8_t *d_raw = nullptr;
    CKKS_HIP(hipMalloc((void **)&d_raw, P->N));
    ckks_secret *S = new ckks_secret();
    S->params = P;
    hipError_t e = hipMalloc((void **)&S->d_s, (size_t)P->W * P->N * sizeof(u64));
    if (e == hipSuccess) e = hipMemcpyAsync(d_raw, s, P->N, hipMemcpyHostToDevice, stream);
    if (e != hipSuccess) {
        hipFree(d_raw);
        hipFree(S->d_s);
        delete S;
        return hip_fail(e, "secret upload");
    }
    LimbIds ids;
    for (u32 t = 0; t < P->W; ++t) ids.id[t] = (uint8_t)t;
    hipLaunchKernelGGL(small_to_residues_kernel<int8_t>, dim3(P->N / EW_THREADS, P->W), dim3(EW_THREADS), 0, stream,
                       d_raw, S->d_s, P->d_mod, ids, P->W, P->N);
    int rc = launch_ntt(P, S->d_s, ids, P->W, P->W, false, stream);
    hipStreamSynchronize(stream);
    hipFree(d_raw);
    if (rc) {
        ckks_client_secret_destroy(S);
        return rc;
    }
    *out = S;
    return CKKS_OK;
}

void ckks_client_secret_destroy(ckks_secret_t *S) {
    if (!S) return;
    hipFree(S->d_s);
    delete S;
}

static int keygen_common(ckks_params_t *P, const ckks_secret_t *S, uint64_t g, const uint64_t *d_a,
                         const int64_t *d_e, uint64_t *d_key, void *stream_, uint32_t relin);

int ckks_client_galois_keygen(ckks_params_t *P, const ckks_secret_t *S, uint64_t g, const uint64_t *d_a,
                              const int64_t *d_e, uint64_t *d_key, void *stream) {
    return keygen_common(P, S, g, d_a, d_e, d_key, stream, 0);
}

int ckks_client_relin_keygen(ckks_params_t *P, const ckks_secret_t *S, const uint64_t *d_a, const int64_t *d_e,
                             uint64_t *d_key, void *stream) {
    return keygen_common(P, S, 1, d_a, d_e, d_key, stream, 1);
}

static int keygen_common(ckks_params_t *P, const ckks_secret_t *S, uint64_t g, const uint64_t *d_a,
                         const int64_t *d_e, uint64_t *d_key, void *stream_, uint32_t relin) {
    hipStream_t stream = (hipStream_t)stream_;
    if (!P || !S || !d_a || !d_e || !d_key || S->params != P) {
        set_error("ckks_client_galois_keygen: null argument or secret of another parameter set");
        return CKKS_E_INVAL;
    }
    if (P->K == 0 || !(g & 1) || g >= 2ull * P->N) {
        set_error("ckks_client_galois_keygen: no special primes, or %llu is not a Galois element",
                  (unsigned long long)g);
        return CKKS_E_INVAL;
    }
    const u32 N = P->N, W = P->W, dnum = P->dnum;
    // scratch: e_hat [dnum][W][N] and P mod q_t table [W]
    int rc = P->ensure_scratch(((size_t)dnum * W * N + W) * sizeof(u64), stream);
    if (rc) return rc;
    u64 *d_ehat = (u64 *)P->d_scratch, *d_pmod = d_ehat + (size_t)dnum * W * N;
    std::vector<u64> pmod(W, 0);
    for (u32 t = 0; t < P->L; ++t) {
        unsigned __int128 v = 1;
        for (u32 k = 0; k < P->K; ++k) v = v * (P->mod[P->L + k] % P->mod[t]) % P->mod[t];
        pmod[t] = (u64)(v * P->hmod[t].one % P->mod[t]);
    }
    CKKS_HIP(hipMemcpyAsync(d_pmod, pmod.data(), W * sizeof(u64), hipMemcpyHostToDevice, stream));
    CKKS_HIP(hipStreamSynchronize(stream));   // pmod is a stack-lifetime host buffer
    LimbIds ids;
    for (u32 t = 0; t < W; ++t) ids.id[t] = (uint8_t)t;
    hipLaunchKernelGGL(small_to_residues_kernel<int64_t>, dim3(N / EW_THREADS, dnum * W), dim3(EW_THREADS), 0, stream,
                       d_e, d_ehat, P->d_mod, ids, W, N);
    CKKS_LAUNCH_CHECK("small_to_residues_kernel");
    rc = launch_ntt(P, d_ehat, ids, W, dnum * W, false, stream);
    if (rc) return rc;
    hipLaunchKernelGGL(keygen_kernel, dim3(N / EW_THREADS, W, dnum), dim3(EW_THREADS), 0, stream, S->d_s, d_a, d_ehat,
                       d_key, P->d_mod, d_pmod, g, W, P->L, P->alpha, P->logN, relin);
    CKKS_LAUNCH_CHECK("keygen_kernel");
    return CKKS_OK;
}

int ckks_client_encrypt(ckks_params_t *P, const ckks_secret_t *S, uint32_t level, const int64_t *d_m,
                        const uint64_t *d_a, const int64_t *d_e, uint64_t *d_ct, void *stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    if (!P || !S || !d_m || !d_a || !d_e || !d_ct || S->params != P) {
        set_error("ckks_client_encrypt: null argument or secret of another parameter set");
        return CKKS_E_INVAL;
    }
    if (level == 0 || level > P->L) {
        set_error("ckks_client_encrypt: level %u outside [1,%u]", level, P->L);
        return CKKS_E_LEVEL;
    }
    const u32 N = P->N;
    int rc = P->ensure_scratch(((size_t)level * N + N) * sizeof(u64), stream);
    if (rc) return rc;
    u64 *d_me = (u64 *)P->d_scratch;
    int64_t *d_sum = (int64_t *)(d_me + (size_t)level * N);
    hipLaunchKernelGGL(add_i64_kernel, dim3(N / EW_THREADS), dim3(EW_THREADS), 0, stream, d_m, d_e, d_sum);
    LimbIds ids;
    for (u32 i = 0; i < level; ++i) ids.id[i] = (uint8_t)i;
    hipLaunchKernelGGL(small_to_residues_kernel<int64_t>, dim3(N / EW_THREADS, level), dim3(EW_THREADS), 0, stream,
                       d_sum, d_me, P->d_mod, ids, level, N);
    CKKS_LAUNCH_CHECK("small_to_residues_kernel");
    rc = launch_ntt(P, d_me, ids, level, level, false, stream);
    if (rc) return rc;
    hipLaunchKernelGGL(encrypt_kernel, dim3(N / EW_THREADS, level), dim3(EW_THREADS), 0, stream, S->d_s, d_a, d_me,
                       d_ct, P->d_mod, level, N);
    CKKS_LAUNCH_CHECK("encrypt_kernel");
    return CKKS_OK;
}

int ckks_client_decrypt(ckks_params_t *P, const ckks_secret_t *S, const uint64_t *d_ct, uint32_t level,
                        uint32_t nlimbs, uint64_t *d_out, void *stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    if (!P || !S || !d_ct || !d_out || S->params != P) {
        set_error("ckks_client_decrypt: null argument or secret of another parameter set");
        return CKKS_E_INVAL;
    }
    if (level == 0 || level > P->L || nlimbs == 0 || nlimbs > level) {
        set_error("ckks_client_decrypt: level %u / nlimbs %u out of range", level, nlimbs);
        return CKKS_E_LEVEL;
    }
    const u32 N = P->N;
    hipLaunchKernelGGL(decrypt_kernel, dim3(N / EW_THREADS, nlimbs), dim3(EW_THREADS), 0, stream, S->d_s, d_ct, d_out,
                       P->d_mod, level, N);
    CKKS_LAUNCH_CHECK("decrypt_kernel");
    LimbIds ids;
    for (u32 i = 0; i < nlimbs; ++i) ids.id[i] = (uint8_t)i;
    return launch_ntt(P, d_out, ids, nlimbs, nlimbs, true, stream);
}

}  // extern "C"
