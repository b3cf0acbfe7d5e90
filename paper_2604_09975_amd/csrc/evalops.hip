// Elementwise homomorphic primitives of Table 1 (add, ptmul), ModSwitchToNext (Sec. 5.4) and the restricted
// rotation RotFirst of App. A.1.  All of them stream their operands once: HBM-bound.
#include <algorithm>
#include <vector>

#include "ckks_internal.h"
#include "common_kernels.h"
#include "modarith.h"

namespace ckks {

// out[row][n] = a[row][n] + b[row][n] mod limb (row % period)
__global__ __launch_bounds__(EW_THREADS) void add_ct_kernel(const u64 *__restrict__ a, const u64 *__restrict__ b,
                                                            u64 *__restrict__ out, const ModConst *__restrict__ mods,
                                                            u32 period, u32 N) {
    const u32 n = (blockIdx.x * EW_THREADS + threadIdx.x) * 2;
    const u32 row = blockIdx.y;
    const u64 q = mods[row % period].q;
    const size_t idx = (size_t)row * N + n;
    const ulonglong2 x = *(const ulonglong2 *)(a + idx), y = *(const ulonglong2 *)(b + idx);
    ulonglong2 r;
    r.x = add_mod(x.x, y.x, q);
    r.y = add_mod(x.y, y.y, q);
    *(ulonglong2 *)(out + idx) = r;
}

// out[comp][i][n] = ct[comp][i][n] * pt[i][n] mod q_i (all canonical)
__global__ __launch_bounds__(EW_THREADS) void ptmul_kernel(const u64 *__restrict__ ct, const u64 *__restrict__ pt,
                                                           u64 *__restrict__ out, const ModConst *__restrict__ mods,
                                                           u32 level, u32 N) {
    const u32 n = (blockIdx.x * EW_THREADS + threadIdx.x) * 2;
    const u32 i = blockIdx.y;
    const ModConst m = mods[i];
    const ulonglong2 w = *(const ulonglong2 *)(pt + (size_t)i * N + n);
    const u64 w0 = mont_mul(w.x, m.r2, m), w1 = mont_mul(w.y, m.r2, m);
    for (u32 comp = 0; comp < 2; ++comp) {
        const size_t idx = ((size_t)comp * level + i) * N + n;
        const ulonglong2 x = *(const ulonglong2 *)(ct + idx);
        ulonglong2 r;
        r.x = mont_mul(x.x, w0, m);
        r.y = mont_mul(x.y, w1, m);
        *(ulonglong2 *)(out + idx) = r;
    }
}

// out = r1 (.) a + r2 (.) b  for one ciphertext pair (the two rotated copies of RotFirst)
__global__ __launch_bounds__(EW_THREADS) void masked_sum_kernel(const u64 *__restrict__ r1, const u64 *__restrict__ r2,
                                                                const u64 *__restrict__ pa, const u64 *__restrict__ pb,
                                                                u64 *__restrict__ out,
                                                                const ModConst *__restrict__ mods, u32 level, u32 N) {
    const u32 n = (blockIdx.x * EW_THREADS + threadIdx.x) * 2;
    const u32 i = blockIdx.y;
    const ModConst m = mods[i];
    const ulonglong2 a = *(const ulonglong2 *)(pa + (size_t)i * N + n), b = *(const ulonglong2 *)(pb + (size_t)i * N + n);
    const u64 a0 = mont_mul(a.x, m.r2, m), a1 = mont_mul(a.y, m.r2, m);
    const u64 b0 = mont_mul(b.x, m.r2, m), b1 = mont_mul(b.y, m.r2, m);
    for (u32 comp = 0; comp < 2; ++comp) {
        const size_t idx = ((size_t)comp * level + i) * N + n;
        const ulonglong2 x = *(const ulonglong2 *)(r1 + idx), y = *(const ulonglong2 *)(r2 + idx);
        ulonglong2 r;
        r.x = add_mod(mont_mul(x.x, a0, m), mont_mul(y.x, b0, m), m.q);
        r.y = add_mod(mont_mul(x.y, a1, m), mont_mul(y.y, b1, m), m.q);
        *(ulonglong2 *)(out + idx) = r;
    }
}

// out[pc][i][n] = in[pc][i][n], i < level-1
__global__ __launch_bounds__(EW_THREADS) void drop_limb_kernel(const u64 *__restrict__ in, u64 *__restrict__ out,
                                                               u32 level, u32 N) {
    const u32 n = (blockIdx.x * EW_THREADS + threadIdx.x) * 2;
    const u32 i = blockIdx.y, pc = blockIdx.z;
    *(ulonglong2 *)(out + ((size_t)pc * (level - 1) + i) * N + n) =
        *(const ulonglong2 *)(in + ((size_t)pc * level + i) * N + n);
}

static int check_level(const ckks_params *P, u32 level, u32 lo, const char *who) {
    if (level < lo || level > P->L) {
        set_error("%s: level %u outside [%u,%u]", who, level, lo, P->L);
        return CKKS_E_LEVEL;
    }
    return CKKS_OK;
}

}  // namespace ckks

using namespace ckks;

// masks: 2*n_out device pointers, [level][N] each
static int shift_bank(ckks_params_t *P, const uint64_t *d_ct_in, uint32_t level, uint32_t n_out, const int32_t *steps,
                      const ckks_gkey_t *const *keys, const uint64_t *const *masks, uint64_t *d_ct_out,
                      hipStream_t stream) {
    int rc;
    const u32 N = P->N;
    const size_t ctw = (size_t)2 * level * N;
    // every key is checked before any work is enqueued
    std::vector<u64> gel(2 * (size_t)n_out);
    bool any = false;
    for (size_t s = 0; s < gel.size(); ++s) {
        ckks_galois_elt(P, steps[s], &gel[s]);
        if (gel[s] == 1) continue;
        any = true;
        if (P->K == 0) {
            set_error("ckks_shift_bank: parameter set has no special primes");
            return CKKS_E_INVAL;
        }
        if (!keys[s]) {
            set_error("ckks_shift_bank: step %d (output %zu, term %zu) has no key", steps[s], s / 2, s % 2);
            return CKKS_E_NOKEY;
        }
        if (keys[s]->params != P || keys[s]->galois_elt != gel[s]) {
            set_error("ckks_shift_bank: key of output %zu, term %zu is for another Galois element", s / 2, s % 2);
            return CKKS_E_INVAL;
        }
    }
    if (words_overlap(d_ct_in, ctw, d_ct_out, (size_t)n_out * ctw)) {
        set_error("ckks_shift_bank: d_ct_out overlaps d_ct_in");
        return CKKS_E_INVAL;
    }
    // scratch: rotated copies of one chunk of outputs, then the hoisted digits and the switch workspace
    const u32 chunk_out = ROT_BATCH / 2;
    const size_t rot_w = (size_t)ROT_BATCH * ctw, dig_w = digits_words(P, level), tmp_w = (size_t)level * N;
    rc = P->ensure_scratch((rot_w + dig_w + tmp_w + switch_scratch_words(P, level, ROT_BATCH)) * sizeof(u64), stream);
    if (rc) return rc;
    u64 *d_rot = (u64 *)P->d_scratch, *d_digits = d_rot + rot_w, *d_tmp = d_digits + dig_w, *d_work = d_tmp + tmp_w;
    if (any) {
        const u64 *c1 = d_ct_in + (size_t)level * N;
        rc = decompose(P, &c1, 1, level, d_digits, d_tmp, stream);
        if (rc) return rc;
    }
    for (u32 o0 = 0; o0 < n_out; o0 += chunk_out) {
        const u32 no = std::min(chunk_out, n_out - o0);
        SwitchItem items[ROT_BATCH];
        const u64 *term[ROT_BATCH];
        u32 n_it = 0;
        for (u32 s = 0; s < 2 * no; ++s) {
            const size_t gs = (size_t)2 * o0 + s;
            if (gel[gs] == 1) {       // the input itself
                term[s] = d_ct_in;
                continue;
            }
            term[s] = d_rot + (size_t)s * ctw;
            SwitchItem &it = items[n_it++];
            it.digits = d_digits;
            it.c1 = d_ct_in + (size_t)level * N;
            it.c0 = d_ct_in;
            it.key = keys[gs]->d_key;
            it.dst = d_rot + (size_t)s * ctw;
            it.galois_elt = gel[gs];
            it.accumulate = 0;
        }
        rc = switch_batch(P, level, items, n_it, d_work, stream);
        if (rc) return rc;
        for (u32 o = 0; o < no; ++o) {
            hipLaunchKernelGGL(masked_sum_kernel, dim3(N / (2 * EW_THREADS), level), dim3(EW_THREADS), 0, stream,
                               term[2 * o], term[2 * o + 1], masks[2 * (o0 + o)], masks[2 * (o0 + o) + 1],
                               d_ct_out + (size_t)(o0 + o) * ctw, P->d_mod, level, N);
            CKKS_LAUNCH_CHECK("masked_sum_kernel");
        }
    }
    return CKKS_OK;
}

extern "C" {

int ckks_plain_expand(const ckks_params_t *P, uint32_t level, const int64_t *d_coeffs, uint32_t count,
                      uint64_t *d_out, void *stream) {
    if (!P || (count && (!d_coeffs || !d_out))) {
        set_error("ckks_plain_expand: null argument");
        return CKKS_E_INVAL;
    }
    int rc = check_level(P, level, 1, "ckks_plain_expand");
    if (rc || count == 0) return rc;
    return expand_plain(P, level, d_coeffs, count, d_out, false, (hipStream_t)stream);
}

int ckks_add(const ckks_params_t *P, const uint64_t *d_ct_a, const uint64_t *d_ct_b, uint32_t level, uint32_t n_ct,
             uint64_t *d_ct_out, void *stream) {
    if (!P || (n_ct && (!d_ct_a || !d_ct_b || !d_ct_out))) {
        set_error("ckks_add: null argument");
        return CKKS_E_INVAL;
    }
    int rc = check_level(P, level, 1, "ckks_add");
    if (rc || n_ct == 0) return rc;
    const size_t rows = (size_t)n_ct * 2 * level;
    for (size_t done = 0; done < rows;) {          // grid.y is limited to 65535 rows; chunks keep the limb phase
        const u32 c = (u32)std::min<size_t>(rows - done, (65535 / level) * level);
        hipLaunchKernelGGL(add_ct_kernel, dim3(P->N / (2 * EW_THREADS), c), dim3(EW_THREADS), 0, (hipStream_t)stream,
                           d_ct_a + done * P->N, d_ct_b + done * P->N, d_ct_out + done * P->N, P->d_mod, level, P->N);
        CKKS_LAUNCH_CHECK("add_ct_kernel");
        done += c;
    }
    return CKKS_OK;
}

int ckks_ptmul(const ckks_params_t *P, const uint64_t *d_ct, uint32_t level, const uint64_t *d_plain,
               uint64_t *d_ct_out, void *stream) {
    if (!P || !d_ct || !d_plain || !d_ct_out) {
        set_error("ckks_ptmul: null argument");
        return CKKS_E_INVAL;
    }
    int rc = check_level(P, level, 1, "ckks_ptmul");
    if (rc) return rc;
    hipLaunchKernelGGL(ptmul_kernel, dim3(P->N / (2 * EW_THREADS), level), dim3(EW_THREADS), 0, (hipStream_t)stream,
                       d_ct, d_plain, d_ct_out, P->d_mod, level, P->N);
    CKKS_LAUNCH_CHECK("ptmul_kernel");
    return CKKS_OK;
}

int ckks_mod_switch_to_next(const ckks_params_t *P, const uint64_t *d_ct_in, uint32_t level_in, uint32_t n_ct,
                            uint64_t *d_ct_out, void *stream) {
    if (!P || (n_ct && (!d_ct_in || !d_ct_out))) {
        set_error("ckks_mod_switch_to_next: null argument");
        return CKKS_E_INVAL;
    }
    int rc = check_level(P, level_in, 2, "ckks_mod_switch_to_next");
    if (rc || n_ct == 0) return rc;
    if (words_overlap(d_ct_in, (size_t)n_ct * 2 * level_in * P->N, d_ct_out, (size_t)n_ct * 2 * (level_in - 1) * P->N)) {
        set_error("ckks_mod_switch_to_next: d_ct_out overlaps d_ct_in");
        return CKKS_E_INVAL;
    }
    if (2 * n_ct > 65535) {
        set_error("ckks_mod_switch_to_next: %u ciphertexts exceed one launch", n_ct);
        return CKKS_E_INVAL;
    }
    hipLaunchKernelGGL(drop_limb_kernel, dim3(P->N / (2 * EW_THREADS), level_in - 1, 2 * n_ct), dim3(EW_THREADS), 0,
                       (hipStream_t)stream, d_ct_in, d_ct_out, level_in, P->N);
    CKKS_LAUNCH_CHECK("drop_limb_kernel");
    return CKKS_OK;
}

int ckks_shift_bank(ckks_params_t *P, const uint64_t *d_ct_in, uint32_t level, uint32_t n_out, const int32_t *steps,
                    const ckks_gkey_t *const *keys, const uint64_t *d_masks, uint64_t *d_ct_out, void *stream) {
    if (!P || !d_ct_in || (n_out && (!steps || !keys || !d_masks || !d_ct_out))) {
        set_error("ckks_shift_bank: null argument");
        return CKKS_E_INVAL;
    }
    int rc = check_level(P, level, 1, "ckks_shift_bank");
    if (rc || n_out == 0) return rc;
    std::vector<const uint64_t *> masks(2 * (size_t)n_out);
    for (size_t s = 0; s < masks.size(); ++s) masks[s] = d_masks + s * (size_t)level * P->N;
    return shift_bank(P, d_ct_in, level, n_out, steps, keys, masks.data(), d_ct_out, (hipStream_t)stream);
}

int ckks_rot_first(ckks_params_t *P, const uint64_t *d_ct_in, uint32_t level, uint32_t L_slots, uint32_t tau,
                   const ckks_gkey_t *key_tau, const ckks_gkey_t *key_wrap, const uint64_t *d_mask_a,
                   const uint64_t *d_mask_b, uint64_t *d_ct_out, void *stream_) {
    if (!P || !d_ct_in || !d_mask_a || !d_mask_b || !d_ct_out) {
        set_error("ckks_rot_first: null argument");
        return CKKS_E_INVAL;
    }
    int rc = check_level(P, level, 1, "ckks_rot_first");
    if (rc) return rc;
    const u32 N = P->N, n = N / 2;
    if (L_slots == 0 || L_slots > n) {
        set_error("ckks_rot_first: L = %u outside [1,%u]", L_slots, n);
        return CKKS_E_INVAL;
    }
    const u32 t = tau % L_slots;
    const int32_t steps[2] = {(int32_t)t, (int32_t)((t + n - L_slots) % n)};
    const ckks_gkey_t *keys[2] = {key_tau, key_wrap};
    const uint64_t *masks[2] = {d_mask_a, d_mask_b};
    return shift_bank(P, d_ct_in, level, 1, steps, keys, masks, d_ct_out, (hipStream_t)stream_);
}

}  // extern "C"
