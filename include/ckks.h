/*
 * C ABI of the MI355X CKKS ciphertext x plaintext matmul library (libckks_hip.so).
 *
 * Scope: the server side of the projection kernel Y = XW of the paper's
 * Sec. 3.2 / App. A.2 (segment-column packing, baby-step/giant-step diagonal
 * method) and the CKKS machinery it stands on: RNS arithmetic over
 * R_Q = Z_Q[X]/(X^N+1) (Sec. 2.2), the primitives add / ptmul / rot / conj of
 * Table 1, and rescale (Sec. 2.2).  The server holds evaluation keys and the
 * model, never the secret key (Sec. 2.3, "Key Distribution"); the ckks_client_*
 * calls at the end are the key holder's side and exist so that callers can
 * produce keys and ciphertexts without any other library.
 *
 * Conventions
 *  - Every call returns 0 (CKKS_OK) or a negative CKKS_E_* code; the message of
 *    the last failure on the calling thread is ckks_last_error().  No call
 *    aborts or throws across this boundary.
 *  - "d_" pointers are DEVICE pointers (HIP, current device); all others are
 *    HOST pointers.  The caller owns every buffer it passes.  Handles returned
 *    by *_create / *_load are owned by the library until the matching *_destroy.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Compute calls enqueue work on it and return without synchronising or
 *    allocating: every table is built and the scratch arena sized by the
 *    *_create calls (ckks_params_create for every call whose need follows from
 *    the parameter set, ckks_weights_create for its projection) or by
 *    ckks_params_reserve.  The *_create / *_load / *_set_* / *_reserve calls are
 *    set-up: they may allocate and synchronise the device.
 *  - The scratch arena and the error text belong to a params handle and to the
 *    calling thread respectively: calls on one handle must come from one thread
 *    at a time and be issued on one stream at a time (two calls in flight on
 *    different streams would share the arena).
 *  - Outputs may not overlap inputs unless a call says so; a call that would
 *    read what it has already overwritten returns CKKS_E_INVAL instead.
 *  - Residues are uint64 in [0, q_i), little endian.  A ciphertext at level l is
 *    [component 2][limb l][N], component 0 = c0, 1 = c1, in the NTT domain:
 *    entry k of a limb is the polynomial evaluated at psi^(2*bitrev(k)+1), psi the
 *    smallest positive 2N-th primitive root of that limb's prime.  Size
 *    2*N*l*8 bytes, the ct_bytes(N, L) of the paper's Eq. in Sec. 5.2.
 *  - Limb ids: 0..L-1 are the ciphertext primes q_i, L..L+K-1 the special primes.
 */
#ifndef CKKS_H
#define CKKS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CKKS_OK 0
#define CKKS_E_INVAL (-1) /* bad argument: null pointer, size, non-prime, ... */
#define CKKS_E_LEVEL (-2) /* level out of range for the operation */
#define CKKS_E_NOKEY (-3) /* a non-identity Galois element without a key */
#define CKKS_E_NOMEM (-4) /* device or host allocation failed */
#define CKKS_E_HIP (-5)   /* a HIP runtime call failed */

#define CKKS_STEP_CONJ INT32_MIN /* "step" meaning complex conjugation (Table 1, conj) */

typedef struct ckks_params ckks_params_t;
typedef struct ckks_gkey ckks_gkey_t;
typedef struct ckks_weights ckks_weights_t;

/* Operation counts of one ckks_ctpt_matmul call (App. A.2.2 counts key switches). */
typedef struct {
    uint64_t key_switches; /* rotations that needed a key */
    uint64_t ptmuls;       /* ciphertext x plaintext products */
    uint64_t limb_ntts;    /* forward + inverse limb transforms */
} ckks_counters_t;

const char *ckks_last_error(void);

/* Prime search used by the benchmark configurations: the first `count` primes
 * among 2^bits - k*2N + 1, k = 1, 2, ... (all are 1 mod 2N).  out: host, count
 * entries.  CKKS_E_INVAL if bits > 61 or the range is exhausted. */
int ckks_find_primes(uint32_t bits, uint32_t logN, uint32_t count, uint64_t *out);

/* Parameter set (Sec. 2.2): ring degree N = 2^logN (10 <= logN <= 17), ciphertext
 * primes q[0..L-1] (q[0] = base), special primes p[0..K-1] (K = 0 allowed: no key
 * switching), dnum digits of alpha = L/dnum limbs for hybrid key switching.
 * Validates: primes distinct, prime, < 2^62, 1 mod 2N; L % dnum == 0; L+K <= 64;
 * alpha, K <= 16.  Builds twiddle and base-conversion tables on the current
 * device. */
int ckks_params_create(uint32_t logN, const uint64_t *q, uint32_t L, const uint64_t *p, uint32_t K,
                       uint32_t dnum, ckks_params_t **out);
void ckks_params_destroy(ckks_params_t *params);

/* Scratch arena of a params handle.  ckks_params_create sizes it for a full batch of hoisted key switches at
 * level L (ckks_rotate_hoisted with any number of steps, ckks_ctmul, ckks_shift_bank, ckks_rot_first, the
 * ckks_client_* calls), ckks_rescale and ckks_encode / ckks_decode; ckks_weights_create grows it to what
 * ckks_ctpt_matmul on those weights needs.  ckks_params_reserve grows it to at least `bytes` (set-up call:
 * synchronises the device; CKKS_E_NOMEM if the device refuses).  Should a compute call ever need more than
 * is reserved it grows the arena itself after draining its stream -- except on a capturing stream, where it
 * returns CKKS_E_NOMEM and the caller reserves first.  ckks_params_scratch_bytes reports the current size. */
int ckks_params_reserve(ckks_params_t *params, uint64_t bytes);
int ckks_params_scratch_bytes(const ckks_params_t *params, uint64_t *bytes);

/* psi of limb `limb` (host out): the root that fixes the NTT-domain bits. */
int ckks_params_root(const ckks_params_t *params, uint32_t limb, uint64_t *psi);

/* Negacyclic NTT / inverse NTT in place on d_data [batch][n_limbs][N]; row
 * (b, i) is a polynomial modulo limb limb_ids[i] (host array, n_limbs <= 64).
 * Forward: natural coefficient order in, bit-reversed evaluation order out
 * (out[k] = a(psi^(2*bitrev(k)+1))).  Inverse undoes it, including 1/N. */
int ckks_ntt(const ckks_params_t *params, uint64_t *d_data, const uint32_t *limb_ids, uint32_t n_limbs,
             uint32_t batch, void *stream);
int ckks_intt(const ckks_params_t *params, uint64_t *d_data, const uint32_t *limb_ids, uint32_t n_limbs,
              uint32_t batch, void *stream);

/* Galois element of a slot rotation: rot by `step` is the cyclic LEFT shift of
 * the n = N/2 slots (Sec. 3.1): 5^(step mod n) mod 2N; CKKS_STEP_CONJ -> 2N-1. */
int ckks_galois_elt(const ckks_params_t *params, int32_t step, uint64_t *galois_elt);

/* Evaluation key for one Galois element (the "Galois keys" of Sec. 2.1).
 * d_key: [dnum][2][L+K][N], NTT domain, canonical residues; component 0 = b_j,
 * 1 = a_j with b_j = -a_j*s + e_j + P*T_j*sigma_g(s).  ckks_galois_key_load COPIES:
 * the library keeps its own copy in its internal (Montgomery) form, 96 MiB at
 * N = 2^16 with 24 + 8 primes, and d_key may be freed once `stream` has drained.
 * ckks_galois_key_adopt BORROWS: d_key is rewritten in place into the internal
 * form (it is no longer a canonical key afterwards) and the handle points at it; the
 * caller keeps ownership and must keep the buffer alive and untouched until the
 * handle is destroyed.  No second copy of the key exists on that path. */
int ckks_galois_key_load(const ckks_params_t *params, uint64_t galois_elt, const uint64_t *d_key,
                         void *stream, ckks_gkey_t **out);
int ckks_galois_key_adopt(const ckks_params_t *params, uint64_t galois_elt, uint64_t *d_key, void *stream,
                          ckks_gkey_t **out);
void ckks_galois_key_destroy(ckks_gkey_t *key);

/* Relinearisation key (Sec. 2.1 "relinearization keys"): same layout as a Galois key, with
 * b_j = -a_j*s + e_j + P*T_j*s^2. */
int ckks_relin_key_load(const ckks_params_t *params, const uint64_t *d_key, void *stream, ckks_gkey_t **out);

/* ctmul of Table 1: slotwise product of two ciphertexts at `level`, relinearised with the same hybrid key
 * switch as a rotation: (t0,t1,t2) = (a0*b0, a0*b1+a1*b0, a1*b1), out = (t0,t1) + ModDown(<digits(t2), key>).
 * d_ct_a, d_ct_b, d_ct_out: [2][level][N] (out may not alias the inputs).  scale(out) = scale(a)*scale(b):
 * follow with ckks_rescale.  CKKS_E_NOKEY without a key. */
int ckks_ctmul(ckks_params_t *params, const uint64_t *d_ct_a, const uint64_t *d_ct_b, uint32_t level,
               const ckks_gkey_t *relin_key, uint64_t *d_ct_out, void *stream);

/* rot / conj of Table 1 for many steps of ONE ciphertext (the rotation banks
 * of Sec. 3.2/3.3 share their input): INTT(c1), digit decomposition and ModUp
 * are done once, then per step: automorphism, inner product with the key,
 * ModDown, + sigma(c0).  d_ct_in [2][level][N]; steps (host) as in
 * ckks_galois_elt; keys (host array of n_steps handles, in step order; an entry
 * may be NULL only if its step is the identity, which is copied); d_ct_out
 * [n_steps][2][level][N], which may not overlap d_ct_in (the switches gather
 * from the input while outputs are written).  Errors: CKKS_E_LEVEL (level 0 or
 * > L), CKKS_E_NOKEY, CKKS_E_INVAL (key of another element, K = 0, overlap). */
int ckks_rotate_hoisted(ckks_params_t *params, const uint64_t *d_ct_in, uint32_t level, const int32_t *steps,
                        uint32_t n_steps, const ckks_gkey_t *const *keys, uint64_t *d_ct_out, void *stream);

/* Plaintext weights of one projection Y = XW (Sec. 3.2, App. A.2.1) at `level`:
 * segment length m, C columns per ciphertext (C divides N/2/m; the C columns
 * repeat over all segments), G input groups, B_out output blocks, N1 baby steps
 * (N1 divides C, N2 = C/N1).  Diagonals are handed over as encoded integer
 * coefficient polynomials and expanded here to `level` limbs in the NTT domain
 * (offline step, not part of the matmul latency).  Diagonal (b, p, g, q) has
 * index ((b*N2 + p)*G + g)*N1 + q; its slot vector holds
 * W[g*C + (c+q) mod C, b*C + (c - p*N1) mod C] in every slot of segment c. */
int ckks_weights_create(const ckks_params_t *params, uint32_t level, uint32_t m, uint32_t C, uint32_t G,
                        uint32_t B_out, uint32_t N1, ckks_weights_t **out);
/* d_coeffs: int64 [count][N] for diagonals first .. first+count-1. */
int ckks_weights_set_diagonals(ckks_weights_t *w, uint32_t first, uint32_t count, const int64_t *d_coeffs,
                               void *stream);
/* d_bias_coeffs: int64 [B_out][N]; the plaintext added to c0 of block b is
 * bias_coeffs[b] * bias_mul (an integer factor that lifts the bias encoding to
 * the product scale). */
int ckks_weights_set_bias(ckks_weights_t *w, const int64_t *d_bias_coeffs, uint64_t bias_mul, void *stream);
/* The three calls above in one: all B_out*N2*G*N1 diagonals (d_coeffs, int64 [B_out][N2][G][N1][N], device) and, if
 * d_bias_coeffs is not NULL, the bias.  On error nothing is left allocated. */
int ckks_weights_load(const ckks_params_t *params, uint32_t level, uint32_t m, uint32_t C, uint32_t G,
                      uint32_t B_out, uint32_t N1, const int64_t *d_coeffs, const int64_t *d_bias_coeffs,
                      uint64_t bias_mul, void *stream, ckks_weights_t **out);
void ckks_weights_destroy(ckks_weights_t *w);

/* Y = XW + bias on ciphertexts (Sec. 3.2):
 *   bank x_q^(g) = rot(x^(g); q*m), q < N1 (hoisted, one call per input);
 *   acc_{b,p} = sum_g sum_q x_q^(g) (.) w_{b,p,g,q};
 *   y_b = acc_{b,0} + sum_{p>=1} rot(acc_{b,p}; p*N1*m);
 *   y_b += conj(y_b) if conj_key is given (decomplexification of Sec. 3.2: the inputs are then the
 *          complexified x^(2u) + i*x^(2u+1), G counts them, and the complex weights of App. A.2.1 carry the
 *          factor 1/2; one conjugation per output block, the count of App. A.2.2);
 *   y_b += bias_b.
 * flags = CKKS_MATMUL_MERGED_GIANT evaluates the giant step as
 *   y_b = acc_{b,0} + (sum_p sigma_p(acc_{b,p}.c0), 0) + ModDown(sum_p sum_j sigma_p(d_j(acc_{b,p}.c1)) key_{p,j}),
 * i.e. the N2-1 switched accumulators are summed over the extended basis and brought down once.  ModDown is
 * not exactly linear, so the residues differ from the default (each rotation a complete key switch) while
 * decrypting to the same values; both orders are defined bit for bit.
 * The library is agnostic of what the slots hold: real packing (real diagonals), complex-pair compression
 * (complex diagonals + conj_key) and the fused QK projection of App. A.2.3 (weights W_Q + i*W_K, no
 * conj_key, Q and K come out in the real and imaginary parts) differ only in the plaintexts handed to
 * ckks_weights_set_diagonals.
 * d_ct_x [G][2][level][N]; baby_keys: N1-1 handles for steps q*m (q = 1..);
 * giant_keys: N2-1 handles for steps p*N1*m; conj_key: NULL or the key of
 * CKKS_STEP_CONJ; d_ct_y [B_out][2][level][N] at the
 * input level and scale(x)*scale(w) -- follow with ckks_rescale, or pass
 * CKKS_MATMUL_RESCALE and receive [B_out][2][level-1][N]; may not overlap
 * d_ct_x.  counters (host, may be NULL) receives the operation counts.
 * CKKS_E_NOKEY for a missing key of a step that is not the identity.
 * CKKS_E_INVAL also for flags with unknown bits and for weights of which some
 * diagonal was never stored (the message names the first one): nothing is
 * enqueued then. */
#define CKKS_MATMUL_MERGED_GIANT 1u /* flags: one ModDown per output block for the whole giant step */
#define CKKS_MATMUL_RESCALE 2u      /* flags: d_ct_y receives the RESCALED blocks, [B_out][2][level-1][N]: the same
                                       residues as this call without the flag followed by ckks_rescale.  With
                                       CKKS_MATMUL_MERGED_GIANT (and no conj_key, N = 2^16, primes below 2^50) the
                                       ModDown of the giant step and the rescale share one pass: the dropped limb is
                                       taken in the coefficient domain before the correction's forward transform, so
                                       each remaining limb is transformed once for both.  CKKS_E_LEVEL at level 1. */
#define CKKS_MATMUL_CONJ_PER_ACC 4u /* flags (needs conj_key, else CKKS_E_NOKEY): the decomplexification in the order
                                       Sec. 3.2 displays it, acc_{b,p} += conj(acc_{b,p}) for every giant-step
                                       accumulator before the fold over p, N2 conjugations per output block instead of
                                       one.  Automorphisms commute, so both orders decrypt to the same values; the
                                       residues differ (other noise) and each order is defined bit for bit. */
int ckks_ctpt_matmul(ckks_params_t *params, const ckks_weights_t *w, const uint64_t *d_ct_x,
                     const ckks_gkey_t *const *baby_keys, const ckks_gkey_t *const *giant_keys,
                     const ckks_gkey_t *conj_key, uint32_t flags, uint64_t *d_ct_y, ckks_counters_t *counters,
                     void *stream);

/* Plaintext in evaluation form for ckks_ptmul / ckks_rot_first: int64 coefficient polynomials d_coeffs
 * [count][N] (an encoding at the caller's scale, Sec. 2.2) -> canonical NTT-domain residues d_out
 * [count][level][N] on limbs 0..level-1. */
int ckks_plain_expand(const ckks_params_t *params, uint32_t level, const int64_t *d_coeffs, uint32_t count,
                      uint64_t *d_out, void *stream);

/* add of Table 1: d_ct_out = d_ct_a + d_ct_b, limb-wise, for n_ct ciphertexts [n_ct][2][level][N] of equal
 * level and scale.  d_ct_out may alias either input. */
int ckks_add(const ckks_params_t *params, const uint64_t *d_ct_a, const uint64_t *d_ct_b, uint32_t level,
             uint32_t n_ct, uint64_t *d_ct_out, void *stream);

/* ptmul of Table 1: both components of d_ct [2][level][N] times the plaintext d_plain [level][N] (from
 * ckks_plain_expand).  scale(out) = scale(ct)*scale(plain): follow with ckks_rescale.  out may alias d_ct. */
int ckks_ptmul(const ckks_params_t *params, const uint64_t *d_ct, uint32_t level, const uint64_t *d_plain,
               uint64_t *d_ct_out, void *stream);

/* ModSwitchToNext (Sec. 5.4): drops limb level_in-1 WITHOUT dividing: value and scale are unchanged, one level
 * of budget is given up.  [n_ct][2][level_in][N] -> [n_ct][2][level_in-1][N]; in and out may not overlap.
 * CKKS_E_LEVEL if level_in < 2. */
int ckks_mod_switch_to_next(const ckks_params_t *params, const uint64_t *d_ct_in, uint32_t level_in, uint32_t n_ct,
                            uint64_t *d_ct_out, void *stream);

/* Bank of masked rotation pairs of ONE ciphertext (the rotation banks of Sec. 3.1 / 3.3 with the shift
 * realisations of App. A.1):
 *   out_i = rot(x; steps[2i]) (.) mask_{2i} + rot(x; steps[2i+1]) (.) mask_{2i+1},   i < n_out.
 * The intra-segment shift Psi^t is the instance steps = (t mod m, (t mod m - m) mod n) with the masks
 * H = 1{r < m - t}, U = 1{r >= m - t} on slot s*m + r; RotFirst_L and Phi_C^Delta are instances too (below).  All
 * 2*n_out rotations share the input's decomposition (hoisting).  steps (host, as in ckks_galois_elt), keys (host
 * array of 2*n_out handles; NULL only where the step is the identity), d_masks [n_out][2][level][N] plaintexts from
 * ckks_plain_expand at one scale; d_ct_out [n_out][2][level][N], may not alias the input.  scale(out) =
 * scale(x)*scale(mask): follow with ckks_rescale.  Errors as ckks_rotate_hoisted. */
int ckks_shift_bank(ckks_params_t *params, const uint64_t *d_ct_in, uint32_t level, uint32_t n_out,
                    const int32_t *steps, const ckks_gkey_t *const *keys, const uint64_t *d_masks,
                    uint64_t *d_ct_out, void *stream);

/* RotFirst_L(x; tau) of App. A.1: cyclic LEFT shift by tau (mod L) inside the first L slots,
 *   rot(x; tau) (.) a + rot(x; (tau - L) mod n) (.) b,
 * a = 1{0 <= i < L - tau}, b = 1{L - tau <= i < L} given by the caller as plaintexts d_mask_a, d_mask_b
 * [level][N] (ckks_plain_expand of their encodings, both at one scale).  Slots L..n-1 come out as zero.  The two
 * rotations share one hoisted decomposition.  key_tau is the key of step tau mod L, key_wrap of step
 * (tau mod L - L) mod n; either may be NULL when its step is 0 (mod n).  With L = C*m and tau = Delta*m this is the
 * restricted segment shift Phi_C^Delta used when fewer than N_seg segments are active.  scale(out) =
 * scale(x)*scale(mask): follow with ckks_rescale.  d_ct_out [2][level][N], may not alias d_ct_in. */
int ckks_rot_first(ckks_params_t *params, const uint64_t *d_ct_in, uint32_t level, uint32_t L_slots, uint32_t tau,
                   const ckks_gkey_t *key_tau, const ckks_gkey_t *key_wrap, const uint64_t *d_mask_a,
                   const uint64_t *d_mask_b, uint64_t *d_ct_out, void *stream);

/* rescale (Sec. 2.2): drops limb level_in-1 and divides by its prime with
 * centred rounding.  d_ct_in [n_ct][2][level_in][N] -> d_ct_out
 * [n_ct][2][level_in-1][N], which may not overlap d_ct_in (CKKS_E_INVAL).
 * CKKS_E_LEVEL if level_in < 2 or > L. */
int ckks_rescale(ckks_params_t *params, const uint64_t *d_ct_in, uint32_t level_in, uint32_t n_ct,
                 uint64_t *d_ct_out, void *stream);

/* ckks_rescale for callers that cannot allocate device memory or tolerate a call that might: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and the same bits
 * as ckks_rescale, but the one scratch buffer (the dropped limbs in the coefficient domain, 2 * n_ct * N words)
 * lives in a static device array of 2^20 words (8 MiB per GPU, held until the process ends) instead of the
 * params handle's arena: CKKS_E_INVAL if 2 * n_ct * N exceeds that (8 ciphertexts at N = 2^16), or if the
 * current device is not the parameter set's.  Calls no hipMalloc / hipFree, enqueues on `stream` and returns.
 * All calls on one GPU share the array: two calls that overlap in time on one GPU (different streams or
 * threads) race; calls on one stream are ordered and safe.  Nothing needs clearing between calls: every word a
 * call reads it has written first. */
int ckks_rescale_static(ckks_params_t *params, const uint64_t *d_ct_in, uint32_t level_in, uint32_t n_ct,
                        uint64_t *d_ct_out, void *stream);

/* ---- key holder's side (the client of Sec. 2.3: KeyGen, Enc, Dec) ----------
 * Randomness is drawn by the caller and passed in, so results are reproducible
 * and comparable bit for bit.  None of these calls is on the server's path. */
typedef struct ckks_secret ckks_secret_t;

/* Secret key s in {-1,0,1}^N (host, int8): keeps NTT(s) on every limb on the device. */
int ckks_client_secret_load(const ckks_params_t *params, const int8_t *s, void *stream, ckks_secret_t **out);
void ckks_client_secret_destroy(ckks_secret_t *secret);

/* Galois key for `galois_elt`: b_j = -a_j*s + e_j + [P*T_j]*sigma_g(s), key[j] = (b_j, a_j), where
 * [P*T_j] is P mod q_i on the limbs of digit j and 0 elsewhere.  d_a [dnum][L+K][N] uniform
 * residues (taken as NTT-domain values), d_e int64 [dnum][N] small errors (coefficients),
 * d_key out [dnum][2][L+K][N] canonical, NTT domain (the layout ckks_galois_key_load takes). */
int ckks_client_galois_keygen(ckks_params_t *params, const ckks_secret_t *secret, uint64_t galois_elt,
                              const uint64_t *d_a, const int64_t *d_e, uint64_t *d_key, void *stream);

/* Relinearisation key: as above with s^2 in place of sigma_g(s). */
int ckks_client_relin_keygen(ckks_params_t *params, const ckks_secret_t *secret, const uint64_t *d_a,
                             const int64_t *d_e, uint64_t *d_key, void *stream);

/* Symmetric encryption at `level`: c1 = a, c0 = -a*s + e + m.  d_m int64 [N] encoded plaintext
 * coefficients, d_a [level][N] uniform residues (NTT domain), d_e int64 [N]; d_ct out [2][level][N]. */
int ckks_client_encrypt(ckks_params_t *params, const ckks_secret_t *secret, uint32_t level, const int64_t *d_m,
                        const uint64_t *d_a, const int64_t *d_e, uint64_t *d_ct, void *stream);

/* c0 + c1*s on the first nlimbs limbs, coefficient domain: d_out [nlimbs][N] canonical residues
 * (the caller lifts them by CRT and decodes). */
int ckks_client_decrypt(ckks_params_t *params, const ckks_secret_t *secret, const uint64_t *d_ct, uint32_t level,
                        uint32_t nlimbs, uint64_t *d_out, void *stream);

/* ---- complex-slot encode / decode on the device (Sec. 2.1 Encode / Decode; slot order of Sec. 3.1) ----
 * Slot j of a plaintext m(X) is m(zeta^(5^j)), zeta = exp(i*pi/N), j < n = N/2, so that a rotation by r is the
 * cyclic left shift of the slot vector.  fp64 throughout (one N-point complex transform per vector); results agree
 * with an exact evaluation to about 1e-13 * N * max|z| relative to the scale, so a rounded coefficient can differ by
 * one unit from another fp64 implementation's when it falls next to a half-integer. */

#define CKKS_ENCODE_REAL 1u /* flags: imaginary parts are taken as zero and the coefficients satisfy
                               c[N-k] = -c[k], c[N/2] = 0 exactly (what ckks_weights_set_diagonals needs to keep
                               half of every limb) */

/* d_slots: device, [count][n] complex doubles (re, im interleaved).  d_coeffs: device, int64 [count][N], the
 * nearest integers to scale * m_k, ready for ckks_client_encrypt, ckks_plain_expand or
 * ckks_weights_set_diagonals.  scale * max|z| must stay below 2^62.  Enqueues on `stream`; uses the library's
 * scratch arena (64 vectors per pass). */
int ckks_encode(ckks_params_t *params, const double *d_slots, uint32_t count, double scale, uint32_t flags,
                int64_t *d_coeffs, void *stream);

/* d_res: device, [count][nlimbs][N] canonical residues of the plaintext polynomial on the first nlimbs (1 or 2)
 * ciphertext primes, coefficient domain (what ckks_client_decrypt writes); the centred lift must be the
 * plaintext itself, i.e. |coefficients| < q_0/2 (or q_0*q_1/2).  d_slots: device, [count][n] complex doubles,
 * m(zeta^(5^j)) / scale. */
int ckks_decode(ckks_params_t *params, const uint64_t *d_res, uint32_t nlimbs, uint32_t count, double scale,
                double *d_slots, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* CKKS_H */
