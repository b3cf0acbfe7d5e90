/*
 * CPU oracle for the server-side RNS-CKKS ciphertext x plaintext matmul path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * HIP library is compared against bit for bit.  It shares no code, header,
 * table generator or constant with the GPU library and must never be imported,
 * linked or executed by the product path.
 *
 * Arithmetic: every modular product is a 128-bit product followed by the C
 * remainder operator; every sum is reduced at once.  No lazy accumulation, no
 * blocking, no fusion.  Threading (OpenMP) is only over independent limbs,
 * Galois elements or output blocks.
 *
 * What the paper fixes and what it leaves open.  The paper works in
 * R_Q = Z_Q[X]/(X^N+1) with Q a product of word-sized primes held as residues
 * (Sec. 2.2, "CKKS Parameters"), lists the primitives add / ptmul / rot / conj
 * (Table 1), defines rot as the cyclic LEFT shift of the slot vector (Sec. 3.1),
 * rescale as division by the last prime (Sec. 2.2) and the projection kernel
 * Y = XW as a baby-step/giant-step sum of rotated inputs times plaintext
 * diagonals (Sec. 3.2, App. A.2.1).  It does not describe the NTT, the
 * key-switching algorithm or base conversion.  Those follow the standard
 * RNS-CKKS hybrid key switch; each reading is stated where it is used.
 *
 * parity unpinned: the residue-level bits produced by mod_up / mod_down /
 * rotate_hoisted / ctpt_matmul at N = 2^16 have no printed values to compare
 * with; they are pinned only through big-integer closed forms, decryption
 * bounds and brute force on tiny rings (tests/test_oracle_*.py).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef unsigned __int128 u128;
typedef uint64_t u64;
typedef int64_t i64;

/* ------------------------------------------------------------------ */
/* scalar modular arithmetic                                           */
/* ------------------------------------------------------------------ */
static inline u64 mulmod(u64 a, u64 b, u64 q) { return (u64)(((u128)a * b) % q); }
static inline u64 addmod(u64 a, u64 b, u64 q) { return (u64)(((u128)a + b) % q); }
static inline u64 submod(u64 a, u64 b, u64 q) { return (u64)(((u128)a + q - b) % q); }

static u64 powmod(u64 a, u64 e, u64 q) {
    u64 r = 1 % q;
    a %= q;
    while (e) {
        if (e & 1) r = mulmod(r, a, q);
        a = mulmod(a, a, q);
        e >>= 1;
    }
    return r;
}
/* q prime: a^(q-2) */
static u64 invmod(u64 a, u64 q) { return powmod(a, q - 2, q); }

u64 orc_mulmod(u64 a, u64 b, u64 q) { return mulmod(a, b, q); }
u64 orc_powmod(u64 a, u64 e, u64 q) { return powmod(a, e, q); }

/* Deterministic Miller-Rabin: the first twelve primes as bases decide every
 * n < 3.3e24, hence every 64-bit n. */
int orc_is_prime(u64 n) {
    static const u64 bases[12] = {2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37};
    if (n < 2) return 0;
    for (int i = 0; i < 12; i++) {
        if (n == bases[i]) return 1;
        if (n % bases[i] == 0) return 0;
    }
    u64 d = n - 1;
    int r = 0;
    while ((d & 1) == 0) { d >>= 1; r++; }
    for (int i = 0; i < 12; i++) {
        u64 x = powmod(bases[i], d, n);
        if (x == 1 || x == n - 1) continue;
        int composite = 1;
        for (int j = 1; j < r; j++) {
            x = mulmod(x, x, n);
            if (x == n - 1) { composite = 0; break; }
        }
        if (composite) return 0;
    }
    return 1;
}

/* Prime rule (reading; the paper names no primes): candidates
 * c_k = 2^bits - k*2N + 1 for k = 1,2,...; the primes among them, in order. */
int orc_find_primes(int bits, int logN, int count, u64 *out) {
    u64 twoN = (u64)2 << logN;
    u64 top = (u64)1 << bits;
    int found = 0;
    for (u64 k = 1; found < count; k++) {
        if (k * twoN >= top) return found;
        u64 c = top - k * twoN + 1;
        if (orc_is_prime(c)) out[found++] = c;
    }
    return found;
}

/* Root rule (reading): psi is the smallest positive integer with
 * psi^N = -1 (mod q).  Any primitive 2N-th root r generates all of them as its
 * odd powers; the minimum over those is taken. */
u64 orc_min_root(u64 q, int logN) {
    u64 N = (u64)1 << logN;
    u64 twoN = 2 * N;
    if ((q - 1) % twoN) return 0;
    u64 r = 0;
    for (u64 x = 2; x < q; x++) {
        u64 c = powmod(x, (q - 1) / twoN, q);
        if (powmod(c, N, q) == q - 1) { r = c; break; }
    }
    u64 r2 = mulmod(r, r, q);
    u64 best = r, cur = r;
    for (u64 i = 1; i < N; i++) {
        cur = mulmod(cur, r2, q);
        if (cur < best) best = cur;
    }
    return best;
}

static u64 brev(u64 x, int bits) {
    u64 r = 0;
    for (int i = 0; i < bits; i++) r |= ((x >> i) & 1) << (bits - 1 - i);
    return r;
}

/* ------------------------------------------------------------------ */
/* context                                                             */
/* ------------------------------------------------------------------ */
typedef struct orc_ctx {
    int logN, L, K, dnum, alpha;
    u64 N;
    u64 *mod;    /* [L+K]: q_0..q_{L-1}, p_0..p_{K-1} */
    u64 *psi;    /* [L+K] */
    u64 **pw;    /* [L+K][2N]: psi^e */
} orc_ctx;

orc_ctx *orc_ctx_create(int logN, const u64 *q, int L, const u64 *p, int K, int dnum) {
    if (dnum <= 0 || L % dnum) return NULL;
    orc_ctx *c = (orc_ctx *)calloc(1, sizeof(orc_ctx));
    c->logN = logN; c->L = L; c->K = K; c->dnum = dnum; c->alpha = L / dnum;
    c->N = (u64)1 << logN;
    int W = L + K;
    c->mod = (u64 *)malloc(sizeof(u64) * W);
    c->psi = (u64 *)malloc(sizeof(u64) * W);
    c->pw = (u64 **)malloc(sizeof(u64 *) * W);
    for (int i = 0; i < W; i++) c->mod[i] = i < L ? q[i] : p[i - L];
#pragma omp parallel for schedule(dynamic)
    for (int i = 0; i < W; i++) {
        c->psi[i] = orc_min_root(c->mod[i], logN);
        c->pw[i] = (u64 *)malloc(sizeof(u64) * 2 * c->N);
        c->pw[i][0] = 1;
        for (u64 e = 1; e < 2 * c->N; e++) c->pw[i][e] = mulmod(c->pw[i][e - 1], c->psi[i], c->mod[i]);
    }
    return c;
}

void orc_ctx_destroy(orc_ctx *c) {
    if (!c) return;
    for (int i = 0; i < c->L + c->K; i++) free(c->pw[i]);
    free(c->pw); free(c->psi); free(c->mod); free(c);
}

u64 orc_modulus(const orc_ctx *c, int limb) { return c->mod[limb]; }
u64 orc_psi(const orc_ctx *c, int limb) { return c->psi[limb]; }

/* ------------------------------------------------------------------ */
/* negacyclic NTT                                                      */
/* ------------------------------------------------------------------ */
/* Definition (reading of "bit-reversed-order convention fixed"):
 *   out[k] = sum_j a[j] * psi^((2*brev(k)+1)*j)  (mod q),  k = 0..N-1,
 * natural coefficient order in, bit-reversed evaluation order out. */
void orc_ntt_naive(const orc_ctx *c, int limb, const u64 *a, u64 *out) {
    u64 q = c->mod[limb], N = c->N, twoN = 2 * N;
    for (u64 k = 0; k < N; k++) {
        u64 e = 2 * brev(k, c->logN) + 1;
        u64 acc = 0;
        for (u64 j = 0; j < N; j++)
            acc = addmod(acc, mulmod(a[j], c->pw[limb][(e * j) % twoN], q), q);
        out[k] = acc;
    }
}

/* The same map by repeated splitting of X^(2t) - psi^(2e) into
 * (X^t - psi^e)(X^t + psi^e): a polynomial lo + X^t*hi reduces to
 * lo + psi^e*hi and lo - psi^e*hi.  At depth s (2^s nodes) node i uses
 * e = (2*brev_s(i)+1) * N / 2^(s+1); leaf k ends at exponent 2*brev(k)+1. */
void orc_ntt(const orc_ctx *c, int limb, u64 *a) {
    u64 q = c->mod[limb], N = c->N;
    for (int s = 0; s < c->logN; s++) {
        u64 nodes = (u64)1 << s, t = N >> (s + 1);
        for (u64 i = 0; i < nodes; i++) {
            u64 e = (2 * brev(i, s) + 1) * (N >> (s + 1));
            u64 w = c->pw[limb][e];
            u64 *lo = a + i * 2 * t, *hi = lo + t;
            for (u64 j = 0; j < t; j++) {
                u64 u = lo[j], v = mulmod(hi[j], w, q);
                lo[j] = addmod(u, v, q);
                hi[j] = submod(u, v, q);
            }
        }
    }
}

/* Inverse: undo the splits from the leaves up, (x,y) -> ((x+y)/2, (x-y)/(2w)),
 * with all the halvings collected into one multiplication by N^-1. */
void orc_intt(const orc_ctx *c, int limb, u64 *a) {
    u64 q = c->mod[limb], N = c->N;
    for (int s = c->logN - 1; s >= 0; s--) {
        u64 nodes = (u64)1 << s, t = N >> (s + 1);
        for (u64 i = 0; i < nodes; i++) {
            u64 e = (2 * brev(i, s) + 1) * (N >> (s + 1));
            u64 winv = c->pw[limb][2 * N - e];
            u64 *lo = a + i * 2 * t, *hi = lo + t;
            for (u64 j = 0; j < t; j++) {
                u64 x = lo[j], y = hi[j];
                lo[j] = addmod(x, y, q);
                hi[j] = mulmod(submod(x, y, q), winv, q);
            }
        }
    }
    u64 ninv = invmod(N % q, q);
    for (u64 j = 0; j < N; j++) a[j] = mulmod(a[j], ninv, q);
}

/* ------------------------------------------------------------------ */
/* Galois automorphisms                                                */
/* ------------------------------------------------------------------ */
/* rot by r (left shift, Sec. 3.1) <-> g = 5^(r mod n) mod 2N; conj <-> 2N-1.
 * Reading: slot j sits at the root zeta^(5^j), zeta = exp(i*pi/N). */
u64 orc_galois_elt(const orc_ctx *c, i64 step, int conj) {
    u64 twoN = 2 * c->N, n = c->N / 2;
    if (conj) return twoN - 1;
    i64 r = step % (i64)n;
    if (r < 0) r += (i64)n;
    u64 g = 1;
    for (i64 i = 0; i < r; i++) g = (g * 5) % twoN;
    return g;
}

/* a(X) -> a(X^g): X^j goes to X^(g*j mod 2N), and X^N = -1. */
void orc_automorph_coeff(const orc_ctx *c, int limb, u64 g, const u64 *in, u64 *out) {
    u64 q = c->mod[limb], N = c->N, twoN = 2 * N;
    for (u64 j = 0; j < N; j++) {
        u64 r = (u64)(((u128)g * j) % twoN);
        if (r < N) out[r] = in[j];
        else out[r - N] = in[j] == 0 ? 0 : q - in[j];
    }
}

/* In the evaluation domain sigma_g(a)(psi^e) = a(psi^(e*g)): a pure gather. */
void orc_automorph_ntt(const orc_ctx *c, u64 g, const u64 *in, u64 *out) {
    u64 N = c->N, twoN = 2 * N;
    for (u64 k = 0; k < N; k++) {
        u64 e = 2 * brev(k, c->logN) + 1;
        u64 e2 = (u64)(((u128)e * g) % twoN);
        u64 k2 = brev((e2 - 1) / 2, c->logN);
        out[k] = in[k2];
    }
}

/* ------------------------------------------------------------------ */
/* base conversion                                                     */
/* ------------------------------------------------------------------ */
static int ext_limb(const orc_ctx *c, int level, int t) { /* index in [level+K) -> global limb */
    return t < level ? t : c->L + (t - level);
}

/* ModUp of digit j at `level` (reading: approximate integer base conversion,
 * no floating-point correction).  D = active limbs [j*alpha, min((j+1)*alpha, level)).
 *   y_i  = c_i * [(Q_D/q_i)^-1]_{q_i}  mod q_i
 *   out_t = sum_{i in D} y_i * [Q_D/q_i]_t  mod t      for t outside D
 *   out_t = c_t                                          for t in D.
 * Input [level][N] and output [level+K][N] are in the coefficient domain. */
void orc_modup(const orc_ctx *c, int level, int j, const u64 *in, u64 *out) {
    u64 N = c->N;
    int lo = j * c->alpha, hi = lo + c->alpha;
    if (hi > level) hi = level;
    int nd = hi - lo;
    u64 *y = (u64 *)malloc(sizeof(u64) * nd * N);
    for (int a = 0; a < nd; a++) {
        int i = lo + a;
        u64 qi = c->mod[i];
        u64 prod = 1; /* Q_D/q_i mod q_i */
        for (int b = lo; b < hi; b++) if (b != i) prod = mulmod(prod, c->mod[b] % qi, qi);
        u64 inv = invmod(prod, qi);
        for (u64 x = 0; x < N; x++) y[a * N + x] = mulmod(in[(u64)i * N + x], inv, qi);
    }
#pragma omp parallel for schedule(dynamic)
    for (int t = 0; t < level + c->K; t++) {
        int gl = ext_limb(c, level, t);
        u64 *o = out + (u64)t * N;
        if (t >= lo && t < hi) { memcpy(o, in + (u64)t * N, sizeof(u64) * N); continue; }
        u64 mt = c->mod[gl];
        for (u64 x = 0; x < N; x++) o[x] = 0;
        for (int a = 0; a < nd; a++) {
            int i = lo + a;
            u64 f = 1; /* Q_D/q_i mod t */
            for (int b = lo; b < hi; b++) if (b != i) f = mulmod(f, c->mod[b] % mt, mt);
            for (u64 x = 0; x < N; x++) o[x] = addmod(o[x], mulmod(y[a * N + x] % mt, f, mt), mt);
        }
    }
    free(y);
}

/* ModDown (reading: no P/2 rounding offset).  u is [level+K][N] in the NTT
 * domain, v is [level][N] in the NTT domain.
 *   y_k = INTT(u_{p_k}) * [(P/p_k)^-1]_{p_k}
 *   w_i = sum_k y_k * [P/p_k]_{q_i}            (coefficient domain)
 *   v_i = (u_{q_i} - NTT_i(w_i)) * [P^-1]_{q_i}. */
void orc_moddown(const orc_ctx *c, int level, const u64 *u, u64 *v) {
    u64 N = c->N;
    int K = c->K, L = c->L;
    u64 *y = (u64 *)malloc(sizeof(u64) * K * N);
#pragma omp parallel for schedule(dynamic)
    for (int k = 0; k < K; k++) {
        u64 pk = c->mod[L + k];
        memcpy(y + (u64)k * N, u + (u64)(level + k) * N, sizeof(u64) * N);
        orc_intt(c, L + k, y + (u64)k * N);
        u64 prod = 1;
        for (int b = 0; b < K; b++) if (b != k) prod = mulmod(prod, c->mod[L + b] % pk, pk);
        u64 inv = invmod(prod, pk);
        for (u64 x = 0; x < N; x++) y[k * N + x] = mulmod(y[k * N + x], inv, pk);
    }
#pragma omp parallel for schedule(dynamic)
    for (int i = 0; i < level; i++) {
        u64 qi = c->mod[i];
        u64 *w = (u64 *)calloc(N, sizeof(u64));
        u64 Pmod = 1;
        for (int k = 0; k < K; k++) {
            Pmod = mulmod(Pmod, c->mod[L + k] % qi, qi);
            u64 f = 1;
            for (int b = 0; b < K; b++) if (b != k) f = mulmod(f, c->mod[L + b] % qi, qi);
            for (u64 x = 0; x < N; x++) w[x] = addmod(w[x], mulmod(y[k * N + x] % qi, f, qi), qi);
        }
        orc_ntt(c, i, w);
        u64 Pinv = invmod(Pmod, qi);
        for (u64 x = 0; x < N; x++)
            v[(u64)i * N + x] = mulmod(submod(u[(u64)i * N + x], w[x], qi), Pinv, qi);
        free(w);
    }
    free(y);
}

/* ------------------------------------------------------------------ */
/* hoisted rotations                                                   */
/* ------------------------------------------------------------------ */
/* Order (reading; binding because mod_up is not linear):
 *   INTT(c1) -> mod_up of every digit once -> NTT ->
 *   for each g: sigma_g on the extended digits -> inner product with the key
 *   -> mod_down of both components -> (sigma_g(c0) + v0, v1).
 * ct_in [2][level][N] NTT domain.  key_g [dnum][2][L+K][N] NTT domain with
 * component 0 = b, 1 = a.  g == 1 is the identity: the input is copied and no
 * key is touched.  out [n_g][2][level][N]. */
void orc_rotate_hoisted(const orc_ctx *c, const u64 *ct_in, int level, const u64 *gelts, int n_g,
                        const u64 *const *keys, u64 *out) {
    u64 N = c->N;
    int K = c->K, L = c->L, W = level + K;
    int beta = (level + c->alpha - 1) / c->alpha;
    const u64 *c0 = ct_in, *c1 = ct_in + (u64)level * N;

    u64 *c1c = (u64 *)malloc(sizeof(u64) * level * N);
    memcpy(c1c, c1, sizeof(u64) * level * N);
#pragma omp parallel for schedule(dynamic)
    for (int i = 0; i < level; i++) orc_intt(c, i, c1c + (u64)i * N);

    u64 *dig = (u64 *)malloc(sizeof(u64) * beta * W * N); /* [beta][W][N] NTT domain */
    for (int j = 0; j < beta; j++) orc_modup(c, level, j, c1c, dig + (u64)j * W * N);
#pragma omp parallel for schedule(dynamic)
    for (int jt = 0; jt < beta * W; jt++) {
        int t = jt % W;
        orc_ntt(c, ext_limb(c, level, t), dig + (u64)jt * N);
    }
    free(c1c);

    /* threads go to the Galois elements when there are several, else to the limbs */
#pragma omp parallel for schedule(dynamic) if (n_g >= 4)
    for (int r = 0; r < n_g; r++) {
        u64 g = gelts[r];
        u64 *o = out + (u64)r * 2 * level * N;
        if (g == 1) { memcpy(o, ct_in, sizeof(u64) * 2 * level * N); continue; }
        const u64 *key = keys[r];
        u64 *u = (u64 *)calloc((size_t)2 * W * N, sizeof(u64)); /* [2][W][N] */
        u64 *tmp = (u64 *)malloc(sizeof(u64) * N);
#pragma omp parallel for schedule(dynamic)
        for (int t = 0; t < W; t++)
            for (int j = 0; j < beta; j++) {
                int gl = ext_limb(c, level, t);
                u64 mt = c->mod[gl];
                u64 *perm = (u64 *)malloc(sizeof(u64) * N);
                orc_automorph_ntt(c, g, dig + ((u64)j * W + t) * N, perm);
                for (int comp = 0; comp < 2; comp++) {
                    const u64 *kk = key + (((u64)j * 2 + comp) * (L + K) + gl) * N;
                    u64 *uu = u + ((u64)comp * W + t) * N;
                    for (u64 x = 0; x < N; x++) uu[x] = addmod(uu[x], mulmod(perm[x], kk[x], mt), mt);
                }
                free(perm);
            }
        orc_moddown(c, level, u, o);
        orc_moddown(c, level, u + (u64)W * N, o + (u64)level * N);
        for (int i = 0; i < level; i++) {
            orc_automorph_ntt(c, g, c0 + (u64)i * N, tmp);
            for (u64 x = 0; x < N; x++) o[(u64)i * N + x] = addmod(o[(u64)i * N + x], tmp[x], c->mod[i]);
        }
        free(tmp); free(u);
    }
    free(dig);
}

/* Variant used by the merged giant step: the key switch of one ciphertext up to, but not including,
 * ModDown.  u_acc [2][level+K][N] += sum_j sigma_g(d_j) (.) key_j  (all limbs, NTT domain) and
 * c0_acc [level][N] += sigma_g(c0).  The decomposition of c1 is that of orc_rotate_hoisted. */
void orc_switch_accumulate(const orc_ctx *c, const u64 *ct_in, int level, u64 g, const u64 *key, u64 *u_acc,
                           u64 *c0_acc) {
    u64 N = c->N;
    int K = c->K, L = c->L, W = level + K;
    int beta = (level + c->alpha - 1) / c->alpha;
    const u64 *c0 = ct_in, *c1 = ct_in + (u64)level * N;
    u64 *c1c = (u64 *)malloc(sizeof(u64) * level * N);
    memcpy(c1c, c1, sizeof(u64) * level * N);
#pragma omp parallel for schedule(dynamic)
    for (int i = 0; i < level; i++) orc_intt(c, i, c1c + (u64)i * N);
    u64 *dig = (u64 *)malloc(sizeof(u64) * beta * W * N);
    for (int j = 0; j < beta; j++) orc_modup(c, level, j, c1c, dig + (u64)j * W * N);
#pragma omp parallel for schedule(dynamic)
    for (int jt = 0; jt < beta * W; jt++) orc_ntt(c, ext_limb(c, level, jt % W), dig + (u64)jt * N);
    free(c1c);
#pragma omp parallel for schedule(dynamic)
    for (int t = 0; t < W; t++) {
        int gl = ext_limb(c, level, t);
        u64 mt = c->mod[gl];
        u64 *perm = (u64 *)malloc(sizeof(u64) * N);
        for (int j = 0; j < beta; j++) {
            orc_automorph_ntt(c, g, dig + ((u64)j * W + t) * N, perm);
            for (int comp = 0; comp < 2; comp++) {
                const u64 *kk = key + (((u64)j * 2 + comp) * (L + K) + gl) * N;
                u64 *uu = u_acc + ((u64)comp * W + t) * N;
                for (u64 x = 0; x < N; x++) uu[x] = addmod(uu[x], mulmod(perm[x], kk[x], mt), mt);
            }
        }
        if (t < level) {
            orc_automorph_ntt(c, g, c0 + (u64)t * N, perm);
            for (u64 x = 0; x < N; x++) c0_acc[(u64)t * N + x] = addmod(c0_acc[(u64)t * N + x], perm[x], mt);
        }
        free(perm);
    }
    free(dig);
}

/* ------------------------------------------------------------------ */
/* plaintext handling                                                  */
/* ------------------------------------------------------------------ */
/* signed integer coefficient -> canonical residue */
static u64 reduce_signed(i64 v, u64 q) {
    if (v >= 0) return (u64)v % q;
    u64 r = ((u64)0 - (u64)v) % q; /* |v| mod q */
    return r ? q - r : 0;
}

/* int64 coefficient polynomial -> NTT-domain residues on limbs 0..level-1 */
void orc_expand_plain(const orc_ctx *c, int level, const i64 *coef, u64 *out) {
    u64 N = c->N;
    for (int i = 0; i < level; i++) {
        for (u64 x = 0; x < N; x++) out[(u64)i * N + x] = reduce_signed(coef[x], c->mod[i]);
        orc_ntt(c, i, out + (u64)i * N);
    }
}

/* ------------------------------------------------------------------ */
/* ct-pt projection (Sec. 3.2 with real packing: the imaginary term of the   */
/* complex weights in App. A.2.1 is dropped)                                  */
/* ------------------------------------------------------------------ */
/* x^(g), g < G at `level`; bank x^(g)_q = rot(x^(g); q*m), q < N1 (one hoisted
 * call per input; q = 0 is the input itself);
 *   acc_{b,p} = sum_g sum_q x^(g)_q (.) w_{b,p,g,q}
 *   y_b = acc_{b,0} + sum_{p>=1} rot(acc_{b,p}; p*N1*m)   (each a full key switch)
 *   y_b += conj(y_b)                                       (only if conj_key is given)
 *   conj_per_acc (variant, needs conj_key): acc_{b,p} += conj(acc_{b,p}) for every p before the giant step, in
 *   place of the line above: the order in which Sec. 3.2 writes the decomplexification.
 *   y_b.c0 += bias_b * bias_mul.
 * diag [B_out][N2][G][N1][N] int64 coefficient-domain encodings; bias
 * [B_out][N] int64 or NULL; baby_keys[q-1] for step q*m, giant_keys[p-1] for
 * step p*N1*m.  Only blocks b_first .. b_first+b_count-1 are computed and
 * written (at their own position in ct_y [B_out][2][level][N]). */
void orc_ctpt_matmul(const orc_ctx *c, int level, int m, int G, int B_out, int N1, int N2,
                     const i64 *diag, const i64 *bias, u64 bias_mul, const u64 *ct_x,
                     const u64 *const *baby_keys, const u64 *const *giant_keys, const u64 *conj_key, u64 *ct_y,
                     int b_first, int b_count, int merged, int conj_per_acc) {
    u64 N = c->N;
    u64 ctw = (u64)2 * level * N;
    (void)B_out;
    /* baby-step bank [G][N1][2][level][N] */
    u64 *bank = (u64 *)malloc(sizeof(u64) * G * N1 * ctw);
    u64 *gel = (u64 *)malloc(sizeof(u64) * (N1 > N2 ? N1 : N2));
    const u64 **kp = (const u64 **)malloc(sizeof(u64 *) * (N1 > N2 ? N1 : N2));
    for (int q = 0; q < N1; q++) {
        gel[q] = orc_galois_elt(c, (i64)q * m, 0);
        kp[q] = q ? baby_keys[q - 1] : NULL;
    }
    for (int g = 0; g < G; g++)
        orc_rotate_hoisted(c, ct_x + (u64)g * ctw, level, gel, N1, kp, bank + (u64)g * N1 * ctw);

    for (int b = b_first; b < b_first + b_count; b++) {
        u64 *acc = (u64 *)calloc((size_t)N2 * ctw, sizeof(u64)); /* [N2][2][level][N] */
#pragma omp parallel for schedule(dynamic)
        for (int p = 0; p < N2; p++) {
            u64 *w = (u64 *)malloc(sizeof(u64) * level * N);
            for (int g = 0; g < G; g++)
                for (int q = 0; q < N1; q++) {
                    const i64 *d = diag + ((((u64)b * N2 + p) * G + g) * N1 + q) * N;
                    orc_expand_plain(c, level, d, w);
                    const u64 *x = bank + ((u64)g * N1 + q) * ctw;
                    for (int comp = 0; comp < 2; comp++)
                        for (int i = 0; i < level; i++) {
                            u64 qi = c->mod[i];
                            u64 *a = acc + (u64)p * ctw + ((u64)comp * level + i) * N;
                            const u64 *xx = x + ((u64)comp * level + i) * N;
                            const u64 *ww = w + (u64)i * N;
                            for (u64 k = 0; k < N; k++) a[k] = addmod(a[k], mulmod(xx[k], ww[k], qi), qi);
                        }
                }
            free(w);
        }
        u64 *y = ct_y + (u64)b * ctw;
        u64 *rot = (u64 *)malloc(sizeof(u64) * ctw);
        /* decomplexification as Sec. 3.2 displays it: the real part of every giant-step accumulator is taken first,
         * c_p = (1/2)(c~_p + conj(c~_p)) with the 1/2 in the weights, and the fold over p follows.  N2 conjugations
         * per output block. */
        if (conj_key && conj_per_acc) {
            u64 g = orc_galois_elt(c, 0, 1);
            for (int p = 0; p < N2; p++) {
                u64 *a = acc + (u64)p * ctw;
                orc_rotate_hoisted(c, a, level, &g, 1, &conj_key, rot);
                for (int ci = 0; ci < 2 * level; ci++) {
                    u64 qi = c->mod[ci % level];
                    for (u64 k = 0; k < N; k++) a[(u64)ci * N + k] = addmod(a[(u64)ci * N + k], rot[(u64)ci * N + k], qi);
                }
            }
        }
        memcpy(y, acc, sizeof(u64) * ctw);
        if (!merged) {
            for (int p = 1; p < N2; p++) {
                u64 g = orc_galois_elt(c, (i64)p * N1 * m, 0);
                const u64 *key = giant_keys[p - 1];
                orc_rotate_hoisted(c, acc + (u64)p * ctw, level, &g, 1, &key, rot);
                for (int ci = 0; ci < 2 * level; ci++) {
                    u64 qi = c->mod[ci % level];
                    for (u64 k = 0; k < N; k++)
                        y[(u64)ci * N + k] = addmod(y[(u64)ci * N + k], rot[(u64)ci * N + k], qi);
                }
            }
        } else if (N2 > 1) {
            /* merged giant step (variant): the N2-1 switched accumulators are summed over the extended basis
             * and brought down by ONE ModDown per component:
             *   y_b = acc_{b,0} + (sum_p sigma_p(acc_{b,p}.c0), 0) + ModDown(sum_p sum_j sigma_p(d_j) key_{p,j}). */
            int Wl = level + c->K;
            u64 *u_acc = (u64 *)calloc((size_t)2 * Wl * N, sizeof(u64));
            u64 *c0_acc = (u64 *)calloc((size_t)level * N, sizeof(u64));
            for (int p = 1; p < N2; p++)
                orc_switch_accumulate(c, acc + (u64)p * ctw, level, orc_galois_elt(c, (i64)p * N1 * m, 0),
                                      giant_keys[p - 1], u_acc, c0_acc);
            orc_moddown(c, level, u_acc, rot);
            orc_moddown(c, level, u_acc + (u64)Wl * N, rot + (u64)level * N);
            for (int ci = 0; ci < 2 * level; ci++) {
                u64 qi = c->mod[ci % level];
                for (u64 k = 0; k < N; k++) {
                    u64 v = addmod(y[(u64)ci * N + k], rot[(u64)ci * N + k], qi);
                    if (ci < level) v = addmod(v, c0_acc[(u64)ci * N + k], qi);
                    y[(u64)ci * N + k] = v;
                }
            }
            free(c0_acc); free(u_acc);
        }
        /* decomplexification (Sec. 3.2): with complexified inputs x^(2u) + i x^(2u+1) and weights that carry
         * the factor 1/2, the real part is y + conj(y).  Taken once per output block after the giant-step fold,
         * the count of App. A.2.2 (#conj = O(B_out)). */
        if (conj_key && !conj_per_acc) {
            u64 g = orc_galois_elt(c, 0, 1);
            orc_rotate_hoisted(c, y, level, &g, 1, &conj_key, rot);
            for (int ci = 0; ci < 2 * level; ci++) {
                u64 qi = c->mod[ci % level];
                for (u64 k = 0; k < N; k++) y[(u64)ci * N + k] = addmod(y[(u64)ci * N + k], rot[(u64)ci * N + k], qi);
            }
        }
        free(rot);
        if (bias) {
            u64 *w = (u64 *)malloc(sizeof(u64) * level * N);
            orc_expand_plain(c, level, bias + (u64)b * N, w);
            for (int i = 0; i < level; i++) {
                u64 qi = c->mod[i];
                u64 bm = bias_mul % qi;
                for (u64 k = 0; k < N; k++)
                    y[(u64)i * N + k] = addmod(y[(u64)i * N + k], mulmod(w[(u64)i * N + k], bm, qi), qi);
            }
            free(w);
        }
        free(acc);
    }
    free(kp); free(gel); free(bank);
}

/* ------------------------------------------------------------------ */
/* rescale (Sec. 2.2: Q_i -> Q_{i-1} by dividing by the last prime)    */
/* ------------------------------------------------------------------ */
/* Reading: centred round-to-nearest.  r = INTT(c_last) in [0,q_last),
 * h = floor(q_last/2), r' = (r+h) mod q_last, and for i < level-1
 *   delta_i = (r' mod q_i - h mod q_i) mod q_i
 *   c_i <- (c_i - NTT_i(delta_i)) * [q_last^-1]_{q_i}.
 * ct_in [n_ct][2][level][N] -> ct_out [n_ct][2][level-1][N]. */
void orc_rescale(const orc_ctx *c, const u64 *ct_in, int level, int n_ct, u64 *ct_out) {
    u64 N = c->N;
    u64 ql = c->mod[level - 1], h = ql / 2;
#pragma omp parallel for schedule(dynamic)
    for (int pc = 0; pc < 2 * n_ct; pc++) {
        const u64 *in = ct_in + (u64)pc * level * N;
        u64 *out = ct_out + (u64)pc * (level - 1) * N;
        u64 *r = (u64 *)malloc(sizeof(u64) * N);
        u64 *d = (u64 *)malloc(sizeof(u64) * N);
        memcpy(r, in + (u64)(level - 1) * N, sizeof(u64) * N);
        orc_intt(c, level - 1, r);
        for (u64 x = 0; x < N; x++) r[x] = addmod(r[x], h, ql);
        for (int i = 0; i < level - 1; i++) {
            u64 qi = c->mod[i];
            u64 qlinv = invmod(ql % qi, qi);
            for (u64 x = 0; x < N; x++) d[x] = submod(r[x] % qi, h % qi, qi);
            orc_ntt(c, i, d);
            for (u64 x = 0; x < N; x++)
                out[(u64)i * N + x] = mulmod(submod(in[(u64)i * N + x], d[x], qi), qlinv, qi);
        }
        free(d); free(r);
    }
}

/* ------------------------------------------------------------------ */
/* add / ptmul / ModSwitchToNext / RotFirst                            */
/* ------------------------------------------------------------------ */
/* add of Table 1: limb-wise sum of n_ct pairs of ciphertexts, [n_ct][2][level][N]. */
void orc_add(const orc_ctx *c, const u64 *a, const u64 *b, int level, int n_ct, u64 *out) {
    u64 N = c->N;
    for (u64 row = 0; row < (u64)n_ct * 2 * level; row++) {
        u64 q = c->mod[row % level];
        for (u64 x = 0; x < N; x++) out[row * N + x] = addmod(a[row * N + x], b[row * N + x], q);
    }
}

/* ptmul of Table 1: both components times a plaintext given as NTT-domain residues pt [level][N]. */
void orc_ptmul(const orc_ctx *c, const u64 *ct, int level, const u64 *pt, u64 *out) {
    u64 N = c->N;
    for (int comp = 0; comp < 2; comp++)
        for (int i = 0; i < level; i++) {
            u64 q = c->mod[i];
            u64 off = ((u64)comp * level + i) * N;
            for (u64 x = 0; x < N; x++) out[off + x] = mulmod(ct[off + x], pt[(u64)i * N + x], q);
        }
}

/* ModSwitchToNext (Sec. 5.4): drop the last RNS prime without rescaling; the plaintext and its scale stay.
 * [n_ct][2][level][N] -> [n_ct][2][level-1][N]. */
void orc_mod_switch(const orc_ctx *c, const u64 *in, int level, int n_ct, u64 *out) {
    u64 N = c->N;
    for (int pc = 0; pc < 2 * n_ct; pc++)
        memcpy(out + (u64)pc * (level - 1) * N, in + (u64)pc * level * N, sizeof(u64) * (level - 1) * N);
}

/* RotFirst_L(x; tau) of App. A.1: cyclic left shift by tau inside the first L slots,
 *   rot(x; tau) (.) a  +  rot(x; (tau - L) mod n) (.) b,
 * with the masks a = 1{0 <= i < L - tau}, b = 1{L - tau <= i < L} handed over as expanded plaintexts
 * mask_a, mask_b [level][N].  The two rotations share their input (one hoisted decomposition).
 * gelts: the two Galois elements, keys: their keys (NULL where an element is 1). */
void orc_rot_first(const orc_ctx *c, const u64 *ct, int level, const u64 *gelts, const u64 *const *keys,
                   const u64 *mask_a, const u64 *mask_b, u64 *out) {
    u64 N = c->N;
    u64 ctw = (u64)2 * level * N;
    u64 *rot = (u64 *)malloc(sizeof(u64) * 2 * ctw);
    u64 *tmp = (u64 *)malloc(sizeof(u64) * ctw);
    orc_rotate_hoisted(c, ct, level, gelts, 2, keys, rot);
    orc_ptmul(c, rot, level, mask_a, out);
    orc_ptmul(c, rot + ctw, level, mask_b, tmp);
    orc_add(c, out, tmp, level, 1, out);
    free(tmp); free(rot);
}

/* Bank of masked rotation pairs from ONE input (Sec. 3.1 "rotation banks", App. A.1):
 *   out_i = rot(x; step_{i,0}) (.) mask_{i,0} + rot(x; step_{i,1}) (.) mask_{i,1},   i < n_out.
 * Psi^t (intra-segment shift), RotFirst_L and Phi_C^Delta are instances with their own masks and steps.
 * All 2*n_out rotations share the input's decomposition (hoisting).  gelts, keys: [n_out][2]; masks
 * [n_out][2][level][N] expanded plaintexts. */
void orc_shift_bank(const orc_ctx *c, const u64 *ct, int level, int n_out, const u64 *gelts, const u64 *const *keys,
                    const u64 *masks, u64 *out) {
    u64 N = c->N;
    u64 ctw = (u64)2 * level * N, ptw = (u64)level * N;
    u64 *rot = (u64 *)malloc(sizeof(u64) * 2 * n_out * ctw);
    u64 *tmp = (u64 *)malloc(sizeof(u64) * ctw);
    orc_rotate_hoisted(c, ct, level, gelts, 2 * n_out, keys, rot);
    for (int i = 0; i < n_out; i++) {
        orc_ptmul(c, rot + (u64)(2 * i) * ctw, level, masks + (u64)(2 * i) * ptw, out + (u64)i * ctw);
        orc_ptmul(c, rot + (u64)(2 * i + 1) * ctw, level, masks + (u64)(2 * i + 1) * ptw, tmp);
        orc_add(c, out + (u64)i * ctw, tmp, level, 1, out + (u64)i * ctw);
    }
    free(tmp); free(rot);
}

/* ------------------------------------------------------------------ */
/* client side used by the tests: keys, encryption, decryption         */
/* ------------------------------------------------------------------ */
/* s: ternary secret in {-1,0,1}^N.  Returns NTT(s) on every limb, [L+K][N]. */
static u64 *secret_ntt(const orc_ctx *c, const int8_t *s) {
    u64 N = c->N;
    int W = c->L + c->K;
    u64 *sn = (u64 *)malloc(sizeof(u64) * W * N);
#pragma omp parallel for schedule(dynamic)
    for (int i = 0; i < W; i++) {
        for (u64 x = 0; x < N; x++) sn[(u64)i * N + x] = reduce_signed((i64)s[x], c->mod[i]);
        orc_ntt(c, i, sn + (u64)i * N);
    }
    return sn;
}

/* Evaluation key that switches from the secret `target` to s (reading: hybrid key switching, dnum digits):
 *   b_j = -a_j*s + e_j + [P*T_j] * target,   key[j] = (b_j, a_j)
 * over all L+K limbs, NTT domain; [P*T_j] is P mod q_i on the limbs of digit j and 0 on every other limb.
 * a [dnum][L+K][N] are NTT-domain residues given by the caller; e [dnum][N] are small signed coefficients;
 * tg [L+K][N] is NTT(target). */
static void keygen_for_target(const orc_ctx *c, const u64 *sn, const u64 *tg, const u64 *a, const i64 *e, u64 *key) {
    u64 N = c->N;
    int L = c->L, K = c->K, W = L + K;
#pragma omp parallel for schedule(dynamic)
    for (int jt = 0; jt < c->dnum * W; jt++) {
        int j = jt / W, t = jt % W;
        u64 mt = c->mod[t];
        u64 *en = (u64 *)malloc(sizeof(u64) * N);
        for (u64 x = 0; x < N; x++) en[x] = reduce_signed(e[(u64)j * N + x], mt);
        orc_ntt(c, t, en);
        u64 f = 0;
        if (t < L && t / c->alpha == j) {
            f = 1;
            for (int k = 0; k < K; k++) f = mulmod(f, c->mod[L + k] % mt, mt);
        }
        const u64 *aj = a + ((u64)j * W + t) * N;
        u64 *kb = key + (((u64)j * 2 + 0) * W + t) * N;
        u64 *ka = key + (((u64)j * 2 + 1) * W + t) * N;
        for (u64 x = 0; x < N; x++) {
            u64 as = mulmod(aj[x], sn[(u64)t * N + x], mt);
            u64 v = submod(en[x], as, mt);
            v = addmod(v, mulmod(f, tg[(u64)t * N + x], mt), mt);
            kb[x] = v;
            ka[x] = aj[x];
        }
        free(en);
    }
}

/* Galois key for element g: target = sigma_g(s). */
void orc_galois_keygen(const orc_ctx *c, const int8_t *s, u64 g, const u64 *a, const i64 *e, u64 *key) {
    u64 N = c->N;
    int W = c->L + c->K;
    u64 *sn = secret_ntt(c, s);
    u64 *tg = (u64 *)malloc(sizeof(u64) * W * N);
    for (int t = 0; t < W; t++) orc_automorph_ntt(c, g, sn + (u64)t * N, tg + (u64)t * N);
    keygen_for_target(c, sn, tg, a, e, key);
    free(tg); free(sn);
}

/* Relinearisation key: target = s^2 (the degree-2 term of a ciphertext product, Table 1 ctmul). */
void orc_relin_keygen(const orc_ctx *c, const int8_t *s, const u64 *a, const i64 *e, u64 *key) {
    u64 N = c->N;
    int W = c->L + c->K;
    u64 *sn = secret_ntt(c, s);
    u64 *tg = (u64 *)malloc(sizeof(u64) * W * N);
    for (int t = 0; t < W; t++)
        for (u64 x = 0; x < N; x++) tg[(u64)t * N + x] = mulmod(sn[(u64)t * N + x], sn[(u64)t * N + x], c->mod[t]);
    keygen_for_target(c, sn, tg, a, e, key);
    free(tg); free(sn);
}

/* ctmul of Table 1: slotwise product of two ciphertexts at `level`, relinearised.
 *   (t0, t1, t2) = (a0*b0, a0*b1 + a1*b0, a1*b1)          pointwise in the NTT domain
 *   (v0, v1) = ModDown( sum_j d_j(t2) (.) key_j )           the same decomposition / ModDown as a rotation
 *   out = (t0 + v0, t1 + v1).                               scale(out) = scale(a)*scale(b): rescale next. */
void orc_ctmul(const orc_ctx *c, const u64 *ct_a, const u64 *ct_b, int level, const u64 *relin_key, u64 *out) {
    u64 N = c->N;
    int Wl = level + c->K;
    u64 *tmp = (u64 *)malloc(sizeof(u64) * 2 * level * N);     /* (t0, t2) laid out like a ciphertext */
    u64 *t1 = (u64 *)malloc(sizeof(u64) * level * N);
    for (int i = 0; i < level; i++) {
        u64 q = c->mod[i];
        const u64 *a0 = ct_a + (u64)i * N, *a1 = ct_a + ((u64)level + i) * N;
        const u64 *b0 = ct_b + (u64)i * N, *b1 = ct_b + ((u64)level + i) * N;
        for (u64 x = 0; x < N; x++) {
            tmp[(u64)i * N + x] = mulmod(a0[x], b0[x], q);
            tmp[((u64)level + i) * N + x] = mulmod(a1[x], b1[x], q);
            t1[(u64)i * N + x] = addmod(mulmod(a0[x], b1[x], q), mulmod(a1[x], b0[x], q), q);
        }
    }
    u64 *u_acc = (u64 *)calloc((size_t)2 * Wl * N, sizeof(u64));
    u64 *c0_acc = (u64 *)calloc((size_t)level * N, sizeof(u64));
    orc_switch_accumulate(c, tmp, level, 1, relin_key, u_acc, c0_acc);       /* g = 1: no automorphism */
    orc_moddown(c, level, u_acc, out);
    orc_moddown(c, level, u_acc + (u64)Wl * N, out + (u64)level * N);
    for (int i = 0; i < level; i++) {
        u64 q = c->mod[i];
        for (u64 x = 0; x < N; x++) {
            out[(u64)i * N + x] = addmod(out[(u64)i * N + x], c0_acc[(u64)i * N + x], q);
            out[((u64)level + i) * N + x] = addmod(out[((u64)level + i) * N + x], t1[(u64)i * N + x], q);
        }
    }
    free(c0_acc); free(u_acc); free(t1); free(tmp);
}

/* Symmetric encryption at `level`: c1 = a (NTT-domain residues, [level][N]),
 * c0 = -a*s + e + m, all stored in the NTT domain.  ct [2][level][N]. */
void orc_encrypt(const orc_ctx *c, int level, const i64 *m, const int8_t *s, const u64 *a, const i64 *e, u64 *ct) {
    u64 N = c->N;
    u64 *sn = secret_ntt(c, s);
#pragma omp parallel for schedule(dynamic)
    for (int i = 0; i < level; i++) {
        u64 qi = c->mod[i];
        u64 *me = (u64 *)malloc(sizeof(u64) * N);
        for (u64 x = 0; x < N; x++) me[x] = addmod(reduce_signed(m[x], qi), reduce_signed(e[x], qi), qi);
        orc_ntt(c, i, me);
        for (u64 x = 0; x < N; x++) {
            u64 as = mulmod(a[(u64)i * N + x], sn[(u64)i * N + x], qi);
            ct[(u64)i * N + x] = submod(me[x], as, qi);
            ct[((u64)level + i) * N + x] = a[(u64)i * N + x];
        }
        free(me);
    }
    free(sn);
}

/* c0 + c1*s on the first nlimbs limbs, returned in the coefficient domain,
 * out [nlimbs][N] canonical residues. */
void orc_decrypt(const orc_ctx *c, const u64 *ct, int level, const int8_t *s, int nlimbs, u64 *out) {
    u64 N = c->N;
    u64 *sn = secret_ntt(c, s);
#pragma omp parallel for schedule(dynamic)
    for (int i = 0; i < nlimbs; i++) {
        u64 qi = c->mod[i];
        for (u64 x = 0; x < N; x++)
            out[(u64)i * N + x] =
                addmod(ct[(u64)i * N + x], mulmod(ct[((u64)level + i) * N + x], sn[(u64)i * N + x], qi), qi);
        orc_intt(c, i, out + (u64)i * N);
    }
    free(sn);
}
