// Host side of a parameter set: validation of the modulus chain, roots of
// unity, twiddle tables and base-conversion tables (all uploaded in Montgomery
// form), and the private scratch arena.
#include <cstring>
#include <stdarg.h>
#include <stdio.h>

#include <algorithm>

#include "ckks_internal.h"

namespace ckks {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

int hip_fail(hipError_t e, const char *what) {
    set_error("HIP error %d (%s) in %s", (int)e, hipGetErrorString(e), what);
    return e == hipErrorOutOfMemory ? CKKS_E_NOMEM : CKKS_E_HIP;
}

typedef unsigned __int128 wide;

static u64 hmul(u64 a, u64 b, u64 q) { return (u64)((wide)a * b % q); }
static u64 hpow(u64 a, u64 e, u64 q) {
    u64 r = 1;
    a %= q;
    for (; e; e >>= 1) {
        if (e & 1) r = hmul(r, a, q);
        a = hmul(a, a, q);
    }
    return r;
}
static u64 hinv(u64 a, u64 q) { return hpow(a % q, q - 2, q); }

// Miller-Rabin with the witness set {2,3,5,7,11,13,17,19,23,29,31,37}, which is
// known to be exact below 3.3e24.
static bool is_prime(u64 n) {
    if (n < 2) return false;
    const u64 wit[] = {2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37};
    for (u64 w : wit) {
        if (n == w) return true;
        if (n % w == 0) return false;
    }
    u64 odd = n - 1;
    int twos = 0;
    while (!(odd & 1)) {
        odd >>= 1;
        ++twos;
    }
    for (u64 w : wit) {
        u64 x = hpow(w, odd, n);
        if (x == 1 || x == n - 1) continue;
        bool witness = true;
        for (int i = 1; i < twos && witness; ++i) {
            x = hmul(x, x, n);
            if (x == n - 1) witness = false;
        }
        if (witness) return false;
    }
    return true;
}

// Smallest psi with psi^N = -1 mod q: take any element of order exactly 2N and
// walk its odd powers.
static u64 smallest_root(u64 q, u32 logN) {
    u64 N = (u64)1 << logN, cof = (q - 1) >> (logN + 1);
    u64 base = 0;
    for (u64 cand = 2; cand < q; ++cand) {
        u64 r = hpow(cand, cof, q);
        if (hpow(r, N, q) == q - 1) {
            base = r;
            break;
        }
    }
    u64 sq = hmul(base, base, q), cur = base, best = base;
    for (u64 i = 1; i < N; ++i) {
        cur = hmul(cur, sq, q);
        best = std::min(best, cur);
    }
    return best;
}

static u32 bitrev(u32 x, u32 bits) {
    u32 r = 0;
    for (u32 i = 0; i < bits; ++i) r |= ((x >> i) & 1u) << (bits - 1 - i);
    return r;
}

static ModConst make_mod(u64 q) {
    ModConst m;
    m.q = q;
    u64 inv = q;  // Newton: correct to 3 bits, doubles each step
    for (int i = 0; i < 6; ++i) inv *= 2 - q * inv;
    m.qinv = inv;
    m.one = (u64)((((wide)1) << 64) % q);
    m.r2 = hmul(m.one, m.one, q);
    return m;
}

static u64 to_mont(u64 x, const ModConst &m) { return hmul(x % m.q, m.one, m.q); }
static u64 shoup(u64 w, u64 q) { return (u64)((((wide)w) << 64) / q); }   // floor(w * 2^64 / q), w < q

template <typename T>
static int upload(T **dst, const std::vector<T> &src) {
    *dst = nullptr;
    if (src.empty()) return CKKS_OK;
    CKKS_HIP(hipMalloc((void **)dst, src.size() * sizeof(T)));
    CKKS_HIP(hipMemcpy(*dst, src.data(), src.size() * sizeof(T), hipMemcpyHostToDevice));
    return CKKS_OK;
}

}  // namespace ckks

using namespace ckks;

// Grows the arena.  Every compute call's need at the sizes the *_create calls know about is reserved there
// (reserve_default, ckks_weights_create) or by ckks_params_reserve, so on the usual path this returns at its first
// line; a larger need is the documented exception: the stream is drained and the arena reallocated, which a
// capturing stream cannot do (the call then fails cleanly and asks for a reservation).
int ckks_params::ensure_scratch(size_t bytes, hipStream_t stream) {
    if (bytes <= scratch_bytes) return CKKS_OK;
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &cap) != hipSuccess) (void)hipGetLastError();
    if (cap != hipStreamCaptureStatusNone) {
        set_error("scratch arena of %zu bytes is too small for this call (%zu bytes) and the stream is capturing: "
                  "call ckks_params_reserve first", scratch_bytes, bytes);
        return CKKS_E_NOMEM;
    }
    if (d_scratch) {
        CKKS_HIP(hipStreamSynchronize(stream));
        CKKS_HIP(hipFree(d_scratch));
        d_scratch = nullptr;
        scratch_bytes = 0;
    }
    CKKS_HIP(hipMalloc(&d_scratch, bytes));
    scratch_bytes = bytes;
    return CKKS_OK;
}

// Conversion tables of every level are built by ckks_params_create; compute calls only look them up.
int ckks_params::level_tables(u32 level, const LevelTables **out) const {
    auto it = levels.find(level);
    if (it == levels.end()) {
        set_error("no conversion tables for level %u", level);
        return CKKS_E_LEVEL;
    }
    *out = &it->second;
    return CKKS_OK;
}

int ckks_params::build_level_tables(u32 level) {
    LevelTables t;
    t.level = level;
    t.beta = (level + alpha - 1) / alpha;
    u32 Wl = level + K;
    std::vector<u64> inv(level), mat((size_t)level * Wl, 0), matf((size_t)level * Wl, 0);
    for (u32 i = 0; i < level; ++i) {
        u32 lo = (i / alpha) * alpha, hi = std::min(lo + alpha, level);
        u64 qi = mod[i], prod = 1;
        for (u32 b = lo; b < hi; ++b)
            if (b != i) prod = hmul(prod, mod[b] % qi, qi);
        inv[i] = to_mont(hinv(prod, qi), hmod[i]);
        for (u32 t2 = 0; t2 < Wl; ++t2) {
            if (t2 >= lo && t2 < hi) continue;
            u32 gl = t2 < level ? t2 : L + (t2 - level);
            u64 mt = mod[gl], f = 1;
            for (u32 b = lo; b < hi; ++b)
                if (b != i) f = hmul(f, mod[b] % mt, mt);
            mat[(size_t)i * Wl + t2] = to_mont(f, hmod[gl]);
            const double fd = (double)f;      // exact below 2^53; read only for targets below 2^50
            std::memcpy(&matf[(size_t)i * Wl + t2], &fd, sizeof fd);
        }
    }
    // tables of the fused decomposition kernel
    std::vector<ModFp> modf_up(level);
    // per digit j and target row t (k for the special rows): the factors of the digit's up to 8 source limbs side
    // by side, zero where the digit is shorter (alpha above 8 does not use these tables)
    std::vector<double> mats((size_t)t.beta * K * 48, 0.0), ft((size_t)t.beta * Wl * 8, 0.0);
    for (u32 i = 0; i < level; ++i) {
        u32 lo = (i / alpha) * alpha, hi = std::min(lo + alpha, level);
        u64 qi = mod[i], prod = 1;
        for (u32 b = lo; b < hi; ++b)
            if (b != i) prod = hmul(prod, mod[b] % qi, qi);
        const u64 invp = hinv(prod, qi);
        ModFp f;
        f.q = (double)qi;
        f.u = 1.0 / (double)qi;
        f.ninv = (double)hmul(hninv[2 * i], invp, qi);
        f.ninv_w = (double)hmul(hninv[2 * i + 1], invp, qi);
        f.ok = (qi >> 50) == 0;
        f.pad = 0;
        modf_up[i] = f;
        const u32 dj = i / alpha, da = i - lo;
        if (da >= 8) continue;
        for (u32 k = 0; k < K; ++k) {
            u64 pk = mod[L + k], fk = 1;
            for (u32 b = lo; b < hi; ++b)
                if (b != i) fk = hmul(fk, mod[b] % pk, pk);
            for (u32 b = 0; b < 2; ++b) {
                u64 g = hmul(hmul(fk, hpow(2, 25 * b, pk), pk), hmod[L + k].one, pk);
                for (u32 c = 0; c < 3; ++c)
                    mats[((((size_t)dj * K + k) * 8 + da) * 2 + b) * 3 + c] = (double)((g >> (20 * c)) & 0xFFFFFu);
            }
        }
        for (u32 t2 = 0; t2 < level; ++t2) {
            if (t2 >= lo && t2 < hi) continue;
            u64 mt = mod[t2], fq = 1;
            for (u32 b = lo; b < hi; ++b)
                if (b != i) fq = hmul(fq, mod[b] % mt, mt);
            ft[((size_t)dj * Wl + t2) * 8 + da] = (double)fq;       // exact below 2^53; used for targets below 2^50
        }
    }
    // entered into the map first, so that ckks_params_destroy frees whatever part was uploaded if a later part fails
    LevelTables &slot = levels.emplace(level, t).first->second;
    int rc = upload(&slot.d_up_inv, inv);
    if (!rc) rc = upload(&slot.d_up_mat, mat);
    if (!rc) rc = upload(&slot.d_up_matf, matf);
    if (!rc) rc = upload(&slot.d_modf_up, modf_up);
    if (!rc) rc = upload(&slot.d_up_mats, mats);
    if (!rc) rc = upload(&slot.d_up_ft, ft);
    return rc;
}

extern "C" {

const char *ckks_last_error(void) { return ckks::g_err; }

int ckks_find_primes(uint32_t bits, uint32_t logN, uint32_t count, uint64_t *out) {
    if (!out || bits > 61 || bits < logN + 2 || logN < 1 || logN > 30) {
        set_error("ckks_find_primes: bad arguments (bits=%u logN=%u)", bits, logN);
        return CKKS_E_INVAL;
    }
    u64 step = (u64)2 << logN, top = (u64)1 << bits;
    u32 found = 0;
    for (u64 k = 1; found < count; ++k) {
        if (k * step >= top / 2) {
            set_error("ckks_find_primes: only %u primes of %u bits", found, bits);
            return CKKS_E_INVAL;
        }
        u64 c = top - k * step + 1;
        if (is_prime(c)) out[found++] = c;
    }
    return CKKS_OK;
}

int ckks_params_create(uint32_t logN, const uint64_t *q, uint32_t L, const uint64_t *p, uint32_t K,
                       uint32_t dnum, ckks_params_t **out) {
    if (!out) {
        set_error("ckks_params_create: out is null");
        return CKKS_E_INVAL;
    }
    *out = nullptr;
    if (!q || (K && !p) || L == 0 || dnum == 0) {
        set_error("ckks_params_create: null prime list or empty chain");
        return CKKS_E_INVAL;
    }
    if (logN < 10 || logN > 17) {
        set_error("ckks_params_create: logN=%u outside [10,17]", logN);
        return CKKS_E_INVAL;
    }
    if (L % dnum) {
        set_error("ckks_params_create: L=%u not divisible by dnum=%u", L, dnum);
        return CKKS_E_INVAL;
    }
    if (dnum > 16) {   // the key inner product sums dnum 124-bit products in 128 bits
        set_error("ckks_params_create: dnum=%u > 16", dnum);
        return CKKS_E_INVAL;
    }
    if (L + K > MAX_LIMBS || L / dnum > MAX_DIGIT || K > MAX_DIGIT) {
        set_error("ckks_params_create: L+K=%u > %u, or digit/special count > %u", L + K, MAX_LIMBS, MAX_DIGIT);
        return CKKS_E_INVAL;
    }
    u64 twoN = (u64)2 << logN;
    std::vector<u64> mod;
    for (u32 i = 0; i < L; ++i) mod.push_back(q[i]);
    for (u32 k = 0; k < K; ++k) mod.push_back(p[k]);
    for (size_t i = 0; i < mod.size(); ++i) {
        u64 v = mod[i];
        if (v >> 62 || v < twoN || v % twoN != 1 || !is_prime(v)) {
            set_error("ckks_params_create: modulus %zu (%llu) is not a prime < 2^62 that is 1 mod 2N", i,
                      (unsigned long long)v);
            return CKKS_E_INVAL;
        }
        for (size_t j = 0; j < i; ++j)
            if (mod[j] == v) {
                set_error("ckks_params_create: modulus %llu listed twice", (unsigned long long)v);
                return CKKS_E_INVAL;
            }
    }
    // lazy sums of alpha (or K) products must stay below 2^64 * target modulus
    u64 maxq = *std::max_element(mod.begin(), mod.end());
    u32 terms = std::max(L / dnum, K);
    if ((wide)terms * maxq >= ((wide)1 << 64)) {
        set_error("ckks_params_create: digit size %u too large for %llu-sized primes", terms, (unsigned long long)maxq);
        return CKKS_E_INVAL;
    }

    ckks_params *P = new ckks_params();
    P->logN = logN;
    P->N = 1u << logN;
    P->L = L;
    P->K = K;
    P->dnum = dnum;
    P->alpha = L / dnum;
    P->W = L + K;
    P->mod = mod;
    hipGetDevice(&P->device);
    u32 N = P->N, W = P->W;
    for (u64 v : mod) {
        P->hmod.push_back(make_mod(v));
        P->psi.push_back(smallest_root(v, logN));
    }
    std::vector<u64> fwd((size_t)W * N, 0), inv((size_t)W * N, 0), ninv((size_t)W * 2);
    std::vector<u64> pw(2 * (size_t)N);
    std::vector<double> fwd_f((size_t)W * N, 0.0), inv_f((size_t)W * N, 0.0);
    std::vector<ModFp> modf(W);
    std::vector<u64> ninv_plain((size_t)W * 2);
    const bool two_pass = logN == 16 || logN == 12;
    std::vector<u64> fwd_s, inv_s;
    if (two_pass) {
        fwd_s.assign((size_t)W * N * 2, 0);
        inv_s.assign((size_t)W * N * 2, 0);
    }
    for (u32 i = 0; i < W; ++i) {
        const ModConst &m = P->hmod[i];
        pw[0] = 1;
        for (u32 e = 1; e < 2 * N; ++e) pw[e] = hmul(pw[e - 1], P->psi[i], m.q);
        for (u32 idx = 1; idx < N; ++idx) {
            u32 e = bitrev(idx, logN);
            fwd[(size_t)i * N + idx] = to_mont(pw[e], m);
            inv[(size_t)i * N + idx] = to_mont(pw[2 * N - e], m);
        }
        u64 ni = hinv(N % m.q, m.q);
        ninv_plain[2 * i] = ni;
        ninv_plain[2 * i + 1] = hmul(ni, pw[2 * N - N / 2], m.q);
        ninv[2 * i] = to_mont(ni, m);
        ninv[2 * i + 1] = to_mont(hmul(ni, pw[2 * N - N / 2], m.q), m);
        // primes below 2^50 also get plain-integer twiddles as doubles for the FMA butterflies
        ModFp f;
        f.q = (double)m.q;
        f.u = 1.0 / (double)m.q;
        f.ninv = (double)ni;
        f.ninv_w = (double)hmul(ni, pw[2 * N - N / 2], m.q);
        f.ok = (m.q >> 50) == 0;
        f.pad = 0;
        modf[i] = f;
        if (f.ok)
            for (u32 idx = 1; idx < N; ++idx) {
                u32 e = bitrev(idx, logN);
                fwd_f[(size_t)i * N + idx] = (double)pw[e];
                inv_f[(size_t)i * N + idx] = (double)pw[2 * N - e];
            }
        else if (two_pass)
            for (u32 idx = 1; idx < N; ++idx) {
                u32 e = bitrev(idx, logN);
                const size_t o = ((size_t)i * N + idx) * 2;
                fwd_s[o] = pw[e];
                fwd_s[o + 1] = shoup(pw[e], m.q);
                inv_s[o] = pw[2 * N - e];
                inv_s[o + 1] = shoup(pw[2 * N - e], m.q);
            }
    }
    std::vector<u64> ninvs((size_t)W * 4);
    for (u32 i = 0; i < W; ++i)
        for (u32 z = 0; z < 2; ++z) {
            ninvs[4 * i + 2 * z] = ninv_plain[2 * i + z];
            ninvs[4 * i + 2 * z + 1] = shoup(ninv_plain[2 * i + z], mod[i]);
        }
    P->hninv = ninv_plain;
    std::vector<u64> dn_inv(K), dn_mat((size_t)K * L), pinv(L), qlinv((size_t)L * L, 0);
    std::vector<double> dn_matf((size_t)L * K * 6, 0.0), pinvf(L, 0.0);
    for (u32 k = 0; k < K; ++k) {
        u64 pk = mod[L + k], prod = 1;
        for (u32 b = 0; b < K; ++b)
            if (b != k) prod = hmul(prod, mod[L + b] % pk, pk);
        dn_inv[k] = to_mont(hinv(prod, pk), P->hmod[L + k]);
        for (u32 i = 0; i < L; ++i) {
            u64 f = 1;
            for (u32 b = 0; b < K; ++b)
                if (b != k) f = hmul(f, mod[L + b] % mod[i], mod[i]);
            dn_mat[(size_t)k * L + i] = to_mont(f, P->hmod[i]);
            // the same factor times 2^0, 2^20, 2^40 mod q_i, each split into 25-bit halves held as doubles: the
            // conversion onto a prime below 2^50 is then a sum of exact 20-bit x 25-bit products in fp64
            for (u32 a = 0; a < 3; ++a) {
                const u64 c = hmul(f, hpow(2, 20 * a, mod[i]), mod[i]);
                dn_matf[(((size_t)i * K + k) * 3 + a) * 2 + 0] = (double)(c & ((1u << 25) - 1));
                dn_matf[(((size_t)i * K + k) * 3 + a) * 2 + 1] = (double)(c >> 25);
            }
        }
    }
    P->dn_fp = true;          // three 20-bit pieces cover a special prime below 2^60
    for (u32 k = 0; k < K; ++k)
        if (mod[L + k] >> 60) P->dn_fp = false;
    for (u32 i = 0; i < L; ++i) {
        u64 pm = 1;
        for (u32 k = 0; k < K; ++k) pm = hmul(pm, mod[L + k] % mod[i], mod[i]);
        pinv[i] = to_mont(hinv(pm, mod[i]), P->hmod[i]);
        pinvf[i] = (double)hinv(pm, mod[i]);
        for (u32 l = 0; l < L; ++l)
            if (l != i) qlinv[(size_t)l * L + i] = to_mont(hinv(mod[l] % mod[i], mod[i]), P->hmod[i]);
    }
    // INTT constants of the special limbs with (P/p_k)^-1 folded in: the ModDown of a key switch then reads
    // y_k = INTT(u_{p_k}) * (P/p_k)^-1 straight from the transform
    std::vector<u64> ninv_dn = ninv, ninvs_dn = ninvs;
    std::vector<ModFp> modf_dn = modf;
    for (u32 k = 0; k < K; ++k) {
        const ModConst &m = P->hmod[L + k];
        u64 pk = mod[L + k], prod = 1;
        for (u32 b = 0; b < K; ++b)
            if (b != k) prod = hmul(prod, mod[L + b] % pk, pk);
        u64 f = hinv(prod, pk);
        u64 n0 = hmul(ninv_plain[2 * (L + k)], f, pk), n1 = hmul(ninv_plain[2 * (L + k) + 1], f, pk);
        ninv_dn[2 * (L + k)] = to_mont(n0, m);
        ninv_dn[2 * (L + k) + 1] = to_mont(n1, m);
        ninvs_dn[4 * (L + k)] = n0;
        ninvs_dn[4 * (L + k) + 1] = shoup(n0, pk);
        ninvs_dn[4 * (L + k) + 2] = n1;
        ninvs_dn[4 * (L + k) + 3] = shoup(n1, pk);
        modf_dn[L + k].ninv = (double)n0;
        modf_dn[L + k].ninv_w = (double)n1;
    }
    int rc = upload(&P->d_mod, P->hmod);
    if (!rc) rc = upload(&P->d_ninv_dn, ninv_dn);
    if (!rc) rc = upload(&P->d_modf_dn, modf_dn);
    if (!rc) rc = upload(&P->d_tw_fwd, fwd);
    if (!rc) rc = upload(&P->d_tw_inv, inv);
    if (!rc) rc = upload(&P->d_ninv, ninv);
    if (!rc) rc = upload(&P->d_modf, modf);
    if (!rc) rc = upload(&P->d_twf_fwd, fwd_f);
    if (!rc) rc = upload(&P->d_twf_inv, inv_f);
    if (!rc) rc = upload(&P->d_dn_inv, dn_inv);
    if (!rc) rc = upload(&P->d_dn_mat, dn_mat);
    if (!rc) rc = upload(&P->d_dn_matf, dn_matf);
    if (!rc) rc = upload(&P->d_pinv, pinv);
    if (!rc) rc = upload(&P->d_pinvf, pinvf);
    if (!rc) rc = upload(&P->d_qlinv, qlinv);
    if (!rc) rc = upload(&P->d_tws_fwd, fwd_s);
    if (!rc) rc = upload(&P->d_tws_inv, inv_s);
    if (!rc) rc = upload(&P->d_ninvs, ninvs);
    if (!rc) rc = upload(&P->d_ninvs_dn, ninvs_dn);
    for (u32 level = 1; !rc && level <= L && K; ++level) rc = P->build_level_tables(level);
    // scratch for every call whose need is known from the parameter set alone: a full batch of hoisted key switches
    // at the top level (ckks_rotate_hoisted with any number of steps, ckks_ctmul, ckks_rot_first, the key holder's
    // calls), ckks_rescale of up to 64 ciphertexts, ckks_encode / ckks_decode
    if (!rc) {
        size_t words = (size_t)128 * N + 4 * (size_t)W * N;                   // rescale; encode: 64 complex vectors
        words = std::max(words, (size_t)64 * 2 * N);
        words = std::max(words, (size_t)dnum * W * N + W);                    // key generation
        if (K) words = std::max(words, (size_t)ROT_BATCH * 2 * L * N + rotate_hoisted_scratch_words(P, L, ROT_BATCH));   // ckks_shift_bank
        rc = P->ensure_scratch(words * sizeof(u64), nullptr);
    }
    if (rc) {
        ckks_params_destroy(P);
        return rc;
    }
    *out = P;
    return CKKS_OK;
}

int ckks_params_reserve(ckks_params_t *P, uint64_t bytes) {
    if (!P) {
        set_error("ckks_params_reserve: params is null");
        return CKKS_E_INVAL;
    }
    CKKS_HIP(hipDeviceSynchronize());
    return P->ensure_scratch((size_t)bytes, nullptr);
}

int ckks_params_scratch_bytes(const ckks_params_t *P, uint64_t *bytes) {
    if (!P || !bytes) {
        set_error("ckks_params_scratch_bytes: null argument");
        return CKKS_E_INVAL;
    }
    *bytes = P->scratch_bytes;
    return CKKS_OK;
}

void ckks_params_destroy(ckks_params_t *P) {
    if (!P) return;
    hipFree(P->d_mod);
    hipFree(P->d_tw_fwd);
    hipFree(P->d_tw_inv);
    hipFree(P->d_ninv);
    hipFree(P->d_modf);
    hipFree(P->d_ninv_dn);
    hipFree(P->d_modf_dn);
    hipFree(P->d_twf_fwd);
    hipFree(P->d_twf_inv);
    hipFree(P->d_dn_inv);
    hipFree(P->d_dn_mat);
    hipFree(P->d_dn_matf);
    hipFree(P->d_pinv);
    hipFree(P->d_pinvf);
    hipFree(P->d_qlinv);
    hipFree(P->d_tws_fwd);
    hipFree(P->d_tws_inv);
    hipFree(P->d_ninvs);
    hipFree(P->d_ninvs_dn);
    for (auto &kv : P->levels) {
        hipFree(kv.second.d_up_inv);
        hipFree(kv.second.d_up_mat);
        hipFree(kv.second.d_up_matf);
        hipFree(kv.second.d_modf_up);
        hipFree(kv.second.d_up_mats);
        hipFree(kv.second.d_up_ft);
    }
    hipFree(P->d_fft_w);
    hipFree(P->d_fft_twist);
    hipFree(P->d_slot_bin);
    hipFree(P->d_scratch);
    for (hipEvent_t ev : P->prof_ev) hipEventDestroy(ev);
    delete P;
}

int ckks_params_root(const ckks_params_t *P, uint32_t limb, uint64_t *psi) {
    if (!P || !psi || limb >= P->W) {
        set_error("ckks_params_root: bad arguments");
        return CKKS_E_INVAL;
    }
    *psi = P->psi[limb];
    return CKKS_OK;
}

int ckks_galois_elt(const ckks_params_t *P, int32_t step, uint64_t *g) {
    if (!P || !g) {
        set_error("ckks_galois_elt: null argument");
        return CKKS_E_INVAL;
    }
    u64 twoN = 2ull * P->N;
    if (step == CKKS_STEP_CONJ) {
        *g = twoN - 1;
        return CKKS_OK;
    }
    int64_t n = P->N / 2, r = ((int64_t)step % n + n) % n;
    *g = hpow(5, (u64)r, twoN);   // 2N is not prime, but square-and-multiply needs no inverse
    return CKKS_OK;
}

}  // extern "C"
