// Internal declarations shared by the library's translation units.
#pragma once
#include <hip/hip_runtime.h>

#include <map>
#include <string>
#include <vector>

#include "../../include/ckks_measure.h"   // includes ckks.h
#include "modarith.h"

namespace ckks {

constexpr u32 MAX_LIMBS = 64;     // L + K
constexpr u32 MAX_DIGIT = 16;     // alpha and K
constexpr u32 ROT_BATCH = 32;     // key switches per batch of kernel launches
constexpr u32 SKIP_ROW = 255;     // limb id meaning "leave this row alone"

constexpr u32 MAX_ROW_IDS = 128;  // rows described by one LimbIds pattern

// limb id of each row of a [batch][n][N] array, row index taken modulo n
struct LimbIds {
    uint8_t id[MAX_ROW_IDS];
};

// fp64 view of a modulus below 2^50: residues, twiddles and products are exact integers in doubles
struct ModFp {
    double q, u;           // q and its rounded reciprocal
    double ninv, ninv_w;   // N^-1 and N^-1 * psi^-(N/2) as plain integers
    u32 ok, pad;           // 1 if q < 2^50 (the FMA butterflies apply)
};

// Half-open device ranges [a, a + na) and [b, b + nb) of 64-bit words share a word.
inline bool words_overlap(const void *a, size_t na, const void *b, size_t nb) {
    const uintptr_t a0 = (uintptr_t)a, a1 = a0 + na * sizeof(u64), b0 = (uintptr_t)b, b1 = b0 + nb * sizeof(u64);
    return na && nb && a0 < b1 && b0 < a1;
}

void set_error(const char *fmt, ...);
int hip_fail(hipError_t e, const char *what);

#define CKKS_HIP(call)                                        \
    do {                                                      \
        hipError_t e_ = (call);                               \
        if (e_ != hipSuccess) return hip_fail(e_, #call);     \
    } while (0)

#define CKKS_LAUNCH_CHECK(name)                               \
    do {                                                      \
        hipError_t e_ = hipGetLastError();                    \
        if (e_ != hipSuccess) return hip_fail(e_, name);      \
    } while (0)

// Base-conversion tables of one level (digits depend on the level only through
// the last, possibly partial, digit).
struct LevelTables {
    u32 level = 0, beta = 0;
    u64 *d_up_inv = nullptr;   // [level]: ((Q_D/q_i)^-1 mod q_i), Montgomery form, D = digit of i
    u64 *d_up_mat = nullptr;   // [level][level+K]: (Q_D/q_i mod t), Montgomery form w.r.t. t; 0 for t in D
    u64 *d_up_matf = nullptr;  // the same factors as doubles (bit patterns), for the conversions done in fp64
    // for the fused decomposition kernel (N = 2^16, every active prime below 2^50):
    ModFp *d_modf_up = nullptr;   // [level]: the limb's ModFp with (Q_D/q_i)^-1 folded into the inverse transform's N^-1
    double *d_up_mats = nullptr;  // [beta][K][8][2][3]: (Q_D/q_i) 2^(25b) 2^64 mod p_k cut into three 20-bit parts
    double *d_up_ft = nullptr;    // [beta][level+K][8]: (Q_D/q_i) mod q_t for the ciphertext-prime targets t
};

}  // namespace ckks

struct ckks_params {
    ckks::u32 logN = 0, N = 0, L = 0, K = 0, dnum = 0, alpha = 0, W = 0;
    int device = 0;
    std::vector<ckks::u64> mod, psi;
    std::vector<ckks::ModConst> hmod;
    std::vector<ckks::u64> hninv;      // [W][2]: N^-1 and N^-1 * psi^-(N/2) as plain residues
    ckks::ModConst *d_mod = nullptr;   // [W]
    ckks::u64 *d_tw_fwd = nullptr;     // [W][N]: psi^bitrev(idx), Montgomery form, idx in [1, N)
    ckks::u64 *d_tw_inv = nullptr;     // [W][N]: psi^-bitrev(idx), Montgomery form
    ckks::u64 *d_ninv = nullptr;       // [W][2]: N^-1 and N^-1 * psi^-(N/2), Montgomery form
    ckks::ModFp *d_modf = nullptr;     // [W]
    ckks::u64 *d_ninv_dn = nullptr;    // like d_ninv, special limbs scaled by (P/p_k)^-1
    // the same constants for the lazy integer butterflies of the two-pass kernels (N = 2^12, 2^16): plain values paired
    // with their quotients floor(w * 2^64 / q); rows of limbs below 2^50 (fp64 butterflies) are left zero
    ckks::u64 *d_tws_fwd = nullptr;    // [W][N][2]
    ckks::u64 *d_tws_inv = nullptr;    // [W][N][2]
    ckks::u64 *d_ninvs = nullptr;      // [W][4]
    ckks::u64 *d_ninvs_dn = nullptr;   // [W][4], special limbs scaled by (P/p_k)^-1
    ckks::ModFp *d_modf_dn = nullptr;  // like d_modf, special limbs scaled by (P/p_k)^-1
    double *d_twf_fwd = nullptr;       // [W][N]: psi^bitrev(idx) as a double (limbs below 2^50 only)
    double *d_twf_inv = nullptr;       // [W][N]
    // ModDown tables (independent of the level)
    ckks::u64 *d_dn_inv = nullptr;     // [K]: (P/p_k)^-1 mod p_k
    ckks::u64 *d_dn_mat = nullptr;     // [K][L]: P/p_k mod q_i
    double *d_dn_matf = nullptr;       // [L][K][3][2]: (2^(20a) * P/p_k) mod q_i as two 25-bit halves (doubles)
    bool dn_fp = false;                // every special prime below 2^60: the fp64 ModDown conversion applies
    ckks::u64 *d_pinv = nullptr;       // [L]: P^-1 mod q_i
    double *d_pinvf = nullptr;         // [L]: the same as plain doubles (exact for primes below 2^53)
    ckks::u64 *d_qlinv = nullptr;      // [L][L]: q_l^-1 mod q_i (rescale), row l
    std::map<ckks::u32, ckks::LevelTables> levels;
    // complex-slot encode / decode (built on first use): exp(-2*pi*i*e/N), e < N/2; exp(-i*pi*k/N), k < N; and the
    // transform bin (5^j mod 2N - 1)/2 of slot j
    double *d_fft_w = nullptr, *d_fft_twist = nullptr;
    ckks::u32 *d_slot_bin = nullptr;
    // private scratch arena
    void *d_scratch = nullptr;
    size_t scratch_bytes = 0;

    // optional timing of the diagonal multiply-accumulate kernel (ckks_profile_*)
    bool prof_on = false;
    std::vector<hipEvent_t> prof_ev;   // start/stop pairs
    size_t prof_used = 0;
    mutable uint64_t limb_ntts = 0;    // limb transforms launched so far (for the operation counters)

    int ensure_scratch(size_t bytes, hipStream_t stream);
    int level_tables(ckks::u32 level, const ckks::LevelTables **out) const;
    int build_level_tables(ckks::u32 level);
};

struct ckks_gkey {
    const ckks_params *params = nullptr;
    ckks::u64 galois_elt = 0;
    ckks::u64 *d_key = nullptr;        // [dnum][2][L+K][N], Montgomery form
    bool owned = true;                 // false: the caller's buffer, converted in place (ckks_galois_key_adopt)
};

struct ckks_weights {
    const ckks_params *params = nullptr;
    ckks::u32 level = 0, m = 0, C = 0, G = 0, B_out = 0, N1 = 0, N2 = 0;
    // Diagonals, NTT domain, index ((b*N2 + p)*G + g)*N1 + q.  Two stores, each allocated when first needed:
    // d_w  [diagonal][level][N] words: per limb a double (q < 2^50) or Montgomery form;
    // d_wp [diagonal][level] packed half-limb records of 50-bit residues, for output blocks whose diagonals all
    //      encode real slot vectors when every active prime is below 2^50 (block_packed).
    ckks::u64 *d_w = nullptr;
    unsigned char *d_wp = nullptr;
    unsigned char *d_wpf = nullptr;    // [diagonal][level] packed whole-limb records: general diagonals, same condition
    ckks::u64 *d_stage = nullptr;      // expansion buffer of the packed store (STAGE_DIAGS diagonals)
    bool packable = false;             // every active prime below 2^50 and N large enough for the palindrome kernel
    ckks::u64 *d_bias = nullptr;       // [B_out][level][N], NTT domain, canonical, times bias_mul; or null
    // per (output block b, input group g), index b*G + g: every diagonal loaded so far encodes a real slot vector;
    // and where the group's diagonals live: 0 = d_w, 1 = half records in d_wp (real), 2 = whole-limb records in d_wpf
    std::vector<uint8_t> block_real;
    std::vector<uint8_t> block_packed;
    std::vector<uint8_t> loaded;       // per diagonal: ckks_weights_set_diagonals has stored it
    ckks::u32 *d_flag = nullptr;       // per-diagonal check results of the chunk being loaded
    ckks::u32 flag_cap = 0;
};

namespace ckks {

// ntt.hip
// pass_mask: bit 0 = the pass that runs first, bit 1 = the pass that runs second (3 = whole transform);
// scaled_dn: inverse only, folds (P/p_k)^-1 into the output of the special limbs.
int launch_ntt(const ckks_params *p, u64 *d_data, const LimbIds &ids, u32 n_limbs, u32 rows, bool inverse,
               hipStream_t stream, u32 pass_mask = 3, bool scaled_dn = false);
inline bool fast_ring(const ckks_params *p) { return p->logN == 16 || p->logN == 12; }

// keyswitch.hip
struct SwitchItem {
    const u64 *digits;   // [beta][level+K][N] extended digits of the source c1, NTT domain; the rows of a digit's own
                         // limbs are NOT filled: they equal the source's own rows and are read from c1
    const u64 *c1;       // [level][N] the decomposed polynomial itself (NTT domain); must outlive the switch
    const u64 *c0;       // [level][N] source c0
    const u64 *key;      // Montgomery-form key
    u64 *dst;            // [2][level][N]
    u64 galois_elt;
    u32 accumulate;      // add into dst instead of overwriting
};
size_t digits_words(const ckks_params *p, u32 level);
size_t switch_scratch_words(const ckks_params *p, u32 level, u32 n_items);
int decompose(ckks_params *p, const u64 *const *c1, u32 n, u32 level, u64 *d_digits, u64 *d_tmp, hipStream_t stream);
int switch_batch(ckks_params *p, u32 level, const SwitchItem *items, u32 n, u64 *d_work, hipStream_t stream);
int moddown_add(ckks_params *p, u32 level, u64 *d_u, u64 *const *dst, u32 n, u64 *d_w, hipStream_t stream);
int moddown_rescale(ckks_params *p, u32 level, u64 *d_u, const u64 *const *z, u64 *const *out, u32 n, u64 *d_w,
                    u64 *d_t, hipStream_t stream);
// Several rotations of n ciphertexts each, summed over the extended basis in one pass:
//   u_r (+)= sum_i sum_j sigma_{g_i}(digits_{i,r,j}) * key_{i,j},   dst_r.c0 += sum_i sigma_{g_i}(c0_{i,r}),
// r < n <= ROT_BATCH, i < n_rot <= MERGE_GROUP.  digits of (i, r) at d_digits + (i*n + r)*digits_words;
// c0 of (i, r) at c0_base + r*c0_stride_r + c0_off[i], its c1 (the decomposed polynomial) level*N words behind it;
// dst_r at dst_base + r*dst_stride.
constexpr u32 MERGE_GROUP = 8;
struct MergedRot {
    const u64 *key[MERGE_GROUP];
    u64 galois_elt[MERGE_GROUP];
    size_t c0_off[MERGE_GROUP];
    u32 n_rot;
};
int switch_accumulate_merged(ckks_params *p, u32 level, const MergedRot &rots, u32 n, const u64 *d_digits,
                             const u64 *c0_base, size_t c0_stride_r, u64 *dst_base, size_t dst_stride, u64 *d_u,
                             bool accumulate, hipStream_t stream);
// hoisted rotations of one ciphertext; the first reserve_words of the scratch arena are left to the caller
size_t rotate_hoisted_scratch_words(const ckks_params *p, u32 level, u32 n_steps);
int rotate_hoisted(ckks_params *p, const u64 *d_ct_in, u32 level, const int32_t *steps, u32 n_steps,
                   const ckks_gkey *const *keys, u64 *d_ct_out, size_t reserve_words, hipStream_t stream);

// matmul.hip
size_t matmul_scratch_words(const ckks_params *p, const ckks_weights *w, bool merged);
// int64 coefficients [count][N] -> NTT-domain residues [count][level][N]; weight_form: doubles / Montgomery per limb
int expand_plain(const ckks_params *p, u32 level, const int64_t *d_coeffs, u32 count, u64 *d_out, bool weight_form,
                 hipStream_t stream);

}  // namespace ckks
