// Negacyclic NTT / INTT over the RNS limbs.
//
// out[k] = a(psi^(2*bitrev(k)+1)): the transform splits X^(2t) - psi^(2e) into
// (X^t - psi^e)(X^t + psi^e) stage by stage; stage s has 2^s nodes and node i
// uses the twiddle psi^bitrev(2^s + i).  A polynomial of N = 2^16 residues
// (512 KiB) does not fit LDS, so the stages are cut into two passes over HBM:
//   pass A: the first stages.  Elements that interact there share their index
//           modulo N/2^a; global accesses stay runs of consecutive residues.
//   pass B: the remaining stages act inside aligned runs of consecutive
//           residues; a workgroup owns 4096 of them.
// The inverse runs pass B then pass A with Gentleman-Sande butterflies and folds
// N^-1 into the last stage.
//
// Two implementations:
//  * N = 2^12 and N = 2^16 (the benchmark rings): every thread keeps 16 residues in
//    registers and does four stages (radix 16) between exchanges through LDS.
//    Pass B covers 12 stages (three rounds, two exchanges) on a 4096-residue tile:
//    the whole transform at N = 2^12, all but the first 4 stages at N = 2^16.
//    Those 4 stages (pass A) pair residues 4096 apart, so a thread that owns a
//    column holds its 16 rows in registers and needs no LDS at all -- which is what
//    lets the base conversions of key switching, which work column by column in the
//    coefficient domain, carry the neighbouring pass A of both transforms.  Limbs whose prime is
//    below 2^50 run their butterflies in fp64: residues, twiddles and the two halves
//    of a product (a*w = h + l exactly, by FMA) are exact integers in doubles, the
//    quotient comes from one multiplication by 1/q, and values stay signed and
//    unreduced for up to four stages (about 10 issue slots per butterfly instead of
//    about 55 for the 64-bit Montgomery butterfly).  Larger primes (the 60-bit
//    special primes) use Montgomery butterflies in the same kernels.
//  * other ring sizes: a plain kernel with one LDS round trip per stage.
#include <algorithm>

#include "ckks_internal.h"
#include "ntt_device.h"

namespace ckks {

constexpr u32 NTT_TILE_LOG = 12;

// strided != 0: pass A layout, local element (x, lo) = (e / LT, e % LT) sits at
//   x * (N >> a) + blockIdx.x * LT + lo   with LT = T >> a.
// strided == 0: pass B layout, local element e sits at blockIdx.x * T + e.
template <bool INV>
__global__ __launch_bounds__(NTT_THREADS) void ntt_pass_kernel(u64 *__restrict__ data,
                                                               const ModConst *__restrict__ mods,
                                                               const u64 *__restrict__ tw,
                                                               const u64 *__restrict__ ninv, LimbIds ids,
                                                               u32 n_limbs, u32 logN, u32 s_lo, u32 s_hi,
                                                               u32 tile_log, u32 strided) {
    extern __shared__ u64 lds[];
    const u32 row = blockIdx.y;
    const u32 limb = ids.id[row % n_limbs];
    if (limb == SKIP_ROW) return;
    const ModConst m = mods[limb];
    const u32 N = 1u << logN, T = 1u << tile_log;
    u64 *poly = data + (size_t)row * N;
    const u64 *twl = tw + (size_t)limb * N;
    const u32 a = s_hi;                       // pass A always covers stages [0, a)
    const u32 lt_log = tile_log - a;          // only meaningful when strided
    const u32 base = blockIdx.x << (strided ? lt_log : tile_log);

    for (u32 e = threadIdx.x; e < T; e += NTT_THREADS) {
        size_t gi = strided ? ((size_t)(e >> lt_log) << (logN - a)) + base + (e & ((1u << lt_log) - 1)) : base + e;
        lds[e] = poly[gi];
    }
    __syncthreads();

    const u32 n_st = s_hi - s_lo;
    for (u32 st = 0; st < n_st; ++st) {
        const u32 s = INV ? s_hi - 1 - st : s_lo + st;
        // local gap between the two legs of a butterfly
        const u32 gap_log = strided ? tile_log - 1 - s : logN - 1 - s;
        const u32 node0 = strided ? 0 : base >> (logN - s);
        for (u32 bf = threadIdx.x; bf < T / 2; bf += NTT_THREADS) {
            const u32 grp = bf >> gap_log, j = bf & ((1u << gap_log) - 1);
            const u32 i0 = (grp << (gap_log + 1)) + j, i1 = i0 + (1u << gap_log);
            const u64 w = twl[(1u << s) + node0 + grp];
            u64 x = lds[i0], y = lds[i1];
            if (!INV) {
                u64 v = mont_mul(y, w, m);
                lds[i0] = add_mod(x, v, m.q);
                lds[i1] = sub_mod(x, v, m.q);
            } else if (s != 0) {
                lds[i0] = add_mod(x, y, m.q);
                lds[i1] = mont_mul(sub_mod(x, y, m.q), w, m);
            } else {
                lds[i0] = mont_mul(add_mod(x, y, m.q), ninv[2 * limb], m);
                lds[i1] = mont_mul(sub_mod(x, y, m.q), ninv[2 * limb + 1], m);
            }
        }
        __syncthreads();
    }

    for (u32 e = threadIdx.x; e < T; e += NTT_THREADS) {
        size_t gi = strided ? ((size_t)(e >> lt_log) << (logN - a)) + base + (e & ((1u << lt_log) - 1)) : base + e;
        poly[gi] = lds[e];
    }
}


// which: 0 = pass A (N = 2^16: first / last 4 stages, registers only), 2 = pass B (12 stages in a 4096 tile)
// FP: the kernel serves the rows whose prime is below 2^50 (fp64 butterflies) or the others (integer butterflies);
// rows of the other kind return at once.  One kernel for both kinds needs the union of the two register budgets
// (130 registers, 3 waves per SIMD in pass B, against 112 to 124 and 4 waves for the separate ones).
template <bool INV, int WHICH, bool FP>
__global__ __launch_bounds__(NTT_THREADS) void ntt_fast_kernel(u64 *__restrict__ data,
                                                               const ModConst *__restrict__ mods,
                                                               const ModFp *__restrict__ modf,
                                                               const u64 *__restrict__ tw,
                                                               const double *__restrict__ twf,
                                                               const u64 *__restrict__ ninv, LimbIds ids,
                                                               u32 n_limbs, u32 logN) {
    __shared__ u64 lds[WHICH == 0 ? 1 : FAST_LDS_WORDS];
    const u32 row = blockIdx.y;
    const u32 limb = ids.id[row % n_limbs];
    if (limb == SKIP_ROW) return;
    const ModFp mf = modf[limb];
    if ((mf.ok != 0) != FP) return;
    u64 *poly = data + ((size_t)row << logN);
    auto load = [&](u32 idx) { return poly[idx]; };
    auto store = [&](u32 idx, u64 v) { poly[idx] = v; };
    const u32 col = blockIdx.x * NTT_THREADS + threadIdx.x;
    if (FP) {
        const FieldFp f = make_field_fp(mf, twf, limb, logN);
        if (WHICH == 0) pass_a16_body<INV>(f, col, load, store);
        if (WHICH == 2) pass_b_body<INV>(f, logN, lds, load, store);
    } else {
        const FieldInt f = make_field_int(mods, tw, ninv, limb, logN);
        if (WHICH == 0) pass_a16_body<INV>(f, col, load, store);
        if (WHICH == 2) pass_b_body<INV>(f, logN, lds, load, store);
    }
}

template <bool INV, int WHICH>
static void launch_fast(const ckks_params *p, u64 *d_data, const LimbIds &ids, u32 n_limbs, u32 rows, u32 tiles,
                        hipStream_t stream, bool scaled_dn) {
    bool any_fp = false, any_int = false;
    for (u32 i = 0; i < n_limbs; ++i) {
        if (ids.id[i] == SKIP_ROW) continue;
        if ((p->mod[ids.id[i]] >> 50) == 0)
            any_fp = true;
        else
            any_int = true;
    }
#define FAST_LAUNCH(FPK)                                                                                             \
    hipLaunchKernelGGL((ntt_fast_kernel<INV, WHICH, FPK>), dim3(tiles, rows), dim3(NTT_THREADS), 0, stream, d_data,   \
                       p->d_mod, scaled_dn ? p->d_modf_dn : p->d_modf, INV ? p->d_tws_inv : p->d_tws_fwd,            \
                       INV ? p->d_twf_inv : p->d_twf_fwd, scaled_dn ? p->d_ninvs_dn : p->d_ninvs, ids, n_limbs,      \
                       p->logN)
    if (any_fp) FAST_LAUNCH(true);
    if (any_int) FAST_LAUNCH(false);
#undef FAST_LAUNCH
}

int launch_ntt(const ckks_params *p, u64 *d_data, const LimbIds &ids, u32 n_limbs, u32 rows, bool inverse,
               hipStream_t stream, u32 pass_mask, bool scaled_dn) {
    if (rows == 0) return CKKS_OK;
    const u32 logN = p->logN;
    const u32 tile_log = logN < NTT_TILE_LOG ? logN : NTT_TILE_LOG;
    const u32 a = logN > NTT_TILE_LOG ? logN - 8 : 0;
    const size_t lds_bytes = sizeof(u64) << tile_log;
    dim3 grid(p->N >> tile_log, rows), block(NTT_THREADS);
    if (pass_mask & 1)
        for (u32 r = 0; r < rows; ++r)
            if (ids.id[r % n_limbs] != SKIP_ROW) ++p->limb_ntts;
    if (rows > 65535) {
        set_error("launch_ntt: %u rows exceed one launch", rows);
        return CKKS_E_INVAL;
    }
    if (logN == 16 || logN == 12) {
        // N = 2^16: pass A (4 stages) and pass B (12 stages); N = 2^12: pass B is the whole transform (forward: the
        // "second" pass, inverse: the "first"), and carries the scaled last stage
        const u32 tb = p->N >> 12;
        const bool two = logN == 16;
        if (!inverse) {
            if ((pass_mask & 1) && two) launch_fast<false, 0>(p, d_data, ids, n_limbs, rows, 16, stream, false);
            if (pass_mask & 2) launch_fast<false, 2>(p, d_data, ids, n_limbs, rows, tb, stream, false);
        } else {
            if (pass_mask & 1) launch_fast<true, 2>(p, d_data, ids, n_limbs, rows, tb, stream, two ? false : scaled_dn);
            if ((pass_mask & 2) && two) launch_fast<true, 0>(p, d_data, ids, n_limbs, rows, 16, stream, scaled_dn);
        }
        CKKS_LAUNCH_CHECK("ntt_fast_kernel");
        return CKKS_OK;
    }
    const u64 *ninv_tab = scaled_dn ? p->d_ninv_dn : p->d_ninv;
    if (!inverse) {
        if (a)
            hipLaunchKernelGGL(ntt_pass_kernel<false>, grid, block, lds_bytes, stream, d_data, p->d_mod, p->d_tw_fwd,
                               p->d_ninv, ids, n_limbs, logN, 0u, a, tile_log, 1u);
        hipLaunchKernelGGL(ntt_pass_kernel<false>, grid, block, lds_bytes, stream, d_data, p->d_mod, p->d_tw_fwd,
                           p->d_ninv, ids, n_limbs, logN, a, logN, tile_log, 0u);
    } else {
        hipLaunchKernelGGL(ntt_pass_kernel<true>, grid, block, lds_bytes, stream, d_data, p->d_mod, p->d_tw_inv,
                           ninv_tab, ids, n_limbs, logN, a, logN, tile_log, 0u);
        if (a)
            hipLaunchKernelGGL(ntt_pass_kernel<true>, grid, block, lds_bytes, stream, d_data, p->d_mod, p->d_tw_inv,
                               ninv_tab, ids, n_limbs, logN, 0u, a, tile_log, 1u);
    }
    CKKS_LAUNCH_CHECK("ntt_pass_kernel");
    return CKKS_OK;
}

}  // namespace ckks

using namespace ckks;

static int ntt_api(const ckks_params_t *P, uint64_t *d_data, const uint32_t *limb_ids, uint32_t n_limbs,
                   uint32_t batch, void *stream, bool inverse) {
    if (P && batch == 0) return CKKS_OK;
    if (!P || !d_data || !limb_ids || n_limbs == 0 || n_limbs > MAX_LIMBS) {
        set_error("ckks_ntt: null argument or n_limbs outside [1,%u]", MAX_LIMBS);
        return CKKS_E_INVAL;
    }
    LimbIds ids;
    for (u32 i = 0; i < n_limbs; ++i) {
        if (limb_ids[i] >= P->W) {
            set_error("ckks_ntt: limb id %u out of range", limb_ids[i]);
            return CKKS_E_INVAL;
        }
        ids.id[i] = (uint8_t)limb_ids[i];
    }
    // long batches go out in slices of at most 32768 rows
    u32 per = (32768 / n_limbs) * n_limbs;
    for (u64 done = 0; done < (u64)batch * n_limbs; done += per) {
        u32 rows = (u32)std::min<u64>(per, (u64)batch * n_limbs - done);
        int rc = launch_ntt(P, d_data + done * P->N, ids, n_limbs, rows, inverse, (hipStream_t)stream);
        if (rc) return rc;
    }
    return CKKS_OK;
}

extern "C" {

int ckks_ntt(const ckks_params_t *P, uint64_t *d_data, const uint32_t *limb_ids, uint32_t n_limbs, uint32_t batch,
             void *stream) {
    return ntt_api(P, d_data, limb_ids, n_limbs, batch, stream, false);
}

int ckks_intt(const ckks_params_t *P, uint64_t *d_data, const uint32_t *limb_ids, uint32_t n_limbs, uint32_t batch,
              void *stream) {
    return ntt_api(P, d_data, limb_ids, n_limbs, batch, stream, true);
}

}  // extern "C"
