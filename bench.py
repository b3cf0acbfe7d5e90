#!/usr/bin/env python3
"""Benchmark of the CKKS ct x pt matmul hot path on one MI355X.

One step = one pass of the whole path on the BERT-base QKV projection under CKKS
(N = 2^16, 24 + 8 primes, scale 2^40, X 128x768 encrypted, W 768x2304 + bias in plaintext):
ckks_ctpt_matmul (hoisted baby-step bank, diagonal multiply-accumulate over the pre-expanded
weights, giant-step key switches summed over the extended basis, bias, and the rescale fused
into the one ModDown per output block), with keys, weights and input ciphertexts resident in HBM.
Prints ONE JSON line; the second headline figure, key switches per second on a hoisted batch
(N = 2^16, L = 24), the NTT batch, the GPT-2-small block and the oracle's CPU time ride in the same line.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

FP64_ISSUE_PEAK = 256 * 64 * 2.4e9      # fp64 vector instructions per second per lane-op: 256 CUs x 64 lanes x 2.4 GHz (78.6 TFLOP/s / 2)
HBM_PEAK_GBS = 8000.0
GIANT_NAMES = {True: "one ModDown per output block (rotated accumulators summed over the extended basis)",
               False: "one complete key switch per rotation"}


def key_switch_bytes(N, level, K, L, dnum):
    """Algorithmic bytes of one key switch inside a hoisted batch: both components of the key over the level + K
    active limbs for each digit, the extended digits once, c0 once, the output once (8 bytes per residue)."""
    alpha = L // dnum
    beta = -(-level // alpha)
    Wl = level + K
    return (2 * beta * Wl + beta * Wl + level + 2 * level) * 8 * N


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def setup_matmul(B, CL, W, P, cl, spec, n1, key_cache=None, fused_qk=False, pairs=False):
    """fused_qk: the d_out columns are [Q | K | V]; Q and K go through ONE projection with the complex weights
    W_Q + i*W_K (App. A.2.3), V through real weights: 2/3 of the output blocks and giant steps.
    pairs: complex-pair compression of Sec. 3.2: inputs x^(2u) + i*x^(2u+1), weights (W_even - i*W_odd)/2, one
    conjugation per output block brings back the real result: half the bank and half the products."""
    import torch
    N, n = P.N, P.N // 2
    level = P.L
    X, Wm, bias = W.matmul_inputs(spec)
    third = spec.d_out // 3
    parts = [(Wm, 0)]                                        # (matrix, first output block)
    if fused_qk:
        parts = [(Wm[:, :third] + 1j * Wm[:, third:2 * third], 0), (Wm[:, 2 * third:], -(-third // spec.C))]
        bias = None
    G = -(-spec.d_in // spec.C)
    if pairs:
        G = -(-G // 2)                                       # complexified inputs
    B_out = sum(-(-M.shape[1] // spec.C) for M, _ in parts)
    N2 = spec.C // n1
    scale = 2.0 ** spec.ring.log_scale
    t0 = time.time()
    key_cache = {} if key_cache is None else key_cache

    def key(step):
        if step not in key_cache:
            key_cache[step] = cl.galois_key(step)
        return key_cache[step]

    baby = [key(q * spec.m) for q in range(1, n1)]
    giant = [key(p * n1 * spec.m) for p in range(1, N2)]
    log(f"[bench] {len(baby) + len(giant)} Galois keys ready in {time.time() - t0:.1f}s")
    xs = CL.pack_columns_complex(X, n, spec.C) if pairs else CL.pack_columns(X, n, spec.C)
    ct_x = torch.stack([cl.encrypt_slots(xs[g], scale, level) for g in range(G)])
    conj = key("conj") if pairs else None
    w = B.ckks_weights_create(P, level, spec.m, spec.C, G, B_out, n1)
    t0 = time.time()
    for M, b_first in parts:
        for b in range(-(-M.shape[1] // spec.C)):
            for p in range(N2):
                if pairs:
                    z = CL.diagonal_slots_complex(M, spec.m, n, spec.C, n1, b, p).reshape(G * n1, n)
                else:
                    z = CL.diagonal_slots(M, spec.m, n, spec.C, n1, b, p).reshape(G * n1, n)
                B.ckks_weights_set_diagonals(w, ((b_first + b) * N2 + p) * G * n1, cl.enc.encode(z, scale))
    if bias is not None:
        nseg = n // spec.m
        bz = np.zeros((B_out, n))
        for b in range(B_out):
            col = b * spec.C + np.arange(nseg) % spec.C
            v = np.where(col < spec.d_out, bias[np.minimum(col, spec.d_out - 1)], 0.0)
            bz[b] = np.repeat(v, spec.m)
        B.ckks_weights_set_bias(w, cl.enc.encode(bz, scale), int(scale))
    torch.cuda.synchronize()
    log(f"[bench] {G * n1 * B_out * N2} weight diagonals encoded and expanded in {time.time() - t0:.1f}s")
    ref = X @ Wm + (bias if bias is not None else 0.0)
    if fused_qk:
        ref = np.concatenate([X @ parts[0][0], X @ parts[1][0] + 0j], axis=1)       # [Q + iK | V]
    return dict(ct_x=ct_x, w=w, baby=baby, giant=giant, conj=conj, ref=ref, G=G, B_out=B_out, N2=N2, scale=scale,
                level=level)


def measured_ceilings(B, P):
    """Streaming rates of plain copy / read / write kernels over 2 GiB buffers and the issue rates of the two
    modular products, measured live (the fractions beside the published peaks are against these)."""
    import torch
    src = torch.ones(1 << 28, dtype=torch.int64, device="cuda")
    dst = torch.empty_like(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(f, reps=5):
        f()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            f()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e-3

    nbytes = src.numel() * 8
    out = {"copy_GBps": 2 * nbytes / timed(lambda: B.ckks_probe_stream(dst, src, B.PROBE_COPY)) / 1e9,
           "read_GBps": nbytes / timed(lambda: B.ckks_probe_stream(dst, src, B.PROBE_READ)) / 1e9,
           "write_GBps": nbytes / timed(lambda: B.ckks_probe_stream(dst, None, B.PROBE_WRITE)) / 1e9}
    del src, dst
    lanes, iters = 1 << 20, 2000
    sink = torch.empty(lanes, dtype=torch.int64, device="cuda")
    for name, kind, limb in (("fp64_mulmod_per_s", B.PROBE_FP64, 0), ("int64_mulmod_per_s", B.PROBE_INT64, P.L),
                             ("int64_lazy_mulmod_per_s", B.PROBE_INT64_LAZY, P.L)):
        if kind == B.PROBE_FP64 and P.q[0] >> 50:
            continue
        out[name] = 4.0 * lanes * iters / timed(lambda: B.ckks_probe_mulmod(P, limb, kind, lanes, iters, sink), 3)
    return out


def read_traffic(workload, n1):
    """HBM bytes per diag_mac_kernel launch from the committed rocprofv3 --pmc summary (FETCH_SIZE and
    WRITE_SIZE runs, scaled by the plain-copy factors stated there); None if it is for another plan."""
    path = os.path.join(ROOT, "profiles", "bert_qkv_diag_mac_hbm_traffic.txt")
    try:
        kv = dict(l.strip().split("=", 1) for l in open(path) if "=" in l and not l.startswith("#"))
        if kv.get("workload") == workload and int(kv.get("N1", -1)) == n1:
            return float(kv["traffic_bytes_per_launch"])
    except (OSError, ValueError, KeyError):
        pass
    return None


def read_valu(workload):
    """Vector-ALU utilisation of the diagonal multiply-accumulate kernel from the committed SQ-counter summary
    (instructions * 4 cycles / SIMDs / elapsed cycles) and the clock the kernel ran at; None for another workload."""
    path = os.path.join(ROOT, "profiles", "bert_qkv_valu_utilisation.txt")
    try:
        kv = dict(l.strip().split("=", 1) for l in open(path) if "=" in l and not l.startswith("#"))
        if kv.get("workload") == workload:
            return {"valu_busy": float(kv["valu_busy"]), "sclk_ghz": float(kv["sclk_ghz"]),
                    "valu_insts_per_launch": float(kv["valu_insts_per_launch"])}
    except (OSError, ValueError, KeyError):
        pass
    return None


def _omp_threads(n):
    """Sets the OpenMP thread count of this process (the oracle's C library is parallelised with OpenMP over
    independent limbs / diagonals / Galois elements only)."""
    import ctypes
    try:
        ctypes.CDLL("libgomp.so.1").omp_set_num_threads(int(n))
        return True
    except OSError:
        return False


def cpu_baseline(W, spec, n1, full=False):
    """The oracle as it stands, on the host cores.  Default: a bounded sample, three distinct 128 x 256 x 256
    corners (input group, output block) of the projection, each timed in its parts; the spread of the three is
    printed and the whole-layer figure is assembled from their means.  full: the whole projection and rescale."""
    import oracle
    from oracle import encoding as E
    ring = spec.ring
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    q = oracle.find_primes(50, ring.logN, 24)
    p = oracle.find_primes(60, ring.logN, 8)
    O = oracle.Oracle(ring.logN, q, p, ring.dnum)
    r = W.rng(spec.seed + 1000)
    s = W.ternary_secret(r, O.N)

    def key(step):
        a = W.uniform_residues(r, O.moduli, O.N, lead=(O.dnum,))
        e = W.gaussian_error(r, (O.dnum, O.N))
        return O.galois_keygen(s, O.galois_elt(step), a, e)

    C, m = spec.C, spec.m
    N2 = C // n1
    G, B_out = -(-spec.d_in // C), -(-spec.d_out // C)
    X, Wm, bias = W.matmul_inputs(spec)
    scale = 2.0 ** ring.log_scale
    mx = E.encode(E.pack_columns(X, O.n, C) + 0j, scale, O.N)
    cts = np.stack([O.encrypt(O.L, mx[g], s, W.uniform_residues(r, O.q, O.N), W.gaussian_error(r, (O.N,)))
                    for g in range(G)])
    baby = [key(qq * m) for qq in range(1, n1)]
    giant = [key(pp * n1 * m) for pp in range(1, N2)]
    gel_bank = [O.galois_elt(qq * m) for qq in range(n1)]

    # single-thread figures for the two smaller configurations: limb transforms and one hoisted batch
    one = {}
    if _omp_threads(1):
        x = W.uniform_residues(r, O.q, O.N)
        t0 = time.time()
        for i in range(O.L):
            O.ntt(i, x[i])
        one["ntt_limb_polys_per_s"] = O.L / (time.time() - t0)
        t0 = time.time()
        O.rotate_hoisted(cts[0], O.L, gel_bank[:5], [None] + baby[:4])
        one["hoisted_key_switches_per_s"] = 4 / (time.time() - t0)
        one["sample"] = "24 forward limb transforms; one hoisted call with 4 key switches (decomposition included)"
        _omp_threads(cores)

    if full:
        diag = E.encode_diagonals(Wm, m, O.N, C, n1, scale)
        bias_c = np.stack([E.encode(E.bias_slots(bias, m, O.n, C, b) + 0j, scale, O.N) for b in range(B_out)])
        t0 = time.time()
        y = O.ctpt_matmul(O.L, m, G, B_out, n1, N2, diag, bias_c, int(scale), cts, baby, giant)
        O.rescale(y, O.L)
        t_full = time.time() - t0
        return dict(value=t_full * 1e3, unit="ms", cores=cores, kind="oracle",
                    sample="the whole 128x768x2304 projection + rescale, one complete key switch per giant rotation",
                    one_thread=one)

    corners = [(0, 0), (1, B_out // 2), (G - 1, B_out - 1)]       # (input group, output block)
    t_bank, t_single, t_diag = [], [], []
    t_all = time.time()
    for g, b in corners:
        Xc, Wc = X[:, g * C:(g + 1) * C], Wm[g * C:(g + 1) * C, b * C:(b + 1) * C]
        diag = E.encode_diagonals(Wc, m, O.N, C, n1, scale)
        ct = cts[g:g + 1]
        t0 = time.time()
        O.rotate_hoisted(ct[0], O.L, gel_bank, [None] + baby)
        t_bank.append(time.time() - t0)
        t0 = time.time()
        O.rotate_hoisted(ct[0], O.L, [O.galois_elt(n1 * m)], giant[:1])
        t_single.append(time.time() - t0)
        t0 = time.time()
        y = O.ctpt_matmul(O.L, m, 1, 1, n1, N2, diag, None, 0, ct, baby, giant)
        O.rescale(y, O.L)
        t_sub = time.time() - t0
        t_diag.append(max(t_sub - t_bank[-1] - (N2 - 1) * t_single[-1], 0.0))   # 256 diagonals + one rescale
    t_all = time.time() - t_all
    mean = lambda v: sum(v) / len(v)
    full_est = G * mean(t_bank) + G * B_out * mean(t_diag) + B_out * (N2 - 1) * mean(t_single)
    spread = {"bank_s": [round(v, 3) for v in t_bank], "single_switch_s": [round(v, 3) for v in t_single],
              "diagonals_256_s": [round(v, 3) for v in t_diag]}
    return dict(value=full_est * 1e3, unit="ms", cores=cores, kind="oracle",
                sample=f"three 128x{C}x{C} corners (input group, output block) = {corners} of the projection run by "
                       f"the oracle in {t_all:.1f}s, each: {n1 - 1} hoisted + {N2 - 1} single key switches, 256 of the "
                       f"{G * B_out * C} diagonals, 1 rescale; value = {G}*bank + {G * B_out}*diagonals + "
                       f"{B_out * (N2 - 1)}*single switch from the means of the three (extrapolated; "
                       f"--cpu-baseline full runs the whole layer)",
                spread=spread, key_switches_per_s_hoisted=(n1 - 1) / mean(t_bank), one_thread=one)


def run_gpt2_block(args, B, CL, W, P, cl, emit=True, steps=None):
    """The four linear layers of a GPT-2-small block (QKV, attention output, FFN up, FFN down) at sequence
    length 128, one after the other; weights of one layer resident at a time; inputs freshly encrypted per
    layer (the MPC boundary between layers is simulated by fresh synthetic activations)."""
    import torch
    from paper_2604_09975_amd import plan
    keys, layers, total = {}, [], 0.0
    n_steps = steps or args.steps
    for spec in W.GPT2_LAYERS:
        n1 = args.n1 or spec.N1
        if args.pair_compression and not args.n1:
            n1 = plan.choose_n1(-(-(-(-spec.d_in // spec.C)) // 2), -(-spec.d_out // spec.C), spec.C)
        S = setup_matmul(B, CL, W, P, cl, spec, n1, keys, pairs=args.pair_compression)
        level, B_out = S["level"], S["B_out"]
        yr = torch.empty((B_out, 2, level - 1, P.N), dtype=torch.int64, device="cuda")

        def step():
            # projection and rescale in one call (CKKS_MATMUL_RESCALE): with the merged giant step the ModDown and the
            # rescale share one pass over the correction
            _, cnt = B.ckks_ctpt_matmul(P, S["w"], S["ct_x"], S["baby"], S["giant"], yr, conj_key=S["conj"],
                                        flags=(0 if args.separate_giant else B.MATMUL_MERGED_GIANT) | B.MATMUL_RESCALE)
            return cnt

        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n_steps):
            cnt = step()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / n_steps
        out_scale = S["scale"] * S["scale"] / P.q[level - 1]
        slots = np.stack([cl.decrypt_slots(yr[b], level - 1, out_scale) for b in range(B_out)])
        err = float(np.abs(CL.unpack_columns(slots.real, spec.m, spec.C, spec.d_out) - S["ref"]).max())
        log(f"[bench] {spec.name}: {ms:.2f} ms, {cnt.key_switches} key switches, max abs err {err:.2e}")
        if not err <= 1e-3:
            log("[bench] ERROR: decrypted result is outside the 1e-3 bound")
            sys.exit(1)
        layers.append({"layer": spec.name, "d_in": spec.d_in, "d_out": spec.d_out, "G": S["G"], "B_out": B_out,
                       "N1": n1, "N2": S["N2"], "ms": ms, "key_switches": int(cnt.key_switches),
                       "ptmuls": int(cnt.ptmuls), "max_abs_err": err})
        total += ms
        S["w"].close()
        del S, yr
        torch.cuda.empty_cache()
    if not emit:
        return {"total_ms": total, "steps": n_steps, "giant_step": GIANT_NAMES[not args.separate_giant],
                "input_packing": "complex pairs (Sec. 3.2)" if args.pair_compression else "real", "layers": layers}
    print(json.dumps({
        "metric": "GPT-2-small block linear layers total latency ms (seq 128, hidden 768)", "value": total,
        "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": total,
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "u64", "data": "synthetic",
        "config": {"workload": "gpt2_small_block_linear_set", "N": P.N, "q_limbs": P.L, "special_limbs": P.K,
                   "dnum": P.dnum, "giant_step": GIANT_NAMES[not args.separate_giant],
                   "input_packing": "complex pairs (Sec. 3.2)" if args.pair_compression else "real", "layers": layers}}),
          flush=True)


def run_ntt(args, B, W, emit=True):
    """NTT microbenchmark: 64 polynomials x 24 limbs of 50-bit primes x 2^16, forward then inverse."""
    import torch
    ring = W.NTT_RING
    q = B.ckks_find_primes(50, ring.logN, 24)
    P = B.ckks_params_create(ring.logN, q, [], ring.dnum)
    x = torch.from_numpy(W.uniform_residues(W.rng(W.NTT_SEED), q, P.N, lead=(W.NTT_BATCH,)).view(np.int64)).cuda()
    ref = x.clone()
    ids = list(range(24))
    e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    for _ in range(args.warmup):
        B.ckks_ntt(P, x, ids, W.NTT_BATCH)
        B.ckks_intt(P, x, ids, W.NTT_BATCH)
    torch.cuda.synchronize()
    fwd = inv = 0.0
    for _ in range(args.steps):
        e[0].record()
        B.ckks_ntt(P, x, ids, W.NTT_BATCH)
        e[1].record()
        B.ckks_intt(P, x, ids, W.NTT_BATCH)
        e[2].record()
        torch.cuda.synchronize()
        fwd += e[0].elapsed_time(e[1])
        inv += e[1].elapsed_time(e[2])
    assert bool((x == ref).all()), "INTT(NTT(x)) != x"
    fwd, inv = fwd / args.steps, inv / args.steps
    nbytes = 2 * 8 * W.NTT_BATCH * 24 * P.N                      # each residue read once and written once
    ach = nbytes / (fwd * 1e-3) / 1e9
    if not emit:
        del x, ref
        P.close()
        torch.cuda.empty_cache()
        return {"workload": ring.name, "batch": W.NTT_BATCH, "limbs": 24, "N": 1 << ring.logN, "forward_ms": fwd,
                "inverse_ms": inv, "forward_GBps": ach, "inverse_GBps": nbytes / (inv * 1e-3) / 1e9,
                "algorithmic_bytes_per_direction": nbytes, "hbm_roofline_frac": ach / HBM_PEAK_GBS,
                "roundtrip_bit_exact": True}
    print(json.dumps({
        "metric": "NTT throughput GB/s (64 x 24 limbs x 2^16, forward)", "value": ach, "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": fwd + inv, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "u64", "data": "synthetic",
        "config": {"workload": ring.name, "batch": W.NTT_BATCH, "limbs": 24, "N": P.N},
        "forward_ms": fwd, "inverse_ms": inv, "inverse_GBps": nbytes / (inv * 1e-3) / 1e9,
        "roofline": {"bound": "hbm", "kernel": "ntt_fast_kernel (both passes)", "achieved": ach, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": ach / HBM_PEAK_GBS, "traffic": None, "bytes_per_launch": nbytes,
                     "ms_per_launch": fwd}}), flush=True)


def run_hoisted(args, B, CL, W, P, cl):
    """Hoisted rotation batch: 26 rotations + conjugation of one fresh ciphertext (N = 2^16, 24 + 8 limbs)."""
    import torch
    level = P.L
    steps = [s for s in W.HOISTED_STEPS if s != (1 << 15)]
    keys = [cl.galois_key(s) for s in steps]
    z = W.unit_disk_slots(W.rng(W.HOISTED_SEED), P.N // 2)
    ct = cl.encrypt_slots(z, 2.0 ** 40, level)
    out = torch.empty((len(steps), 2, level, P.N), dtype=torch.int64, device="cuda")
    for _ in range(max(args.warmup, 1)):
        B.ckks_rotate_hoisted(P, ct, level, steps, keys, out)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        B.ckks_rotate_hoisted(P, ct, level, steps, keys, out)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    err = max(float(np.abs(cl.decrypt_slots(out[i], level, 2.0 ** 40) - (np.conj(z) if s == "conj" else np.roll(z, -s))).max())
              for i, s in list(enumerate(steps))[::9])
    assert err < 585 * P.N / 2.0 ** 40, err
    ks = len(steps) / ms * 1e3
    # the step set read literally as 32 distinct steps: rotations 1..31 and the conjugation
    steps32 = list(range(1, 32)) + ["conj"]
    have = dict(zip(steps, keys))
    keys32 = [have[s] if s in have else cl.galois_key(s) for s in steps32]
    out32 = torch.empty((32, 2, level, P.N), dtype=torch.int64, device="cuda")
    B.ckks_rotate_hoisted(P, ct, level, steps32, keys32, out32)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(args.steps):
        B.ckks_rotate_hoisted(P, ct, level, steps32, keys32, out32)
    e1.record()
    torch.cuda.synchronize()
    ms32 = e0.elapsed_time(e1) / args.steps
    err32 = float(np.abs(cl.decrypt_slots(out32[30], level, 2.0 ** 40) - np.roll(z, -31)).max())
    assert err32 < 585 * P.N / 2.0 ** 40, err32
    print(json.dumps({
        "metric": "key-switches/s at N=2^16 L=24 (hoisted batch)", "value": ks, "unit": "key-switches/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u64", "data": "synthetic",
        "config": {"workload": "hoisted_rotation_batch", "N": P.N, "q_limbs": P.L, "special_limbs": P.K,
                   "dnum": P.dnum, "key_switches": len(steps)},
        "max_abs_err": err,
        "literal_32_steps": {"steps": "1..31 and conj", "key_switches": 32, "ms": ms32,
                             "key_switches_per_s": 32 / ms32 * 1e3, "max_abs_err": err32},
        "roofline": {"bound": "hbm", "kernel": "ckks_rotate_hoisted (all kernels)", "achieved": key_switch_bytes(P.N, level, P.K, P.L, P.dnum) * ks / 1e9,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": key_switch_bytes(P.N, level, P.K, P.L, P.dnum) * ks / (HBM_PEAK_GBS * 1e9),
                     "traffic": None, "bytes_per_launch": key_switch_bytes(P.N, level, P.K, P.L, P.dnum) * len(steps), "ms_per_launch": ms}}), flush=True)


def run_primitives(args, B, CL, W, P, cl):
    """Latency of the homomorphic primitives of Table 1 on one ciphertext (the set Table 6 times): rot, conj,
    ptmul, add, ctmul, each with the rescale that follows it in the protocols where one does.  N = 2^16, at the
    top level (24 limbs) and at 17 limbs (multiplicative depth 16)."""
    import torch
    n = P.N // 2
    r = W.rng(W.HOISTED_SEED)
    za, zb = W.unit_disk_slots(r, n), W.unit_disk_slots(r, n)
    k_rot, k_conj, k_relin = cl.galois_key(1), cl.galois_key("conj"), cl.relin_key()
    res = {}
    for level in (P.L, 17):
        ca, cb = cl.encrypt_slots(za, 2.0 ** 40, level), cl.encrypt_slots(zb, 2.0 ** 40, level)
        pt = B.ckks_plain_expand(P, level, cl.enc.encode(zb, 2.0 ** 40)[None])[0]
        o1 = torch.empty((1, 2, level, P.N), dtype=torch.int64, device="cuda")
        o2 = torch.empty((2, level, P.N), dtype=torch.int64, device="cuda")
        lo = torch.empty((1, 2, level - 1, P.N), dtype=torch.int64, device="cuda")
        ops = {
            "rot": lambda: B.ckks_rotate_hoisted(P, ca, level, [1], [k_rot], o1),
            "conj": lambda: B.ckks_rotate_hoisted(P, ca, level, ["conj"], [k_conj], o1),
            "ptmul": lambda: B.ckks_ptmul(P, ca, level, pt, o2),
            "ptmul+rescale": lambda: (B.ckks_ptmul(P, ca, level, pt, o2), B.ckks_rescale(P, o2, level, 1, lo)),
            "add": lambda: B.ckks_add(P, ca, cb, level, 1, o2),
            "ctmul": lambda: B.ckks_ctmul(P, ca, cb, level, k_relin, o2),
            "ctmul+rescale": lambda: (B.ckks_ctmul(P, ca, cb, level, k_relin, o2), B.ckks_rescale(P, o2, level, 1, lo)),
            "rescale": lambda: B.ckks_rescale(P, o2, level, 1, lo),
        }
        out = {}
        reps = max(args.steps, 1) * 20
        for name, f in ops.items():
            for _ in range(3):
                f()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                f()
            e1.record()
            torch.cuda.synchronize()
            out[name] = e0.elapsed_time(e1) / reps
        # end-to-end checks of what was timed
        B.ckks_ctmul(P, ca, cb, level, k_relin, o2)
        B.ckks_rescale(P, o2, level, 1, lo)
        err = float(np.abs(cl.decrypt_slots(lo[0], level - 1, 2.0 ** 80 / P.q[level - 1]) - za * zb).max())
        assert err < 1e-5, err
        B.ckks_rotate_hoisted(P, ca, level, [1], [k_rot], o1)
        err = float(np.abs(cl.decrypt_slots(o1[0], level, 2.0 ** 40) - np.roll(za, -1)).max())
        assert err < 585 * P.N / 2.0 ** 40, err
        res["limbs_%d" % level] = out
        if level == P.L:
            # bank of 16 intra-segment shifts Psi^t (m = 128): 32 rotations from one decomposition + masks
            m, ts = 128, list(range(1, 17))
            steps, masks = [], []
            for t in ts:
                h, u, st = CL.psi_masks(n, m, t)
                steps += list(st)
                masks += [cl.enc.encode(h, 2.0 ** 40), cl.enc.encode(u, 2.0 ** 40)]
            keymap = {s: cl.galois_key(s) for s in sorted(set(steps))}
            d_masks = B.ckks_plain_expand(P, level, torch.stack(masks)).reshape(len(ts), 2, level, P.N)
            bank = torch.empty((len(ts), 2, level, P.N), dtype=torch.int64, device="cuda")
            f = lambda: B.ckks_shift_bank(P, ca, level, steps, [keymap[s] for s in steps], d_masks, bank)
            f()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(max(args.steps, 1)):
                f()
            e1.record()
            torch.cuda.synchronize()
            bank_ms = e0.elapsed_time(e1) / max(args.steps, 1)
            bl = B.ckks_rescale(P, bank, level, len(ts))
            zz = cl.decrypt_slots(bl[4], level - 1, 2.0 ** 80 / P.q[level - 1])
            want = np.roll(za.reshape(n // m, m), -ts[4], axis=1).reshape(n)
            err = float(np.abs(zz - want).max())
            assert err < 1e-5, err
            res["psi_bank_16_shifts"] = {"ms": bank_ms, "key_switches": len(steps), "max_abs_err": err}
    top = res["limbs_%d" % P.L]
    print(json.dumps({
        "metric": "ctmul latency ms at N=2^16 L=24 (tensor + relinearisation)", "value": top["ctmul"], "unit": "ms",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": top["ctmul"],
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "u64", "data": "synthetic",
        "config": {"workload": "primitive_latencies", "N": P.N, "q_limbs": P.L, "special_limbs": P.K, "dnum": P.dnum},
        "latency_ms": res}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--n1", type=int, default=0, help="baby steps (0 = the configuration's default)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-baseline", default="sample", choices=["sample", "full", "none"],
                    help="oracle timing on the host cores: three sampled corners of the layer (default), the whole "
                         "layer (about two minutes), or none")
    ap.add_argument("--no-extras", action="store_true",
                    help="bert_qkv only: skip the NTT microbenchmark and the GPT-2 block that ride in the same line")
    ap.add_argument("--no-check", action="store_true")
    ap.add_argument("--workload", default="bert_qkv", choices=["bert_qkv", "gpt2_block", "hoisted", "ntt", "primitives"],
                    help="bert_qkv (default, the headline configuration), the four GPT-2-small block layers, the "
                         "hoisted rotation batch alone, or the NTT microbenchmark")
    ap.add_argument("--no-hoisted", action="store_true", help="skip the hoisted-rotation batch")
    ap.add_argument("--separate-giant", action="store_true",
                    help="giant step as one complete key switch (own ModDown) per rotation instead of the merged form")
    ap.add_argument("--merged-giant", action="store_true",
                    help="giant step with one ModDown per output block (CKKS_MATMUL_MERGED_GIANT); the default")
    ap.add_argument("--fused-qk", action="store_true",
                    help="bert_qkv only: Q and K through one projection with weights W_Q + i*W_K (no bias)")
    ap.add_argument("--pair-compression", action="store_true",
                    help="complex-pair compression of the inputs (Sec. 3.2): half the bank, one conjugation per "
                         "output block; N1 re-planned unless --n1 is given")
    ap.add_argument("--copy-probe", action="store_true",
                    help="run only a plain 4 GiB device-to-device copy, 10 times (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus above 1 is not supported (no collectives are part of "
              "the path). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    torch.cuda.set_device(0)
    if args.copy_probe:
        src = torch.ones(1 << 29, dtype=torch.int64, device="cuda")     # 4 GiB
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"probe": "copy", "bytes_read_per_launch": src.numel() * 8,
                          "bytes_written_per_launch": src.numel() * 8, "launches": 10}))
        return
    from paper_2604_09975_amd import binding as B, client as CL, plan, workload as W
    if args.workload == "ntt":
        run_ntt(args, B, W)
        return
    spec = W.BERT_QKV
    n1 = args.n1 or spec.N1
    ring = spec.ring
    q = B.ckks_find_primes(50, ring.logN, 24)
    p = B.ckks_find_primes(60, ring.logN, 8)
    P = B.ckks_params_create(ring.logN, q, p, ring.dnum)
    cl = CL.Client(P, spec.seed)
    if args.workload == "gpt2_block":
        run_gpt2_block(args, B, CL, W, P, cl)
        return
    if args.workload == "hoisted":
        run_hoisted(args, B, CL, W, P, cl)
        return
    if args.workload == "primitives":
        run_primitives(args, B, CL, W, P, cl)
        return
    if args.pair_compression and args.fused_qk:
        print("bench.py: --pair-compression and --fused-qk are different packings of the same layer; pick one.",
              file=sys.stderr)
        sys.exit(2)
    if args.pair_compression and not args.n1:
        n1 = plan.choose_n1(-(-(-(-spec.d_in // spec.C)) // 2), -(-spec.d_out // spec.C), spec.C)
    S = setup_matmul(B, CL, W, P, cl, spec, n1, fused_qk=args.fused_qk, pairs=args.pair_compression)
    N, level, B_out, G, N2 = P.N, S["level"], S["B_out"], S["G"], S["N2"]
    yr = torch.empty((B_out, 2, level - 1, N), dtype=torch.int64, device="cuda")

    merged = not args.separate_giant

    def step(merged_giant=merged):
        # projection and rescale in one call (CKKS_MATMUL_RESCALE): the same residues as ckks_ctpt_matmul followed by
        # ckks_rescale; with the merged giant step the ModDown and the rescale share one pass over the correction
        _, cnt = B.ckks_ctpt_matmul(P, S["w"], S["ct_x"], S["baby"], S["giant"], yr, conj_key=S["conj"],
                                    flags=(B.MATMUL_MERGED_GIANT if merged_giant else 0) | B.MATMUL_RESCALE)
        return cnt

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    B.ckks_profile_begin(P)
    t0 = time.time()
    e0.record()
    for _ in range(args.steps):
        cnt = step()
    e1.record()
    torch.cuda.synchronize()
    wall = time.time() - t0
    ms_per_step = e0.elapsed_time(e1) / args.steps
    mac_ms, mac_launches = B.ckks_profile_end(P)
    mac_ms /= max(mac_launches, 1)

    # correctness of what was timed: decrypt, decode, compare with the fp64 product
    max_err = None
    if not args.no_check:
        out_scale = S["scale"] * S["scale"] / P.q[level - 1]
        slots = np.stack([cl.decrypt_slots(yr[b], level - 1, out_scale) for b in range(B_out)])
        if args.fused_qk:
            Y = CL.unpack_columns(slots, spec.m, spec.C, S["ref"].shape[1])
        else:
            Y = CL.unpack_columns(slots.real, spec.m, spec.C, spec.d_out)
        max_err = float(np.abs(Y - S["ref"]).max())
        log(f"[bench] decrypted max abs error vs fp64 X@W+b: {max_err:.3e}")
        if not max_err <= 1e-3:
            log("[bench] ERROR: decrypted result is outside the 1e-3 bound")
            sys.exit(1)

    # the other evaluation order of the giant step, for reference (not the headline value)
    step(not merged)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(args.steps):
        step(not merged)
    e1.record()
    torch.cuda.synchronize()
    other_ms = e0.elapsed_time(e1) / args.steps

    # hoisted rotation batch (N = 2^16, L = 24): 26 rotations + conjugation from one ciphertext, and the step set
    # read literally as 32 distinct steps (rotations 1..31 and the conjugation)
    steps = [] if args.no_hoisted else [s for s in W.HOISTED_STEPS if s != (1 << 15)]
    keys = [cl.galois_key(s) for s in steps]
    ct = cl.encrypt_slots(W.unit_disk_slots(W.rng(W.HOISTED_SEED), P.N // 2), S["scale"], level)
    reps = 10

    def time_batch(st, ks):
        o = torch.empty((len(st), 2, level, N), dtype=torch.int64, device="cuda")
        B.ckks_rotate_hoisted(P, ct, level, st, ks, o)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            B.ckks_rotate_hoisted(P, ct, level, st, ks, o)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    rot_ms = time_batch(steps, keys)
    ks_per_s = len(steps) / rot_ms * 1e3 if steps else None
    literal32 = None
    if steps:
        steps32 = list(range(1, 32)) + ["conj"]
        have = dict(zip(steps, keys))
        keys32 = [have[s_] if s_ in have else cl.galois_key(s_) for s_ in steps32]
        ms32 = time_batch(steps32, keys32)
        literal32 = {"steps": "1..31 and conj", "key_switches": 32, "ms": ms32, "key_switches_per_s": 32 / ms32 * 1e3}
        del keys32
    del keys

    # algorithmic bytes of one diagonal multiply-accumulate launch: the bank once, the accumulators once (8 bytes
    # per residue), and of every weight limb the half that is not determined by the other half (the diagonals
    # encode real slot vectors, whose transforms are palindromes) in the packed store's 50 bits per residue
    limb_poly = 8 * N
    half_limb_packed = 3 * N + N // 8
    n_diag = G * n1 * B_out * N2
    mac_bytes = n_diag * level * half_limb_packed + (G * n1 * 2 * level + B_out * N2 * 2 * level) * limb_poly
    # the same count with unpacked half limbs (8 bytes per residue), the unit the byte budget of the method is
    # usually stated in
    mac_bytes_8 = (n_diag * level // 2 + G * n1 * 2 * level + B_out * N2 * 2 * level) * limb_poly
    if args.fused_qk:   # the complex Q+iK blocks (half of the blocks) are read in full, 8 bytes per residue
        n_cplx = G * n1 * (B_out // 2) * N2
        mac_bytes += n_cplx * level * (limb_poly - half_limb_packed)
        mac_bytes_8 += n_cplx * level * limb_poly // 2
    # the same launch in double-precision operations: 7 per residue product (exact product split, quotient,
    # remainder, two additions), 4 products per stored weight residue
    mac_ops = 7.0 * 4.0 * n_diag * level * (N // 2)
    achieved = mac_bytes / (mac_ms * 1e-3) / 1e9
    ks_bytes = key_switch_bytes(N, level, P.K, P.L, P.dnum)
    traffic = read_traffic(spec.name, n1) if not (args.fused_qk or args.pair_compression) else None
    # bytes the whole step must move, two counts: (i) the budget the method is usually stated in, every weight limb
    # in full at 8 bytes per residue + Galois keys + inputs + outputs; (ii) what this formulation has to read: the
    # weight store as it is laid out (packed half limbs for real diagonals, packed whole limbs for complex ones)
    key_bytes = (len(S["baby"]) + len(S["giant"]) + (1 if S["conj"] is not None else 0)) * P.dnum * 2 * (P.L + P.K) * limb_poly
    io_bytes = (G + B_out) * 2 * level * limb_poly
    step_bytes_8 = n_diag * level * limb_poly + key_bytes + io_bytes
    n_cplx_w = (G * n1 * (B_out // 2) * N2) if args.fused_qk else (n_diag if args.pair_compression else 0)
    step_bytes_stored = (n_diag - n_cplx_w) * level * half_limb_packed + n_cplx_w * level * 2 * half_limb_packed \
        + key_bytes + io_bytes
    out = {
        "metric": "ct-pt matmul latency ms (128x768x2304)",
        "value": ms_per_step,
        "unit": "ms",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u64",
        "data": "synthetic",
        "config": {"workload": spec.name + ("_fused_qk" if args.fused_qk else ""), "N": N, "q_limbs": P.L, "special_limbs": P.K, "dnum": P.dnum,
                   "log_scale": ring.log_scale, "m": spec.m, "d_in": spec.d_in, "d_out": spec.d_out,
                   "C": spec.C, "G": G, "B_out": B_out, "N1": n1, "N2": N2,
                   "giant_step": GIANT_NAMES[merged],
                   "input_packing": "complex pairs (Sec. 3.2)" if args.pair_compression else "real",
                   "key_switches_per_step": int(cnt.key_switches), "ptmuls_per_step": int(cnt.ptmuls),
                   "limb_ntts_per_step": int(cnt.limb_ntts),
                   "primes": {"rule": "2^b - k*2N + 1, k = 1, 2, ..., the primes in order of k", "q_bits": 50,
                              "p_bits": 60, "q": [int(v) for v in P.q], "p": [int(v) for v in P.p]}},
        "other_giant_step": {"giant_step": GIANT_NAMES[not merged], "ms_per_step": other_ms},
        "key_switches_per_s": ks_per_s,
        "hoisted_batch": {"key_switches": len(steps), "ms": rot_ms, "bytes_per_key_switch": ks_bytes,
                          "hbm_roofline_frac": ks_bytes * ks_per_s / (HBM_PEAK_GBS * 1e9) if steps else None,
                          "literal_32_steps": literal32},
        "matmul_hbm_roofline_frac": (step_bytes_8 / (ms_per_step * 1e-3)) / (HBM_PEAK_GBS * 1e9),
        "matmul_bytes": {"at_8_bytes_per_residue_full_limbs": step_bytes_8, "as_stored": step_bytes_stored,
                         "frac_as_stored": (step_bytes_stored / (ms_per_step * 1e-3)) / (HBM_PEAK_GBS * 1e9)},
        "max_abs_err": max_err,
        "wall_s_timed_region": wall,
        "roofline": {"bound": "hbm", "kernel": "diag_mac_sym_kernel", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "traffic_source": "profiles/bert_qkv_diag_mac_hbm_traffic.txt (rocprofv3 --pmc FETCH_SIZE / "
                                       "WRITE_SIZE runs of this command, committed; not measured in this run)"
                                       if traffic is not None else None,
                     "bytes_per_launch": mac_bytes, "ms_per_launch": mac_ms,
                     "fp64_issue_frac": mac_ops / (mac_ms * 1e-3) / FP64_ISSUE_PEAK,
                     "frac_at_8_bytes_per_residue": mac_bytes_8 / (mac_ms * 1e-3) / 1e9 / HBM_PEAK_GBS},
    }
    if not (args.fused_qk or args.pair_compression or args.n1):
        out["roofline"]["valu"] = read_valu(spec.name)
        if out["roofline"]["valu"] is not None:
            out["roofline"]["valu"]["source"] = ("profiles/bert_qkv_valu_utilisation.txt (rocprofv3 --pmc SQ counters "
                                                 "of this command, committed; not measured in this run)")
    ceil = measured_ceilings(B, P)
    out["measured_ceilings"] = ceil
    out["roofline"]["frac_of_measured_read"] = achieved / ceil["read_GBps"]
    if "fp64_mulmod_per_s" in ceil:     # 4 products per stored weight residue, against the bare product chain
        out["roofline"]["frac_of_measured_fp64_mulmod"] = (mac_ops / 7.0) / (mac_ms * 1e-3) / ceil["fp64_mulmod_per_s"]
    if steps:
        out["hoisted_batch"]["frac_of_measured_copy"] = ks_bytes * ks_per_s / (ceil["copy_GBps"] * 1e9)
    if not args.no_extras and not (args.fused_qk or args.pair_compression or args.n1):
        # the other configurations ride in the same line: free the headline's weights and keys first
        S["w"].close()
        del S, yr, ct
        torch.cuda.empty_cache()
        out["ntt"] = run_ntt(args, B, W, emit=False)
        log(f"[bench] ntt: forward {out['ntt']['forward_ms']:.3f} ms, inverse {out['ntt']['inverse_ms']:.3f} ms")
        out["gpt2_block"] = run_gpt2_block(args, B, CL, W, P, cl, emit=False, steps=min(args.steps, 3))
        log(f"[bench] gpt2 block: {out['gpt2_block']['total_ms']:.2f} ms")
    if not args.no_cpu_baseline and args.cpu_baseline != "none":
        t0 = time.time()
        out["cpu_baseline"] = cpu_baseline(W, spec, n1, full=args.cpu_baseline == "full")
        log(f"[bench] cpu baseline took {time.time() - t0:.1f}s")
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
