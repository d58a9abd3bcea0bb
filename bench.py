#!/usr/bin/env python3
"""Benchmark of the HE secure-aggregation hot path on one MI355X.

One step = one whole federated round of the workload on one GPU: every client's
he_encrypt_masked, then he_aggregate, then he_decrypt_merge (inputs resident in HBM).
Prints ONE JSON line; `value` = K * P_enc / step time (client parameters carried through
encrypt -> aggregate -> decrypt per second); per-phase rates are in `phases`.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload resnet18_full]
"""
import argparse
import json
import os
import sys
import time

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))

HBM_PEAK_GBS = 8000.0
# 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz: 32-bit integer add / min / mul_lo / mul_hi all issue
# at one wave64 instruction per 4 cycles per SIMD on gfx950 (measured), so this is the peak
# for the integer butterfly instruction mix.
ALU_PEAK_TOPS = 256 * 4 * 16 * 2.4e9 / 1e12
# Operation counts of the integer butterflies as the kernels execute them (one 32-bit instruction each):
OPS_BFLY_FWD = 11        # Shoup product (mul_hi, 2 x 64-bit multiply-add) + its reduction (2) + modular add (3) + modular sub (3)
OPS_BFLY_FWD_LAZY = 8    # outputs whose next use is a Shoup multiplicand stay in [0, 2q): add (1) + sub (2)
OPS_BFLY_INV = 10        # modular add (3) + x - y + q (2) + Shoup product (3) + its reduction (2)
OPS_POINTWISE = 5        # Shoup product + reduction
OPS_LAST_STAGE_NINV = 1.5  # standalone inverse: 1/N is folded into its last stage, whose sum output then takes a Shoup product too
COPY_CEILING_GBS = 5700.0  # fallback when the copy is not measured in the run: what a plain device copy reaches on this chip, read + write bytes
PASS_PLAN = {14: (4, 4, 3, 3), 13: (4, 3, 3, 3)}   # stages per LDS pass of the specialised transforms


def fwd_ops_per_coeff(log_n, lazy_last):
    """Forward transform: inside a pass half the butterflies of every stage but the last are lazy; the last stage of
    the last pass is lazy when a key product follows (encrypt, decrypt).  Half a butterfly per coefficient and stage."""
    plan = PASS_PLAN.get(log_n)
    if plan is None:
        return 0.5 * log_n * (OPS_BFLY_FWD + 1)      # generic kernels: four-instruction Shoup product, no lazy butterflies
    ops = 0.0
    for p, r in enumerate(plan):
        ops += (r - 1) * 0.5 * (OPS_BFLY_FWD + OPS_BFLY_FWD_LAZY) / 2
        ops += 0.5 * (OPS_BFLY_FWD_LAZY if (lazy_last and p == len(plan) - 1) else OPS_BFLY_FWD)
    return ops


def encrypt_ops_per_ct(N, L):
    """Per limb: one forward and two inverse transforms, two key products, and per coefficient the residues of u (3),
    m + e0 (1 + 5) and e1 (3) and two modular additions (3 each)."""
    log_n = N.bit_length() - 1
    per_coeff = fwd_ops_per_coeff(log_n, True) + 2 * 0.5 * log_n * OPS_BFLY_INV + 2 * OPS_POINTWISE + 3 + 6 + 3 + 6
    return L * N * per_coeff


def measured_traffic(workload):
    """HBM bytes per launch from the committed rocprofv3 FETCH_SIZE / WRITE_SIZE summary, if any."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", f"hbm_traffic_{workload}.txt")
    out = {}
    if os.path.exists(path):
        for line in open(path):
            parts = line.split()
            if len(parts) >= 3 and parts[0] == "traffic_bytes_per_launch":
                out[parts[1]] = float(parts[2])
    return out


def measured_valu_busy(workload):
    """Vector-ALU busy percentage per kernel from the committed rocprofv3 VALUBusy summary, if any."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", f"valu_utilisation_{workload}.txt")
    out = {}
    if os.path.exists(path):
        for line in open(path):
            parts = line.split()
            if len(parts) >= 3 and parts[0] == "valu_busy_pct":
                out[parts[1]] = float(parts[2])
    return out


def measured_wave_instructions(workload):
    """Vector-ALU wave instructions per launch (rocprofv3 SQ_INSTS_VALU) per kernel from the committed summary, if any."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", f"alu_counters_{workload}.txt")
    out = {}
    if os.path.exists(path):
        for line in open(path):
            parts = line.split()
            if len(parts) >= 4 and parts[0] == "valu_wave_instructions_per_launch":
                out[parts[1]] = (float(parts[2]), float(parts[3]))      # (instructions, ciphertexts in that launch)
    return out


def issue_rates():
    """Runs the register-only instruction-rate loops of libhe_issue_rates.so (include/he_issue_rates.h)."""
    import ctypes as C
    from paper_2303_10837_amd import build
    lib = C.CDLL(build.RATES_LIB_PATH)
    lib.he_issue_rates_name.restype = C.c_char_p
    n = lib.he_issue_rates_count()
    ns, n_simd = (C.c_double * n)(), C.c_uint32(0)
    rc = lib.he_issue_rates_run(0, ns, C.byref(n_simd))
    if rc != 0:
        raise RuntimeError(f"he_issue_rates_run: hip error {rc}")
    rows = []
    for i in range(n):
        k = lib.he_issue_rates_instructions(i)
        rows.append({"what": lib.he_issue_rates_name(i).decode(), "instructions": k, "ns_per_simd": ns[i],
                     "cycles_at_2.4GHz": ns[i] * 2.4, "cycles_per_instruction": ns[i] * 2.4 / k,
                     "chip_lane_TOPs": k * 64 * n_simd.value / ns[i] / 1e3})
    return {"n_simd": n_simd.value, "waves_per_simd": 8, "rows": rows}


def _oracle_ciphertext_job(job):
    """One ciphertext index of the round on the CPU oracle: every client's encode + encrypt, the server's weighted sum
    and rescale (or plain sum), decrypt, lift, decode.  Runs in the parent (one core) and in spawned worker processes
    (all cores); a worker imports numpy and the oracle only, never torch or the HIP library."""
    params, seed, alpha, c, slots, client_weighted = job
    from oracle import encoder as oenc, fedavg as ofed, scheme as osch
    from oracle.params import Params
    p = Params(*params)
    keys = _ORACLE_KEYS.get((params, seed))
    if keys is None:
        keys = _ORACLE_KEYS.setdefault((params, seed), osch.keygen(p, seed))
    if client_weighted:
        cts = [osch.encrypt(p, keys, oenc.encode_fft(np.float64(a) * z, p.log2_n, p.scale_bits), seed + 1, i, c)
               for i, (z, a) in enumerate(zip(slots, alpha))]
        return ofed.decode_ct_level(p, keys, osch.sum_ciphertexts(p, cts), p.n_limbs)[:1]
    cts = [osch.encrypt(p, keys, oenc.encode_fft(z, p.log2_n, p.scale_bits), seed + 1, i, c) for i, z in enumerate(slots)]   # round seed != key seed
    return ofed.decode_ct(p, keys, osch.aggregate(p, cts, alpha))[:1]


_ORACLE_KEYS = {}


def cpu_baseline(w, slots_of, n_ct, alpha, budget_s=10.0, client_weighted=False):
    """Times the CPU oracle on a bounded sample of ciphertext indices of the same workload: once in this process (one
    core) and once over spawned worker processes, one per host core the box gives a one-GPU job (at most 16).
    slots_of(c) -> the K clients' slot vectors (float64 [n]) of ciphertext index c; the gather itself (n loads per
    client) is done by the caller and not timed."""
    import multiprocessing as mp
    K = w.n_clients
    params = (w.log2_n, w.n_limbs - 1 if client_weighted else w.n_limbs, w.scale_bits, w.cbd_eta)
    n_slots = (1 << w.log2_n) // 2
    job = lambda c: (params, w.seed, [float(a) for a in alpha], int(c), slots_of(int(c)), client_weighted)
    _oracle_ciphertext_job(job(0))                       # key generation and table set-up, not timed
    t0 = time.perf_counter()
    _oracle_ciphertext_job(job(min(1, n_ct - 1)))
    t_one = time.perf_counter() - t0
    n1 = int(max(1, min(n_ct, budget_s // max(t_one, 1e-3))))
    idx1 = np.linspace(0, n_ct - 1, n1).astype(int)
    jobs = [job(c) for c in idx1]
    t0 = time.perf_counter()
    for j in jobs:
        _oracle_ciphertext_job(j)
    dt1 = time.perf_counter() - t0
    one = {"value": n1 * n_slots * K / dt1, "unit": "params/s", "cores": 1,
           "sample": f"{n1} of {n_ct} ciphertext indices x {K} clients, {dt1:.1f} s"}
    cores = max(1, min(16, os.cpu_count() or 1))
    n_all = int(max(cores, min(n_ct, 2 * cores * max(1, budget_s // max(t_one, 1e-3) // 2))))
    idx_all = np.linspace(0, n_ct - 1, n_all).astype(int)
    jobs = [job(c) for c in idx_all]
    with mp.get_context("spawn").Pool(cores) as pool:
        pool.map(_oracle_ciphertext_job, [job(0)] * cores, chunksize=1)      # every worker: imports, keys, tables
        t0 = time.perf_counter()
        pool.map(_oracle_ciphertext_job, jobs, chunksize=1)
        dt_all = time.perf_counter() - t0
    return {"value": n_all * n_slots * K / dt_all, "unit": "params/s", "cores": cores, "kind": "oracle",
            "sample": f"{n_all} of {n_ct} ciphertext indices x {K} clients (encode, encrypt, aggregate, decrypt, decode "
                      f"per index), {dt_all:.1f} s over {cores} worker processes; host reports {os.cpu_count()} cores",
            "one_core": one}


def aggregate_k_sweep(he, ctx, torch, n_ct=512, ks=(3, 8, 16, 32, 64, 128, 200), reps=5):
    """Server-side cost against the number of clients (the paper's figure on up to 200 clients): he_aggregate alone on
    K distinct ciphertext buffers of n_ct ciphertexts each, filled with uniform residues (timing does not depend on
    the values; parity for large K is a test).  Above 64 clients the library folds 64 clients per launch into an
    internal accumulator, whose extra traffic is part of the measured time but not of the algorithmic bytes."""
    N, L = ctx.N, ctx.L
    q_min = ctx.primes[-1]
    bufs = [torch.randint(0, q_min, (n_ct, 2, L, N), dtype=torch.int32, device="cuda") for _ in range(max(ks))]
    out = torch.empty((n_ct, 2, L - 1, N), dtype=torch.int32, device="cuda")
    rows = []
    for K in ks:
        counts = np.random.default_rng(K).integers(100, 1001, K).astype(np.float64)
        alpha = counts / counts.sum()
        he.he_aggregate(ctx, alpha, bufs[:K], [None] * K, out, None)
        torch.cuda.synchronize()
        he.he_debug_timing_enable(ctx, True)
        he.he_debug_timing_read(ctx)
        for _ in range(reps):
            he.he_aggregate(ctx, alpha, bufs[:K], [None] * K, out, None)
        ms, launches = he.he_debug_timing_read(ctx)["aggregate"]
        he.he_debug_timing_enable(ctx, False)
        ms_call = ms / reps
        alg = n_ct * 8 * N * (K * L + L - 1)
        rows.append({"clients": K, "ms": ms_call, "launches_per_call": launches // reps,
                     "encrypted_params_per_s": n_ct * (N // 2) / (ms_call * 1e-3),
                     "algorithmic_GBps": alg / (ms_call * 1e-3) / 1e9, "frac_of_hbm_peak": alg / (ms_call * 1e-3) / 1e9 / HBM_PEAK_GBS})
    del bufs
    return {"n_ct": n_ct, "ring_degree": N, "limbs": L, "rows": rows}


def crypto_param_sweep(he, torch, P=1_663_370, K=3, reps=3):
    """Packing batch and scaling bits against time, ciphertext size and decoded error (the paper's table on crypto
    parameters, measured there on a CNN of 1,663,370 parameters with 3 clients; here a Gaussian vector of that size).
    Ring degrees 2^11 and 2^12 run on the generic kernels, 2^13 and 2^14 on the specialised ones."""
    rs = np.random.default_rng(20230310)
    ws_host = [rs.normal(0, 0.05, P).astype(np.float32) for _ in range(K)]
    counts = rs.integers(100, 1001, K).astype(np.float64)
    alpha = counts / counts.sum()
    ws = [torch.from_numpy(x).cuda() for x in ws_host]
    ref = sum(float(a) * x.double() for a, x in zip(alpha, ws))
    rows = []
    for log2_n in (11, 12, 13, 14):
        for scale_bits in (20, 30):
            ctx = he.Context(log2_n, 3, scale_bits, 21)
            keys = he.he_keygen(ctx, 7)
            mask = he.he_mask_create(ctx, P, [0], [P])
            cts = [torch.empty((mask.n_ct, 2, ctx.L, ctx.N), dtype=torch.int32, device="cuda") for _ in range(K)]
            ct_g = torch.empty((mask.n_ct, 2, ctx.L - 1, ctx.N), dtype=torch.int32, device="cuda")
            out = torch.empty((P,), dtype=torch.float32, device="cuda")
            none = [None] * K

            def rnd():
                for i in range(K):
                    he.he_encrypt_masked(ctx, keys, mask, 7, i, ws[i], cts[i], None)
                he.he_aggregate(ctx, alpha, cts, none, ct_g, None)
                he.he_decrypt_merge(ctx, keys, mask, ct_g, None, out)

            rnd()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                rnd()
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3 / reps
            err = (out.double() - ref).abs()
            rows.append({"packing_batch": ctx.N // 2, "scale_bits": scale_bits, "limbs": ctx.L, "ms_per_round": ms,
                         "ciphertext_MB_per_client": mask.n_ct * 2 * ctx.L * ctx.N * 4 / 1e6,
                         "plain_MB_per_client": P * 4 / 1e6,
                         "max_abs_err": float(err.max()), "rms_err": float(err.pow(2).mean().sqrt())})
            del cts, ct_g, out
            keys.close()
            mask.close()
            ctx.close()
    return {"params": P, "clients": K, "rows": rows}


def mask_select_bench(he, ctx, torch, sizes=(25_600_000, 110_000_000, 1_300_000_000), ratio=0.1, reps=3):
    """Select(global privacy map, p) on model-sized maps (layer-structured synthetic sensitivities): wall time of the
    whole set-up call (three histogram passes, mark, the mask object's tables built on the device, temporaries)."""
    rows = []
    for P in sizes:
        g = torch.Generator(device="cuda").manual_seed(P % 1000)
        sens = torch.rand(P // 4096 + 1, generator=g, device="cuda").repeat_interleave(4096)[:P].contiguous()
        sens += 0.05 * torch.rand(P, generator=g, device="cuda")
        he.he_mask_select_top(ctx, sens, ratio).close()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            m = he.he_mask_select_top(ctx, sens, ratio)
            n_runs = int(he.load().he_mask_n_runs(m.h))
            m.close()
        ms = (time.perf_counter() - t0) * 1e3 / reps
        alg = P * (3 * 4 + 4 + 1 + 2)      # three histogram passes and the mark pass read 4 B, mark writes 1 B, two run passes read 1 B
        rows.append({"params": P, "ratio": ratio, "runs": n_runs, "ms": ms, "algorithmic_GBps": alg / (ms * 1e-3) / 1e9})
        del sens
    return rows


def fragmented_mask_bench(he, torch, P=110_000_000, ratio=0.1, reps=4):
    """One client's round (encrypt, aggregate with weight 1, decrypt) on P parameters under masks of the same size and
    different structure: the top `ratio` of a synthetic sensitivity map whose values are shared by `layer` consecutive
    parameters plus 5 % per-parameter noise (layer = 1: a per-parameter selection, runs of one or two parameters), and
    32 equal blocks.  Kernel times per round from the library's own events."""
    ctx = he.Context(14, 4)
    keys = he.he_keygen(ctx, 1)
    g = torch.Generator(device="cuda").manual_seed(5)
    w = torch.randn(P, generator=g, device="cuda") * 0.02
    rows, k = [], 0

    def probe(mask, tag):
        ct = torch.empty((mask.n_ct, 2, 4, ctx.N), dtype=torch.int32, device="cuda")
        pl = torch.empty(mask.n_plain, device="cuda")
        ctg = torch.empty((mask.n_ct, 2, 3, ctx.N), dtype=torch.int32, device="cuda")
        out = torch.empty(P, device="cuda")

        def rnd():
            he.he_encrypt_masked(ctx, keys, mask, 5, 0, w, ct, pl)
            he.he_aggregate(ctx, [1.0], [ct], [pl], ctg, pl)
            he.he_decrypt_merge(ctx, keys, mask, ctg, pl, out)
        rnd()
        torch.cuda.synchronize()
        he.he_debug_timing_enable(ctx, True)
        he.he_debug_timing_read(ctx)
        for _ in range(reps):
            rnd()
        t = he.he_debug_timing_read(ctx)
        he.he_debug_timing_enable(ctx, False)
        rows.append({"mask": tag, "runs": int(he.load().he_mask_n_runs(mask.h)), "encrypted_params": mask.P_enc,
                     "kernels_ms_per_round": {kk: v[0] / reps for kk, v in t.items() if v[1]},
                     "max_abs_err": float((out - w).abs().max())})

    for layer in (4096, 64, 1):
        lay = torch.rand(P // layer + 1, generator=g, device="cuda").repeat_interleave(layer)[:P].contiguous()
        sens = lay + 0.05 * torch.rand(P, generator=g, device="cuda")
        del lay
        m = he.he_mask_select_top(ctx, sens, ratio)
        del sens
        probe(m, f"top {ratio} of a map with layers of {layer}")
        k = m.P_enc
        m.close()
    blk = he.he_mask_create(ctx, P, list(range(0, P, P // 32))[:32], [k // 32] * 32)
    probe(blk, "32 blocks")
    blk.close()
    keys.close()
    ctx.close()
    return {"params": P, "ratio": ratio, "rows": rows}


HEADLINE = "fm1p3b_sel5"          # the largest workload that runs whole on one GPU (32 clients x 1.3 B parameters)
HEADLINE_MIN_FREE_GIB = 200       # what it needs resident; on a GPU with less free HBM the headline is bert_full
OTHER_WORKLOADS = ("tiny_full", "resnet18_full", "resnet50_sel10", "bert_sel10", "bert_full")


def measure_copy_ceiling(torch, n_bytes=1 << 30, reps=8):
    """What a plain device-to-device copy of 1 GiB reaches on this machine right now (read + write bytes per second)."""
    src = torch.empty(n_bytes // 4, dtype=torch.int32, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    dst.copy_(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    return 2 * n_bytes * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9


def run_workload(he, si, torch, name, args, steps, warmup, headline, copy_gbs=None):
    """Times `steps` whole rounds of one workload and returns its result row (for the headline workload: the full
    record with rooflines, standalone transform rates and the CPU baseline)."""
    w = si.WORKLOADS[name]
    K = w.n_clients
    client_weighted = args.variant == "client_weighted"
    n_limbs = w.n_limbs - 1 if client_weighted else w.n_limbs     # no rescale: the level never drops
    ctx = he.Context(w.log2_n, n_limbs, w.scale_bits, w.cbd_eta)
    keys = he.he_keygen(ctx, w.seed)
    starts, lens = si.mask_runs(w)
    mask = he.he_mask_create(ctx, w.n_params, starts, lens)
    alpha = si.client_alphas(w)
    # A workload whose client vectors do not fit next to all clients' ciphertexts (the 1.3 B-parameter one: 166 GB of
    # inputs beside 133 GB of ciphertexts) keeps `n_distinct` vectors resident and hands client i vector i mod
    # n_distinct (cost does not depend on the values); each client's plaintext remainder is folded into the float64
    # accumulator right after its encryption (he_aggregate_add), and all K ciphertext sets stay resident and are
    # streamed through he_aggregate once.
    streamed = args.stream_clients or K * w.n_params * 4 > 64e9
    n_distinct = min(K, 4) if streamed else K
    on_device = streamed or w.n_params >= 50_000_000              # torch's seeded device generator for the long vectors
    if on_device:
        ws = [si.client_params_torch(w, i, "cuda") for i in range(n_distinct)]
    else:
        ws = [torch.from_numpy(si.client_params_numpy(w, i)).cuda() for i in range(n_distinct)]
    ws = [ws[i % n_distinct] for i in range(K)]
    N, L, n_ct, P_enc = ctx.N, ctx.L, mask.n_ct, mask.P_enc
    n_pl = mask.n_plain
    cts = [torch.empty((n_ct, 2, L, N), dtype=torch.int32, device="cuda") for _ in range(K)]
    plains = [] if streamed else [torch.empty((n_pl,), dtype=torch.float32, device="cuda") for _ in range(K)]
    L_out = L if client_weighted else L - 1
    ct_g = torch.empty((n_ct, 2, L_out, N), dtype=torch.int32, device="cuda")
    pl_g = torch.empty((n_pl,), dtype=torch.float32, device="cuda")
    out = torch.empty((w.n_params,), dtype=torch.float32, device="cuda")
    # The server is its own party with its own copy of the public crypto context (it never holds a key).  In the
    # streamed form it works on a second stream and folds the plaintext remainders of G clients at a time into its
    # float64 accumulator (one read-modify-write of the accumulator per G clients; the first fold only writes it and
    # the last one writes the rounded result instead).  With one set of G buffers the
    # clients wait for the fold before they reuse a buffer; a second set lets them go on, which gains nothing here
    # (the fold and the encryption kernels share the memory system) and costs the memory a larger G can use.
    acc_none = acc_plain = ct_none = server = server_stream = None
    G, N_HALVES = args.fold_group, args.fold_buffers
    if streamed:
        if client_weighted:
            sys.exit("bench.py: --variant client_weighted is not combined with streamed clients")
        server = he.Context(w.log2_n, n_limbs, w.scale_bits, w.cbd_eta)
        server_stream = torch.cuda.Stream()
        plains = [torch.empty((n_pl,), dtype=torch.float32, device="cuda") for _ in range(min(K, N_HALVES * G))]
        acc_none, acc_plain = he.he_aggregate_begin(server, 0, n_pl)
        ct_none = torch.empty((0, 2, L_out, N), dtype=torch.int32, device="cuda")
        torch.cuda.synchronize()
    ev = [None] * 4
    phase_ms = np.zeros(3)
    # encryption randomness: a fresh seed for every round (step), unrelated to the key generation seed; never reused with a client id
    round_seed = [(w.seed << 20) ^ 0x5EED]

    def next_round_seed():
        round_seed[0] += 1
        return round_seed[0]

    def step_streamed(record):
        seed_t = next_round_seed()
        cur = torch.cuda.current_stream()
        if record:
            ev[0].record()
        server_stream.wait_stream(cur)
        one_group = K <= G                              # then: begin, add, finalize; else the first fold writes the
        if n_pl and one_group:                          # accumulator and the last one writes the result
            with torch.cuda.stream(server_stream):
                he.he_aggregate_begin(server, 0, n_pl, acc_none, acc_plain)
        folded = {}                                    # buffer half -> event: the server has read these remainders
        for g0 in range(0, K, G):
            grp = list(range(g0, min(g0 + G, K)))
            half = (g0 // G) % N_HALVES
            if half in folded:
                cur.wait_event(folded[half])
            slots = [half * G + (i - g0) for i in grp]
            for i, sl in zip(grp, slots):
                he.he_encrypt_masked(ctx, keys, mask, seed_t, i, ws[i], cts[i], plains[sl % len(plains)])
            if n_pl:
                sent = torch.cuda.Event()
                sent.record(cur)
                with torch.cuda.stream(server_stream):
                    server_stream.wait_event(sent)
                    fold_args = (server, alpha[grp[0]:grp[-1] + 1], [None] * len(grp), [plains[sl % len(plains)] for sl in slots],
                                 acc_none, acc_plain)
                    if one_group:
                        he.he_aggregate_add(*fold_args)
                    elif g0 == 0:
                        he.he_aggregate_add_first(*fold_args)
                    elif g0 + G >= K:
                        he.he_aggregate_add_last(*fold_args, ct_none, pl_g)
                    else:
                        he.he_aggregate_add(*fold_args)
                    folded[half] = torch.cuda.Event()
                    folded[half].record(server_stream)
        cur.wait_stream(server_stream)
        if record:
            ev[1].record()      # the encrypt phase of this form includes the server's folding of the remainders
        he.he_aggregate(server, alpha, cts, [None] * K, ct_g, None)
        if n_pl and one_group:
            he.he_aggregate_finalize(server, acc_none, acc_plain, ct_none, pl_g)
        if record:
            ev[2].record()
        he.he_decrypt_merge(ctx, keys, mask, ct_g, pl_g, out)
        if record:
            ev[3].record()

    # --client-streams S > 1: the clients are independent parties; S of them at a time work side by side, each with
    # its own context (scratch), key handles and stream, so that one client's kernel tails and under-filled launches
    # overlap with the next client's work.  Per-kernel event times then include the sharing of the chip.
    S = max(1, min(args.client_streams, K))
    lanes = [(ctx, keys, mask, None)]
    for _ in range(1, S):
        c2 = he.Context(w.log2_n, n_limbs, w.scale_bits, w.cbd_eta)
        lanes.append((c2, he.he_keygen(c2, w.seed), he.he_mask_create(c2, w.n_params, starts, lens), torch.cuda.Stream()))
    torch.cuda.synchronize()

    def step_resident(record):
        seed_t = next_round_seed()
        cur = torch.cuda.current_stream()
        if record:
            ev[0].record()
        for _, _, _, st in lanes[1:]:
            st.wait_stream(cur)
        for i in range(K):
            c_i, k_i, m_i, st = lanes[i % S]
            with torch.cuda.stream(st if st is not None else cur):
                if client_weighted:
                    he.he_encrypt_masked_weighted(c_i, k_i, m_i, seed_t, i, alpha[i], ws[i], cts[i], plains[i])
                else:
                    he.he_encrypt_masked(c_i, k_i, m_i, seed_t, i, ws[i], cts[i], plains[i])
        for _, _, _, st in lanes[1:]:
            cur.wait_stream(st)
        if record:
            ev[1].record()
        if client_weighted:
            he.he_aggregate_sum(ctx, cts, plains, ct_g, pl_g)
        else:
            he.he_aggregate(ctx, alpha, cts, plains, ct_g, pl_g)
        if record:
            ev[2].record()
        if client_weighted:
            he.he_decrypt_merge_level(ctx, keys, mask, L, ct_g, pl_g, out)
        else:
            he.he_decrypt_merge(ctx, keys, mask, ct_g, pl_g, out)
        if record:
            ev[3].record()

    step = step_streamed if streamed else step_resident
    timed_ctxs = [ctx] + ([server] if server is not None else []) + [l[0] for l in lanes[1:]]

    def timing_read():
        tot = {}
        for c in timed_ctxs:
            for k, (ms, n) in he.he_debug_timing_read(c).items():
                t = tot.get(k, (0.0, 0))
                tot[k] = (t[0] + ms, t[1] + n)
        return tot

    for _ in range(warmup):
        step(False)
    torch.cuda.synchronize()
    for c in timed_ctxs:
        he.he_debug_timing_enable(c, True)
    timing_read()
    t0 = time.perf_counter()
    step_events = []
    for _ in range(steps):
        ev[:] = [torch.cuda.Event(enable_timing=True) for _ in range(4)]   # own events per step, read after the region
        step_events.append(list(ev))
        step(True)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    for e4 in step_events:
        phase_ms += [e4[i].elapsed_time(e4[i + 1]) for i in range(3)]
    kern = timing_read()
    for c in timed_ctxs:
        he.he_debug_timing_enable(c, False)
    ms_step = dt * 1e3 / steps
    phase_ms /= steps
    # The same steps once more without the per-kernel event pairs and the phase events: what the instrumentation of
    # the timed region above costs (reported beside `value`, never as `value`).
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step(False)
    torch.cuda.synchronize()
    ms_step_plain = (time.perf_counter() - t0) * 1e3 / steps

    # sanity: the decoded aggregate is FedAvg up to the CKKS noise (not part of the timing)
    if streamed:
        plains.clear()
        torch.cuda.empty_cache()
    ref = torch.zeros(w.n_params, dtype=torch.float64, device="cuda")
    for a, x in zip(alpha, ws):
        ref.add_(x, alpha=float(a))
    max_err = float((out.double() - ref).abs().max())
    del ref

    # rooflines of the encryption kernel (ALU-bound; the dominant one by accumulated device time in every workload but
    # the tiny one) and of the aggregation kernel (HBM-bound), from the event pairs of the timed region
    enc_ms, enc_launches = kern["encrypt"]
    agg_ms, agg_launches = kern["aggregate"]
    enc_ops = encrypt_ops_per_ct(N, L) * n_ct * K * steps                # all launches of the timed region
    enc_tops = enc_ops / (enc_ms * 1e-3) / 1e12 if enc_ms else 0.0
    enc_bytes = (8 * L + 7) * N * n_ct * K * steps                       # 2*L*N residues written + m (int32), u, e0, e1 (int8) read once
    agg_bytes = n_ct * 2 * N * 4 * (K * L + L_out) * steps
    agg_gbs = agg_bytes / (agg_ms * 1e-3) / 1e9 if agg_ms else 0.0
    dominant = max(kern, key=lambda k: kern[k][0])
    traffic, busy = measured_traffic(w.name), measured_valu_busy(w.name)
    prof_note = f"replayed from profiles/hbm_traffic_{w.name}.txt and profiles/valu_utilisation_{w.name}.txt (rocprofv3 --pmc runs of this command), not measured in this run"
    roofline = {"kernel": "k_encrypt_s", "bound": "alu", "achieved": enc_tops, "peak": ALU_PEAK_TOPS, "unit": "TOP/s",
                "frac": enc_tops / ALU_PEAK_TOPS, "traffic": traffic.get("k_encrypt"),
                "valu_busy_pct_profiled": busy.get("k_encrypt"), "profiled_fields": prof_note,
                "avg_launch_ms": enc_ms / max(enc_launches, 1), "launches": int(enc_launches),
                "algorithmic_ops_per_launch": enc_ops / max(enc_launches, 1),
                "algorithmic_bytes_per_launch": enc_bytes / max(enc_launches, 1),
                "hbm_GBps": enc_bytes / (enc_ms * 1e-3) / 1e9 if enc_ms else 0.0,
                "hbm_frac": enc_bytes / (enc_ms * 1e-3) / 1e9 / HBM_PEAK_GBS if enc_ms else 0.0}
    roofline_agg = {"kernel": "k_aggregate", "bound": "hbm", "achieved": agg_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": agg_gbs / HBM_PEAK_GBS, "traffic": traffic.get("k_aggregate"),
                    "valu_busy_pct_profiled": busy.get("k_aggregate"), "profiled_fields": prof_note,
                    "algorithmic_bytes_per_launch": agg_bytes / max(agg_launches, 1),
                    "avg_launch_ms": agg_ms / max(agg_launches, 1), "launches": int(agg_launches),
                    "target_hbm_frac": 0.6, "met": bool(agg_gbs / HBM_PEAK_GBS >= 0.6)}
    # the plaintext path (HBM-bound): compaction / scatter of the remainder and its float64 averaging
    mv_ms, mv_launches = kern.get("plain_move", (0.0, 0))
    pf_ms, pf_launches = kern.get("plain_fedavg", (0.0, 0))
    mv_bytes = 8 * n_pl * (K + 1) * steps                               # K compactions and one scatter: 4 B read + 4 B written each
    if streamed:   # folds of G clients: K reads; the first fold writes the accumulator (8 B), middle ones read and write
        folds = -(-K // G)                         # it, the last one reads it and writes float32 (one fold: begin, add, finalize)
        pf_bytes = n_pl * (4 * K + (16 * (folds - 1) + 4 if folds > 1 else 16 + 8 + 4)) * steps
    else:
        pf_bytes = n_pl * (4 * K + 4) * steps
    roofline_plain = None
    if n_pl:
        roofline_plain = {
            "k_plain_move": {"bound": "hbm", "achieved": mv_bytes / (mv_ms * 1e-3) / 1e9 if mv_ms else 0.0, "peak": HBM_PEAK_GBS,
                             "unit": "GB/s", "frac": mv_bytes / (mv_ms * 1e-3) / 1e9 / HBM_PEAK_GBS if mv_ms else 0.0,
                             "frac_of_copy_ceiling": mv_bytes / (mv_ms * 1e-3) / 1e9 / (copy_gbs or COPY_CEILING_GBS) if mv_ms else 0.0,
                             "copy_ceiling_GBps": copy_gbs or COPY_CEILING_GBS,
                             "avg_launch_ms": mv_ms / max(mv_launches, 1), "launches": int(mv_launches),
                             "note": "K compactions (he_encrypt_masked) and one scatter (he_decrypt_merge), 4 B read + 4 B written per plaintext parameter each"},
            "k_plain_fedavg": {"bound": "hbm", "achieved": pf_bytes / (pf_ms * 1e-3) / 1e9 if pf_ms else 0.0, "peak": HBM_PEAK_GBS,
                               "unit": "GB/s", "frac": pf_bytes / (pf_ms * 1e-3) / 1e9 / HBM_PEAK_GBS if pf_ms else 0.0,
                               "avg_launch_ms": pf_ms / max(pf_launches, 1), "launches": int(pf_launches)}}
    # encoder and decoder: fp64 FFT through LDS plus (decoder) the exact lift; reported against their fp64 / integer
    # operation counts
    ec_ms, ec_launches = kern.get("encode", (0.0, 0))
    dc_ms, dc_launches = kern.get("decode", (0.0, 0))
    dq_ms, dq_launches = kern.get("decrypt", (0.0, 0))
    side = {"encode_ms_per_step": ec_ms / steps, "decode_ms_per_step": dc_ms / steps, "decrypt_ms_per_step": dq_ms / steps,
            "encode_cts_per_s": n_ct * K * steps / (ec_ms * 1e-3) if ec_ms else 0.0,
            "decode_cts_per_s": n_ct * steps / (dc_ms * 1e-3) if dc_ms else 0.0,
            "decrypt_cts_per_s": n_ct * steps / (dq_ms * 1e-3) if dq_ms else 0.0}
    # ALU rooflines of the encoder (Philox sampler + fp64 FFT), the decryption kernel and the decoder (exact lift + FFT):
    # executed vector instructions per ciphertext from the committed rocprofv3 SQ_INSTS_VALU summary x 64 lanes x the
    # ciphertext rate measured here, against the same one-instruction-per-4-cycles peak
    wi = measured_wave_instructions(w.name)
    for kname, rate in (("k_encode_r", side["encode_cts_per_s"]), ("k_decrypt_s", side["decrypt_cts_per_s"]), ("k_decode_h", side["decode_cts_per_s"])):
        if kname in wi and wi[kname][1]:
            per_ct = wi[kname][0] / wi[kname][1]
            tops = per_ct * 64 * rate / 1e12
            side["roofline_" + kname] = {"bound": "alu", "achieved": tops, "peak": ALU_PEAK_TOPS, "unit": "TOP/s", "frac": tops / ALU_PEAK_TOPS,
                                         "wave_instructions_per_ciphertext_profiled": per_ct}

    phase_bytes = [K * (4 * P_enc + 8 * n_pl + n_ct * 8 * L * N),                       # parameters read, remainder copied, ciphertexts written
                   n_ct * 8 * N * (K * L + L_out) + n_pl * (4 * K + 4),               # K ciphertexts and remainders read, one of each written
                   n_ct * 8 * L_out * N + 4 * P_enc + 8 * n_pl]                        # ciphertext read, parameters written, remainder copied
    if streamed:   # the K reads of the remainders happen while the clients encrypt; only the final write is in the server phase
        phase_bytes[0] += n_pl * 4 * K
        phase_bytes[1] -= n_pl * 4 * K
    res = {
        "value": K * P_enc / (ms_step * 1e-3), "unit": "params/s", "ms_per_step": ms_step, "steps": steps, "warmup": warmup,
        "whole_model_params_per_s": K * w.n_params / (ms_step * 1e-3),
        "config": {"workload": w.name, "variant": args.variant, "streamed_clients": streamed, "client_streams": S,
                   "distinct_client_vectors": n_distinct, "clients": K, "params_per_client": w.n_params, "encrypted_params": P_enc,
                   "n_ct_per_client": n_ct, "ring_degree": N, "limbs": L, "scale_bits": w.scale_bits,
                   "value_definition": "clients * encrypted_params / step time; step = all clients encrypt + aggregate + decrypt; "
                                       "whole_model_params_per_s = clients * params_per_client / the same step time (gather, "
                                       "plaintext FedAvg and merge of the unencrypted share included)"},
        "phases": {"encrypt_ms": phase_ms[0], "aggregate_ms": phase_ms[1], "decrypt_ms": phase_ms[2],
                   "encrypt_params_per_s": K * P_enc / (phase_ms[0] * 1e-3),
                   "aggregate_params_per_s": P_enc / (phase_ms[1] * 1e-3),
                   "decrypt_params_per_s": P_enc / (phase_ms[2] * 1e-3),
                   # the same phases as fractions of what HBM alone would allow (algorithmic bytes of the phase / time / peak)
                   "encrypt_frac_of_hbm_roofline": phase_bytes[0] / (phase_ms[0] * 1e-3) / (HBM_PEAK_GBS * 1e9),
                   "aggregate_frac_of_hbm_roofline": phase_bytes[1] / (phase_ms[1] * 1e-3) / (HBM_PEAK_GBS * 1e9),
                   "decrypt_frac_of_hbm_roofline": phase_bytes[2] / (phase_ms[2] * 1e-3) / (HBM_PEAK_GBS * 1e9)},
        "uninstrumented": {"ms_per_step": ms_step_plain, "value": K * P_enc / (ms_step_plain * 1e-3),
                           "note": "same steps without the per-kernel event pairs and phase events of the timed region"},
        "kernels_ms_per_step": {k: v[0] / steps for k, v in kern.items() if v[1]},
        "dominant_kernel": dominant,
        "roofline": roofline, "roofline_aggregate": roofline_agg, "roofline_plain": roofline_plain, "encode_decode": side,
        "max_abs_err_vs_float64_fedavg": max_err,
    }
    if headline:
        res["roofline_ntt"] = ntt_rooflines(he, ctx, torch, w.name)
        if args.calibrate_copy:
            src = torch.empty(1 << 28, dtype=torch.int32, device="cuda").fill_(1)   # 1 GiB
            dst = torch.empty_like(src)
            dst.copy_(src)
            torch.cuda.synchronize()
            del src, dst
        if args.k_sweep:
            res["aggregate_k_sweep"] = aggregate_k_sweep(he, ctx, torch)
        if args.param_sweep:
            res["crypto_param_sweep"] = crypto_param_sweep(he, torch)
        if args.select_bench:
            res["mask_select"] = mask_select_bench(he, ctx, torch)
        if args.fragmented_masks:
            res["fragmented_masks"] = fragmented_mask_bench(he, torch)
        if args.issue_rates:
            res["issue_rates"] = issue_rates()
        if not args.no_cpu_baseline:
            from oracle import fedavg as ofed                                  # host index arithmetic of the gather only
            n = N // 2
            uniq = {id(x): x for x in ws}

            def slots_of(c):
                t = np.arange(c * n, min((c + 1) * n, P_enc))
                idx = torch.from_numpy(ofed.packed_to_param(starts, lens, t)).cuda()
                got = {k: np.concatenate([x[idx].double().cpu().numpy(), np.zeros(n - len(t))]) for k, x in uniq.items()}
                return [got[id(x)] for x in ws]

            res["cpu_baseline"] = cpu_baseline(w, slots_of, n_ct, alpha, client_weighted=client_weighted)
    del cts, plains, ct_g, pl_g, out, ws, acc_plain, acc_none
    for c2, k2, m2, _ in lanes[1:]:
        k2.close(), m2.close(), c2.close()
    keys.close(), mask.close(), ctx.close()
    if server is not None:
        server.close()
    torch.cuda.empty_cache()
    return res


def ntt_rooflines(he, ctx, torch, workload, batch=4096, reps=5):
    """Standalone transform (he_debug_ntt, in place): forward and inverse timed separately over `batch` polynomials.
    8 B of HBM traffic per coefficient (one read, one write); reported against the HBM peak, which is what the 60 %
    target refers to, and against the integer ALU peak, which is what bounds the kernel."""
    N, L = ctx.N, ctx.L
    log_n = N.bit_length() - 1
    polys = torch.randint(0, ctx.primes[-1], (batch, N), dtype=torch.int32, device="cuda")
    out = {}
    for inverse, tag in ((False, "forward"), (True, "inverse")):
        he.he_debug_ntt(ctx, inverse, L - 1, polys)
        torch.cuda.synchronize()
        he.he_debug_timing_enable(ctx, True)
        he.he_debug_timing_read(ctx)
        for _ in range(reps):
            he.he_debug_ntt(ctx, inverse, L - 1, polys)
        ms, launches = he.he_debug_timing_read(ctx)["ntt"]
        he.he_debug_timing_enable(ctx, False)
        coeff_per_s = batch * N * launches / (ms * 1e-3)
        ops = (0.5 * log_n * OPS_BFLY_INV + OPS_LAST_STAGE_NINV) if inverse else fwd_ops_per_coeff(log_n, False)
        tops = coeff_per_s * ops / 1e12
        hbm_frac = coeff_per_s * 8 / 1e9 / HBM_PEAK_GBS
        out[tag] = {"kernel": "k_ntt_batch_s<%d,%s>" % (log_n, "true" if inverse else "false"), "bound": "alu",
                    "achieved": tops, "peak": ALU_PEAK_TOPS, "unit": "TOP/s", "frac": tops / ALU_PEAK_TOPS,
                    "ops_per_coeff": ops, "coeff_per_s": coeff_per_s, "avg_launch_ms": ms / launches, "launches": int(launches),
                    "algorithmic_bytes_per_launch": batch * N * 8, "hbm_GBps": coeff_per_s * 8 / 1e9, "hbm_frac": hbm_frac,
                    "hbm_frac_ceiling_at_perfect_issue": ALU_PEAK_TOPS * 1e12 / ops * 8 / 1e9 / HBM_PEAK_GBS,
                    "target_hbm_frac": 0.6, "met": bool(hbm_frac >= 0.6),
                    "traffic": measured_traffic(workload).get("k_ntt_batch_" + tag),
                    "valu_busy_pct_profiled": measured_valu_busy(workload).get("k_ntt_batch_" + tag)}
    del polys
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default=None,
                    help=f"headline workload (default: {HEADLINE}, the largest one, or bert_full when less than "
                         f"{HEADLINE_MIN_FREE_GIB} GiB of HBM are free)")
    ap.add_argument("--only", action="store_true", help="run the headline workload only (no rows for the other workloads)")
    ap.add_argument("--other-steps", type=int, default=5, help="timed steps of each of the other workloads' rows")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--variant", default="server_weighted", choices=["server_weighted", "client_weighted"],
                    help="client_weighted: clients encode alpha_i * W_i, the server only adds ciphertexts (no rescale), one limb fewer")
    ap.add_argument("--param-sweep", action="store_true",
                    help="also run packing batch 1024..8192 x scaling bits 20/30 on a 1.66M-parameter vector, 3 clients")
    ap.add_argument("--fragmented-masks", action="store_true",
                    help="also time one client's round on 110 M parameters under top-p selections of different granularity and under blocks")
    ap.add_argument("--select-bench", action="store_true",
                    help="also time the encryption-mask selection (top-p of a sensitivity map) on 25.6M / 110M / 1.3B entries")
    ap.add_argument("--k-sweep", action="store_true",
                    help="also time he_aggregate alone for K = 3 ... 200 clients (server cost against the number of clients)")
    ap.add_argument("--issue-rates", action="store_true",
                    help="also run the register-only instruction-rate loops behind the integer-ALU peak (libhe_issue_rates.so)")
    ap.add_argument("--stream-clients", action="store_true",
                    help="fold each client's plaintext remainder into the server's accumulator right after its encryption "
                         "(he_aggregate_begin/add/finalize) and keep only 4 distinct client vectors resident; chosen by "
                         "itself when the clients' vectors exceed 64 GB")
    ap.add_argument("--fold-group", type=int, default=16, help="streamed clients: remainders the server folds per he_aggregate_add")
    ap.add_argument("--fold-buffers", type=int, default=1, help="streamed clients: groups of remainder buffers (2 = the next group encrypts while one is folded)")
    ap.add_argument("--client-streams", type=int, default=1,
                    help="number of clients that encrypt side by side, each on its own context and stream (default 1: one after the other)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (known HBM traffic, for scaling rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (ciphertext indices are independent, so more GPUs "
                 "would shard by ciphertext index with no collectives); run with --gpus 1")

    import torch
    from paper_2303_10837_amd import binding as he, synth_inputs as si

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    free_gib = torch.cuda.mem_get_info()[0] / 2 ** 30
    name, fallback = args.workload, None
    if name is None:
        name = HEADLINE
        if free_gib < HEADLINE_MIN_FREE_GIB:
            name, fallback = "bert_full", f"{HEADLINE} needs {HEADLINE_MIN_FREE_GIB} GiB of free HBM, this GPU has {free_gib:.0f}"
    copy_gbs = measure_copy_ceiling(torch)      # a plain 1 GiB copy on this machine: the yardstick of the plaintext kernels beside the 8 TB/s peak
    head = run_workload(he, si, torch, name, args, args.steps, args.warmup, True, copy_gbs)
    res = {"metric": "encrypted params/sec (encrypt, aggregate, decrypt) + NTT/agg HBM GB/s % of peak",
           "value": head.pop("value"), "unit": head.pop("unit"), "n_gpus": 1, "steps": head.pop("steps"),
           "warmup": head.pop("warmup"), "ms_per_step": head.pop("ms_per_step"), "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "u32", "data": "synthetic"}
    res.update(head)
    res["config"]["free_hbm_gib_at_start"] = free_gib
    res["config"]["plain_copy_GBps_measured"] = copy_gbs
    if fallback:
        res["config"]["headline_fallback"] = fallback
    if not args.only and args.workload is None:
        rows = {}
        keep = ("value", "unit", "ms_per_step", "steps", "whole_model_params_per_s", "phases", "uninstrumented", "kernels_ms_per_step",
                "dominant_kernel", "roofline", "roofline_aggregate", "roofline_plain", "encode_decode", "max_abs_err_vs_float64_fedavg")
        for other in OTHER_WORKLOADS:
            if other == name:
                continue
            r = run_workload(he, si, torch, other, args, args.other_steps, 1, False, copy_gbs)
            rows[other] = {k: r[k] for k in keep}
            rows[other]["config"] = {k: r["config"][k] for k in ("clients", "params_per_client", "encrypted_params", "n_ct_per_client",
                                                                  "ring_degree", "limbs", "streamed_clients")}
        res["workloads"] = rows
        if "fragmented_masks" not in res:      # beside the block masks of the workloads: the masks a per-parameter selection gives
            try:
                res["fragmented_masks"] = fragmented_mask_bench(he, torch)
            except Exception as e:             # a side figure never costs the run its result line
                res["fragmented_masks"] = {"error": f"{type(e).__name__}: {e}"}
    print(json.dumps(res))


if __name__ == "__main__":
    main()
