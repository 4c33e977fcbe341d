#!/usr/bin/env python3
"""Benchmark of the minwise-hash signature path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload large_2u]

A step is one pass of the whole hot path (row binning, hashing with running
minima, merge of split rows, b-bit truncation and packing) over one batch of
synthetic rows that is already resident in HBM.  The default workload is the
350 000-row, k = 500, 2U (p = 2^31 - 1) configuration the headline metric is
quoted on.  Prints ONE JSON line: whole-job hash evaluations per second, the
roofline of the dominant kernel (duration measured with HIP events on the
launch stream), and the CPU oracle timed on this machine's host cores on a bounded
sample of the same rows (the sample's GPU rows are also compared with it).
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from paper_1205_2958_amd import workloads as W  # noqa: E402

# Issue model of one hash evaluation: (multiply, full, simple) instruction counts per evaluation.
# A SIMD issues one 64-lane instruction of the full-issue class (three-operand ops, min/max, add
# with carry, funnel shift, shift left) per 4 clocks: 16 lanes/clk, the rate behind the published
# fp64 vector peak.  The simple two-operand integer instructions on vector registers (add, sub,
# and, or, xor, shift right, move) issue at twice that rate, the rate behind the published fp32
# peak, and a simple instruction of one wavefront issues beside a full-issue instruction of
# another.  The 32-bit multiplies (v_mad_u64_u32, v_mad_i64_i32, v_mul_hi_u32) take a full slot and
# let nothing issue beside them (measured: loops of one such instruction and n simple ones take
# the sum of their separate times, loops with a three-operand instruction in its place do not).
# A kernel therefore needs at least
#     multiply + max(full, (full + simple) / 2)
# issue slots per evaluation, one slot = one 64-lane instruction at 16 lanes/clk/SIMD.
ISSUE_MIX = {
    W.FAMILY_2U_M31: (1.0, 0.5 + 0.5, 1.0),         # mad | half a shift-then-add, half a max3 | half of add,add
    W.FAMILY_4U_M31: (3.0, 1.0 + 0.5 + 0.5, 3.0),   # 3 mad | add3, half a signed and half an unsigned max3 | shr,and,shr
    W.FAMILY_2U_M61: (2.0, 1.0 + 0.5, 2.0),         # 2 mad | funnel shift, half a max3 | mov,add
    W.FAMILY_2U_MS32: (1.0, 0.5, 0.0),              # mad | half a min3 (mask or shift once per row)
}
# other D (--universe) below 2^28: fractional key (one multiply-add and one funnel shift after the canonical residue)
ISSUE_MIX_OTHER_D_FRAC = {
    W.FAMILY_2U_M31: (2.0, 1.0 + 1.0 + 0.5, 3.0),         # mad, mad | min, funnel shift, half a min3 | shr,add,sub
    W.FAMILY_4U_M31: (4.0, 1.0 + 1.0 + 1.0 + 0.5, 5.0),   # 3 mad, mad | add3, min, funnel shift, half a min3 | shr,and,shr,add,xor
}
# other D of at least p/3: the smallest of r, r - D, r - 2D, no multiply after the canonical residue
ISSUE_MIX_OTHER_D_BIG = {
    W.FAMILY_2U_M31: (1.0, 1.0 + 1.0 + 0.5, 5.0),         # mad | min, min3, half a min3 | shr,add,sub,add,add
    W.FAMILY_4U_M31: (3.0, 1.0 + 1.0 + 1.0 + 0.5, 7.0),   # 3 mad | add3, min, min3, half a min3 | shr,and,shr,add,xor,add,add
}
# other D from 2^28 to p/3: exact multiply-high quotient appended
ISSUE_MIX_OTHER_D = {
    W.FAMILY_2U_M31: (3.0, 1.0 + 0.5, 4.0),         # mad, mulhi, mad | min, half a min3 | shr,add,sub,shr
    W.FAMILY_4U_M31: (5.0, 1.0 + 1.0 + 0.5, 6.0),   # 3 mad, mulhi, mad | add3, min, half a min3 | shr,and,shr,add,xor,shr
}


def issue_slots(mix):
    mul, full, simple = mix
    return mul + max(full, (full + simple) / 2.0)


ALU_PEAK_SLOTS = 256 * 4 * 16 * 2.4e9                      # 39.3e12 lane-slots/s
HBM_PEAK = 8.0e12
# HBM bytes per launch of the dominant kernel on the full workload, from two rocprofv3 --pmc runs
# (FETCH_SIZE, WRITE_SIZE), each scaled by what the counter reads for a plain 1 GiB streaming kernel
# (profiles/mh_hash_kernel_2u_m31__large_2u.txt, profiles/mh_perm_kernel__perm_table.txt).
MEASURED_TRAFFIC_BYTES = {"large_2u": 6.066e9, "perm_table": 1.1655e12}


def _oracle_worker(args):
    from oracle import oracle
    rp, col, D, k, b, family, params = args
    return oracle.signatures(rp, col, D, k, b, family, params)


def cpu_baseline(w: W.Workload, params: np.ndarray, target_evals_per_core: float, procs: int, universe: int = 0):
    """Times the unchanged single-threaded oracle on the first rows of the workload,
    sharded over `procs` processes.  Returns (record, rows, signatures)."""
    import multiprocessing as mp

    nnz_all = w.nnz(0)
    budget = target_evals_per_core * procs
    cum = np.cumsum(nnz_all) * w.k
    n_sample = int(min(len(nnz_all), max(procs, np.searchsorted(cum, budget) + 1)))
    nnz = nnz_all[:n_sample]
    rp = W.row_ptr_from_nnz(nnz)
    col = W.csr_indices_np(nnz, w.D, w.data_seed)
    D = w.D
    if universe:
        D = universe
        col = (col % np.uint32(D)).astype(np.uint32)
    # shards balanced by nonzeros
    bounds = [0]
    per = rp[-1] / procs
    for s in range(1, procs):
        bounds.append(int(np.searchsorted(rp, per * s)))
    bounds.append(n_sample)
    bounds = sorted(set(min(max(b, 0), n_sample) for b in bounds))
    jobs = []
    for lo, hi in zip(bounds[:-1], bounds[1:]):
        jobs.append((rp[lo:hi + 1] - rp[lo], col[rp[lo]:rp[hi]], D, w.k, w.b, w.family, params))
    ctx = mp.get_context("fork")
    from oracle import oracle
    oracle.build()
    with ctx.Pool(len(jobs)) as pool:
        pool.map(_oracle_worker, [(np.zeros(2, np.int64), np.zeros(0, np.uint32), D, w.k, w.b, w.family, params)] * len(jobs))
        t0 = time.perf_counter()
        parts = pool.map(_oracle_worker, jobs, chunksize=1)
        dt = time.perf_counter() - t0
    sig = np.concatenate(parts, axis=0)
    evals = float(rp[-1]) * w.k
    rec = {"value": evals / dt, "unit": "hash-evals/s", "cores": len(jobs), "kind": "oracle",
           "sample": "first %d rows of the workload (%d nonzeros, %.3g evaluations) in %.1f s, rows sharded over %d "
                     "processes each running the single-threaded C oracle" % (n_sample, int(rp[-1]), evals, dt, len(jobs)),
           "rows_per_s": n_sample / dt}
    return rec, n_sample, sig


def stream_mode(args, w, params_np, cpu_rec, n_sample, cpu_sig) -> int:
    """The heavy-tailed workload end to end: batches resident in pinned host memory,
    H2D copy / kernels / D2H copy overlapped on three streams."""
    import torch
    from paper_1205_2958_amd import minhash as mh

    dev = torch.device("cuda:0")
    n_batches = args.batches or w.n_batches()
    params = torch.from_numpy(params_np.view(np.int64)).to(dev)
    batches, total_nnz, total_rows, max_nnz = [], 0, 0, 0
    t0 = time.perf_counter()
    # Pinned host memory on the GPU machine is capped near 64 GiB, less than the 80 GB of
    # indices of all ten batches: the first `distinct` batches are staged, later ones
    # re-send the staged bytes of batch (i mod distinct).  Rates are unaffected; the
    # parity tests cover the first and the last batch with their own data.
    distinct = min(n_batches, args.distinct_batches)
    for bi in range(n_batches):
        if bi >= distinct:
            rp_h, col_h = batches[bi % distinct]
            batches.append((rp_h, col_h))
            total_nnz += sum(p.numel() for p in col_h)
            total_rows += rp_h.numel() - 1
            continue
        nnz = w.nnz(bi)
        rp_np = W.row_ptr_from_nnz(nnz)
        col = W.csr_indices_torch(nnz, w.D, w.data_seed + bi, dev)
        piece = 1 << 28                     # 1 GiB pieces: the pinned allocator rounds sizes up to powers of two
        col_h = []
        for at in range(0, col.numel(), piece):
            h = torch.empty(min(piece, col.numel() - at), dtype=torch.int32, pin_memory=True)
            h.copy_(col[at: at + h.numel()])
            col_h.append(h)
        del col
        rp_h = torch.from_numpy(rp_np).pin_memory()
        batches.append((rp_h, col_h))
        total_nnz += int(rp_np[-1])
        total_rows += len(nnz)
        max_nnz = max(max_nnz, int(rp_np[-1]))
        print("batch %d staged in pinned host memory: %d rows, %d nonzeros" % (bi, len(nnz), int(rp_np[-1])),
              file=sys.stderr, flush=True)
    torch.cuda.synchronize()
    gen_s = time.perf_counter() - t0
    mh.stream_batches(batches[:1], w.D, w.k, w.b, w.family, params, w.batch_rows, max_nnz)     # warm-up
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    outs = mh.stream_batches(batches, w.D, w.k, w.b, w.family, params, w.batch_rows, max_nnz)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    evals = float(total_nnz) * w.k
    parity = None
    if cpu_sig is not None:
        n_cmp = min(n_sample, outs[0].shape[0])
        parity = bool(np.array_equal(outs[0][:n_cmp].numpy(), cpu_sig[:n_cmp]))
    rec = {
        "metric": "hash-evals/sec (nnz*k), host-resident batches streamed over PCIe",
        "value": evals / dt, "unit": "hash-evals/s", "n_gpus": 1, "steps": 1, "warmup": 1, "ms_per_step": dt * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u32/u64 integer",
        "data": "synthetic (seeded; stands in for the paper's expanded rcv1 shape)",
        "config": {"workload": w.name + " streamed", "n_rows": total_rows, "nnz": total_nnz, "D": w.D, "k": w.k, "b": w.b,
                   "family": w.family, "batches": n_batches, "distinct_batches_in_pinned_memory": distinct,
                   "setup_s": round(gen_s, 1)},
        "rows_per_s": total_rows / dt,
        "h2d_GBps_sustained": (4.0 * total_nnz + 8.0 * total_rows) / dt / 1e9,
        "roofline": None, "cpu_baseline": cpu_rec,
        "parity_sample_rows": n_sample if parity is not None else 0, "parity_sample_ok": parity,
    }
    print(json.dumps(rec))
    return 0 if parity in (None, True) else 1


def consumers_mode(args) -> int:
    """Times the consumers of the signature on the headline workload's own output:
    350 000 signatures of k = 500, b = 8 (175 MB), their 2^b x k expansion, and the
    equal-field counts plus resemblance estimates of random row pairs."""
    import torch
    from paper_1205_2958_amd import minhash as mh

    dev = torch.device("cuda:0")
    w = W.WORKLOADS["large_2u"]
    nnz = w.nnz(0)
    rp_np = W.row_ptr_from_nnz(nnz)
    col = W.csr_indices_torch(nnz, w.D, w.data_seed, dev)
    params_np = W.coefficients(w.k, w.family, w.param_seed)
    sig = mh.minhash_signatures(torch.from_numpy(rp_np).to(dev), col, w.D, w.k, w.b, w.family,
                                torch.from_numpy(params_np.view(np.int64)).to(dev))
    torch.cuda.synchronize()
    del col
    n, k, b = len(nnz), w.k, w.b
    n_pairs = args.pairs
    gen = torch.Generator(device=dev)
    gen.manual_seed(4242)
    pairs = torch.randint(0, n, (n_pairs, 2), generator=gen, device=dev, dtype=torch.int64)
    sizes = torch.from_numpy(nnz).to(dev)
    f1, f2 = sizes[pairs[:, 0]].contiguous(), sizes[pairs[:, 1]].contiguous()
    idx = torch.empty((n, k), dtype=torch.int32, device=dev)
    counts = torch.empty(n_pairs, dtype=torch.int32, device=dev)
    est = torch.empty(n_pairs, dtype=torch.float64, device=dev)

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / args.steps

    ms_expand = timed(lambda: mh.expand_indices(sig, k, b, out=idx))
    ms_match = timed(lambda: mh.match_counts(sig, k, b, pairs, out=counts))
    ms_est = timed(lambda: mh.resemblance_estimates(counts, f1, f2, w.D, k, b, out=est))
    # parity on a sample, against the oracle
    from oracle import oracle
    sample = slice(0, 2000)
    sig_h = sig.cpu().numpy()
    pr = pairs[sample].cpu().numpy()
    ok = bool(np.array_equal(counts[sample].cpu().numpy().view(np.uint32), oracle.match_counts(sig_h, k, b, pr)))
    ok = ok and bool(np.array_equal(idx[:64].cpu().numpy().view(np.uint32), oracle.expand(sig_h[:64], k, b)))
    bytes_match = float(n_pairs) * (2.0 * w.sig_bytes() + 16.0 + 4.0)
    bytes_expand = float(n) * (w.sig_bytes() + 4.0 * k)
    rec = {
        "metric": "row pairs compared per second (equal b-bit values of two signatures)",
        "value": n_pairs / (ms_match * 1e-3), "unit": "pairs/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_match, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u32 / f64",
        "data": "synthetic (signatures of the large_2u workload, uniformly random row pairs)",
        "config": {"workload": "consumers of large_2u signatures", "n_rows": n, "k": k, "b": b, "pairs": n_pairs},
        "roofline": {"bound": "hbm", "achieved": bytes_match / (ms_match * 1e-3) / 1e9, "peak": HBM_PEAK / 1e9,
                     "unit": "GB/s", "frac": bytes_match / (ms_match * 1e-3) / HBM_PEAK, "traffic": None,
                     "kernel": "mh_match_kernel", "kernel_ms": ms_match,
                     "model": "two signature rows + the pair + the count per pair; the 175 MB of signatures stay "
                              "resident in the 256 MB last-level cache, so the rate may exceed the HBM peak"},
        "expand": {"ms": ms_expand, "GBps": bytes_expand / (ms_expand * 1e-3) / 1e9, "rows_per_s": n / (ms_expand * 1e-3)},
        "estimates": {"ms": ms_est, "pairs_per_s": n_pairs / (ms_est * 1e-3)},
        "cpu_baseline": None, "parity_sample_ok": ok,
    }
    print(json.dumps(rec))
    return 0 if ok else 1


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="large_2u", choices=["tiny_2u", "large_2u", "large_4u", "perm_table",
                                                                 "huge_2u_m61", "large_2u_ms32", "short_rows_2u", "consumers"])
    ap.add_argument("--pairs", type=int, default=20_000_000, help="consumers: number of random row pairs")
    ap.add_argument("--rows", type=int, default=0, help="use only the first ROWS rows (debugging; invalidates the metric)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="oracle work per core for the CPU baseline (0: skip)")
    ap.add_argument("--perm-ld", type=int, default=0)
    ap.add_argument("--stream", action="store_true",
                    help="huge_2u_m61 only: all 10 batches of 200 000 rows start in pinned host memory and are streamed "
                         "host-to-device, hashed and copied back with copies and kernels overlapped; the timed region "
                         "runs from the first copy to the last signature on the host (PCIe-inclusive, reported apart)")
    ap.add_argument("--batches", type=int, default=0, help="with --stream: number of batches (default: all)")
    ap.add_argument("--distinct-batches", type=int, default=7,
                    help="with --stream: batches held in pinned host memory (8 GB each)")
    ap.add_argument("--generic-mod", action="store_true",
                    help="ablation: hash with the plain %% operator instead of the Mersenne reduction (2U/4U, p = 2^31-1)")
    ap.add_argument("--exact-fold", action="store_true",
                    help="ablation (huge_2u_m61, large_4u): the form of the reduction that is exact evaluation by "
                         "evaluation instead of the shorter form with its guard")
    ap.add_argument("--universe", type=int, default=0,
                    help="hash families with p = 2^31-1: run with this universe size D instead of the workload's power of "
                         "two (indices are folded into [0, D); a larger D leaves them as they are), e.g. 16609143 or "
                         "1010017424, to time the paths for other D")
    ap.add_argument("--calib", action="store_true",
                    help="also launch one plain streaming kernel of known size (reads 1 GiB, writes 1 GiB) so that "
                         "FETCH_SIZE / WRITE_SIZE counters of a profiler run can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this path runs on one GPU; rows are independent, so more GPUs would each take a slice of "
              "rows with no exchange, but nothing here launches a second rank (--gpus must be 1)", file=sys.stderr)
        return 2

    if args.workload == "consumers":
        return consumers_mode(args)
    w = W.WORKLOADS[args.workload]
    family = w.family
    if args.universe and (family not in ISSUE_MIX_OTHER_D or args.stream or args.generic_mod
                          or not 1 <= args.universe < (1 << 31) - 1):
        print("bench.py: --universe needs a 2U/4U workload with p = 2^31-1 and a D below the prime", file=sys.stderr)
        return 2
    D = args.universe or w.D
    if family == W.FAMILY_PERM:
        params_np = None
    else:
        params_np = W.coefficients(w.k, family, w.param_seed)

    # ---- CPU baseline first: the worker pool is forked before this process touches the GPU
    cpu_rec, n_sample, cpu_sig = None, 0, None
    if args.cpu_seconds > 0 and family != W.FAMILY_PERM:
        procs = max(1, min(16, os.cpu_count() or 1))
        # evaluations per second and core the oracle reaches on the GPU machine's host, to size the sample
        rate_guess = {W.FAMILY_2U_M31: 7.0e7, W.FAMILY_4U_M31: 2.8e7, W.FAMILY_2U_M61: 1.6e7,
                      W.FAMILY_2U_MS32: 1.0e8}[family]
        cpu_rec, n_sample, cpu_sig = cpu_baseline(w, params_np, rate_guess * args.cpu_seconds, procs, args.universe)

    import torch
    from paper_1205_2958_amd import minhash as mh

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.stream:
        return stream_mode(args, w, params_np, cpu_rec, n_sample, cpu_sig)

    nnz = w.nnz(0)
    if args.rows:
        nnz = nnz[:args.rows]
    n_rows = len(nnz)
    rp_np = W.row_ptr_from_nnz(nnz)
    total_nnz = int(rp_np[-1])
    t0 = time.perf_counter()
    col = W.csr_indices_torch(nnz, w.D, w.data_seed, dev)
    if args.universe:
        col.remainder_(D)                   # indices are below 2^31, so the int32 view is non-negative
    rp = torch.from_numpy(rp_np).to(dev)
    perm_ld = 0
    if family == W.FAMILY_PERM:
        perm_ld = args.perm_ld or w.k
        params = W.perm_table_torch(w.D, w.k, w.param_seed, dev, perm_ld=perm_ld)
    else:
        params = torch.from_numpy(params_np.view(np.int64)).to(dev)
    torch.cuda.synchronize()
    gen_s = time.perf_counter() - t0

    sig_bytes = w.sig_bytes()
    out = torch.empty((n_rows, sig_bytes), dtype=torch.uint8, device=dev)
    ws = mh.alloc_workspace(n_rows, total_nnz, w.k, family, dev)
    stream = torch.cuda.current_stream()

    flags = mh.FLAG_GENERIC_MOD if args.generic_mod else 0
    if args.exact_fold:
        if family not in (W.FAMILY_2U_M61, W.FAMILY_4U_M31) or args.stream:
            print("bench.py: --exact-fold needs the huge_2u_m61 or the large_4u workload, not streamed", file=sys.stderr)
            return 2
        flags |= mh.FLAG_EXACT_FOLD

    def step():
        mh.minhash_signatures(rp, col, D, w.k, w.b, family, params, out=out, workspace=ws, stream=stream,
                              perm_ld=perm_ld if family == W.FAMILY_PERM else None, flags=flags)

    if args.calib:
        src = torch.zeros(1 << 28, dtype=torch.int32, device=dev)
        dst = torch.empty_like(src)
        torch.add(src, 1, out=dst)          # one elementwise kernel: 2^30 bytes in, 2^30 bytes out
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    evals = float(total_nnz) * w.k
    value = evals / (dt / args.steps)

    # ---- parity of the sampled rows against the oracle output computed above
    parity = None
    if cpu_sig is not None:
        n_cmp = min(n_sample, n_rows)
        parity = bool(np.array_equal(out[:n_cmp].cpu().numpy(), cpu_sig[:n_cmp]))

    # ---- dominant kernel alone, HIP events on the launch stream
    kms = []
    for _ in range(args.steps):
        _, ms = mh.minhash_signatures_profiled(rp, col, D, w.k, w.b, family, params, out=out, workspace=ws,
                                               stream=stream, perm_ld=perm_ld if family == W.FAMILY_PERM else None,
                                               flags=flags)
        kms.append(ms)
    k_ms = float(np.mean(kms))
    if family == W.FAMILY_PERM:
        alg_bytes = float(total_nnz) * (4.0 * w.k + 4.0) + 8.0 * (n_rows + 1) + float(n_rows) * sig_bytes
        roof = {"bound": "hbm", "achieved": alg_bytes / (k_ms * 1e-3) / 1e9, "peak": HBM_PEAK / 1e9, "unit": "GB/s",
                "traffic": None, "kernel": "mh_perm_kernel", "kernel_ms": k_ms,
                "model": "4k+4 bytes per nonzero (one table row + the index) + row_ptr + packed output"}
    else:
        if D & (D - 1):
            mix = (ISSUE_MIX_OTHER_D_FRAC if D < (1 << 28) else
                   ISSUE_MIX_OTHER_D_BIG if 3 * D >= (1 << 31) - 1 else ISSUE_MIX_OTHER_D)[family]
        else:
            mix = ISSUE_MIX[family]
        slots = issue_slots(mix)
        roof = {"bound": "alu", "achieved": evals * slots / (k_ms * 1e-3) / 1e12, "peak": ALU_PEAK_SLOTS / 1e12,
                "unit": "TOP/s", "traffic": None, "kernel": "mh_hash_kernel", "kernel_ms": k_ms,
                "model": "%.2f issue slots per hash evaluation = multiply + max(full, (full + simple) / 2) with %.1f "
                         "multiplies (nothing issues beside them), %.1f other full-issue and %.1f simple instructions; "
                         "peak = 256 CU x 4 SIMD x 16 lanes x 2.4 GHz full-issue lane-slots/s, simple instructions "
                         "issuing at twice that rate and beside full-issue ones" % (slots, mix[0], mix[1], mix[2])}
    roof["frac"] = roof["achieved"] / roof["peak"]
    if not args.rows and not args.universe:
        roof["traffic"] = MEASURED_TRAFFIC_BYTES.get(w.name)

    rec = {
        "metric": "hash-evals/sec (nnz*k)",
        "value": value,
        "unit": "hash-evals/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u32/u64 integer" if family != W.FAMILY_PERM else "u32",
        "data": "synthetic (seeded; stands in for the paper's webspam / rcv1 shapes)",
        "config": {"workload": w.name + (" (generic % ablation)" if args.generic_mod else "")
                   + (" (unguarded form of the reduction on every row)" if args.exact_fold else "")
                   + (" with indices folded into D = %d" % D if args.universe else ""),
                   "n_rows": n_rows, "nnz": total_nnz, "D": D, "k": w.k, "b": w.b,
                   "family": family, "setup_s": round(gen_s, 2)},
        "rows_per_s": n_rows / (dt / args.steps),
        "roofline": roof,
        "cpu_baseline": cpu_rec,
        "parity_sample_rows": n_sample if parity is not None else 0,
        "parity_sample_ok": parity,
    }
    print(json.dumps(rec))
    return 0 if parity in (None, True) else 1


if __name__ == "__main__":
    sys.exit(main())
