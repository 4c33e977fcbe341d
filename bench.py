#!/usr/bin/env python3
"""Benchmark of the minwise-hash signature path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload large_2u]

A step is one pass of the whole hot path (row binning, hashing with running
minima, merge of split rows, b-bit truncation and packing) over one batch of
synthetic rows that is already resident in HBM.  The headline workload is the
350 000-row, k = 500, 2U (p = 2^31 - 1) configuration the metric is quoted on.
Prints ONE JSON line: whole-job hash evaluations per second, the roofline of
the dominant kernel (duration measured with HIP events on the launch stream),
and the CPU oracle timed on this machine's host cores on a bounded, seeded,
length-stratified sample of the same rows (the sample's GPU rows are compared
with it).  Without --workload the same line carries, under "workloads", the
same measurements for the other configurations (4U on the same rows, the
permutation table, one resident batch of the heavy-tailed 2U p = 2^61 - 1
workload, the 1 000-row batch, the multiply-shift 2U that the paper times, two
million short rows), each with its own roofline and parity sample,
and four batches of the heavy-tailed workload streamed from pinned host memory
as packed index rows (copies, kernels and copies back overlapped; that rate
includes PCIe and is never the top-level value).

    python bench.py --probe      instruction-issue and memory-system probes
                                 (the denominators the rooflines are set against)
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
    # three Horner steps of 2 mad | funnel shift, add with carry out, add with carry in | mov, and; then add3, half a min3 | shr, and
    W.FAMILY_4U_M61: (6.0, 9.0 + 1.0 + 0.5, 6.0 + 2.0),
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
# 2U with p = 2^61-1 and other D up to 2^32/3 (half_2u61_steps32): the folded 61-bit value, then its residue modulo
# D' = D 2^j in 32-bit steps; one more exact quotient when D is below 2^29
ISSUE_MIX_M61_OTHER_D = (
    # mad, mad, mulhi, mad | funnel shift, add with carry out, add with carry in, funnel shift, min3, min, half a min3 |
    # mov, and, shr, add, sub, sub, add, add
    (4.0, 6.5, 8.0),
    (6.0, 6.5, 10.0),      # D below 2^29: mulhi, mad | | shr, mov
)
# 4U with p = 2^61-1 and such a D: the three Horner steps (6 mad | 9 | 6), then the same second part (mulhi, mad |
# funnel shift, min3, min, half a min3 | shr, add, sub, sub, add, add)
ISSUE_MIX_4U_M61_OTHER_D = (
    (8.0, 12.5, 12.0),
    (10.0, 12.5, 14.0),
)


def issue_slots(mix):
    mul, full, simple = mix
    return mul + max(full, (full + simple) / 2.0)


ALU_PEAK_SLOTS = 256 * 4 * 16 * 2.4e9                      # 39.3e12 lane-slots/s
HBM_PEAK = 8.0e12
# HBM bytes per launch of the dominant kernel on the full workload, from two rocprofv3 --pmc runs
# (FETCH_SIZE, WRITE_SIZE), each scaled by what the counter reads for a plain copy kernel of known
# size.  A profiler cannot run inside this process, so the figure is carried over from the committed
# summary named beside it and holds for the kernels of that summary.
PROFILED_TRAFFIC = {
    "large_2u": (6.080e9, "profiles/mh_hash_kernel_2u_m31__large_2u.txt"),
    "large_4u": (6.077e9, "profiles/mh_hash_kernel_4u_m31__large_4u.txt"),
    "perm_table": (1.16641e12, "profiles/mh_perm_kernel__perm_table.txt"),
    "huge_2u_m61": (9.374e9, "profiles/mh_hash_kernel_2u_m61__huge_2u_m61_batch0.txt"),
    "large_2u_ms32": (6.027e9, "profiles/mh_hash_kernel_2u_ms32__large_2u_ms32.txt"),
    "short_rows_2u": (1.848e9, "profiles/mh_hash_kernel_2u_m31__short_rows_2u.txt"),
}
# counter summaries (SQ_INSTS_VALU per evaluation against the model's instruction count) per family
ISSUE_MODEL_EVIDENCE = "profiles/issue_rates__probe.txt, profiles/sq_counters__hash_kernels.txt"
# evaluations per second and core the oracle reaches on the GPU machine's host, to size its samples
ORACLE_RATE_GUESS = {W.FAMILY_2U_M31: 7.0e7, W.FAMILY_4U_M31: 2.8e7, W.FAMILY_2U_M61: 1.6e7, W.FAMILY_2U_MS32: 1.0e8,
                     W.FAMILY_PERM: 6.0e7, W.FAMILY_4U_M61: 6.0e6}
SUB_WORKLOADS = ("large_4u", "perm_table", "huge_2u_m61", "tiny_2u", "large_2u_ms32", "short_rows_2u")
STREAMED_BATCHES = 4                    # batches of the streamed sub-record of a default run (all ten: --workload huge_2u_m61 --stream --packed)
SPLIT = 8192                                                # rows longer than this are cut into chunks


def issue_mix_for(family: int, D: int):
    if family == W.FAMILY_2U_M61 and D & (D - 1):
        return ISSUE_MIX_M61_OTHER_D[0 if D > (1 << 29) else 1]
    if family == W.FAMILY_4U_M61 and D & (D - 1):
        return ISSUE_MIX_4U_M61_OTHER_D[0 if D > (1 << 29) else 1]
    if D & (D - 1):
        return (ISSUE_MIX_OTHER_D_FRAC if D < (1 << 28) else
                ISSUE_MIX_OTHER_D_BIG if 3 * D >= (1 << 31) - 1 else ISSUE_MIX_OTHER_D)[family]
    return ISSUE_MIX[family]


def measure(w: W.Workload, args, pool, dev, cpu_seconds: float, universe: int = 0, flags: int = 0, perm_ld_arg: int = 0,
            rows_limit: int = 0, per_core: bool = False):
    """One workload, resident in HBM: K timed steps of the whole path, the dominant kernel
    timed by itself with HIP events, a stratified sample of rows compared with the oracle
    (timed on the host cores).  Returns the record of this workload."""
    import torch
    from paper_1205_2958_amd import minhash as mh

    family, D = w.family, universe or w.D
    nnz = w.nnz(0)
    if rows_limit:
        nnz = nnz[:rows_limit]
    n_rows = len(nnz)
    rp_np = W.row_ptr_from_nnz(nnz)
    total_nnz = int(rp_np[-1])
    evals = float(total_nnz) * w.k
    params_np = None if family == W.FAMILY_PERM else W.coefficients(w.k, family, w.param_seed)

    # ---- the sample the oracle computes: chosen by row length alone, generated on the host
    sample, cover, cpu_rec, want = None, None, None, None
    if pool is not None and cpu_seconds > 0:
        budget = ORACLE_RATE_GUESS[family] * cpu_seconds * pool.procs
        sample, cover = W.stratified_rows(nnz, w.k, budget, seed=4000 + w.data_seed, split=SPLIT, max_row_evals=budget / 4,
                                          heavy_from=100_000 if w.nnz_kind == "lomax" else None)
        s_rp = W.row_ptr_from_nnz(nnz[sample])
        s_col = W.csr_indices_np(nnz[sample], w.D, w.data_seed, rows=sample)
        if universe:
            s_col = (s_col % np.uint32(D)).astype(np.uint32)
        if family != W.FAMILY_PERM:
            want, dt, used = pool.signatures(s_rp, s_col, D, w.k, w.b, family, params_np)
            s_evals = float(s_rp[-1]) * w.k
            cpu_rec = {"value": s_evals / dt, "unit": "hash-evals/s", "cores": used, "kind": "oracle",
                       "sample": "%d rows of the workload (%s), %d nonzeros, %.3g evaluations = %.3g %% of the batch, in "
                                 "%.1f s; rows dealt to %d processes, each running the single-threaded C oracle"
                                 % (cover["rows"], cover["rule"], cover["nonzeros"], s_evals, cover["pct_of_evaluations"], dt, used),
                       "rows_per_s": cover["rows"] / dt}
            if per_core:
                # one process alone on the box: the first rows of the sample worth about a third of a shard's time
                cum = np.cumsum(np.diff(s_rp)) * w.k
                n1 = int(min(len(sample), max(1, np.searchsorted(cum, ORACLE_RATE_GUESS[family] * cpu_seconds / 3.0) + 1)))
                _, dt1, _ = pool.signatures(s_rp[:n1 + 1], s_col[:int(s_rp[n1])], D, w.k, w.b, family, params_np, procs=1)
                cpu_rec["per_core"] = {"value": float(s_rp[n1]) * w.k / dt1, "unit": "hash-evals/s", "cores": 1,
                                       "sample": "the first %d rows of the same sample (%d nonzeros) on one process, the other "
                                                 "cores idle, %.1f s" % (n1, int(s_rp[n1]), dt1)}

    # ---- the batch on the device
    t0 = time.perf_counter()
    col = W.csr_indices_torch(nnz, w.D, w.data_seed, dev)
    if universe:
        col.remainder_(D)                   # indices are below 2^31, so the int32 view is non-negative
    rp = torch.from_numpy(rp_np).to(dev)
    perm_ld = 0
    if family == W.FAMILY_PERM:
        perm_ld = perm_ld_arg or w.k
        params = W.perm_table_torch(w.D, w.k, w.param_seed, dev, perm_ld=perm_ld)
    else:
        params = torch.from_numpy(params_np.view(np.int64)).to(dev)
    torch.cuda.synchronize()
    gen_s = time.perf_counter() - t0

    sig_bytes = w.sig_bytes()
    out = torch.empty((n_rows, sig_bytes), dtype=torch.uint8, device=dev)
    ws = mh.alloc_workspace(n_rows, total_nnz, w.k, family, dev)
    stream = torch.cuda.current_stream()
    call = dict(out=out, workspace=ws, stream=stream, perm_ld=perm_ld if family == W.FAMILY_PERM else None, flags=flags)

    for _ in range(args.warmup):
        mh.minhash_signatures(rp, col, D, w.k, w.b, family, params, **call)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        mh.minhash_signatures(rp, col, D, w.k, w.b, family, params, **call)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    status = mh.status(ws)

    # ---- a call this short is launch-bound: the same call captured in a HIP graph and replayed
    graph_rec = None
    if ms_per_step < 1.0:
        eager = out.clone()
        reps = max(args.steps, 200)
        t0 = time.perf_counter()
        for _ in range(reps):
            mh.minhash_signatures(rp, col, D, w.k, w.b, family, params, **call)
        torch.cuda.synchronize()
        eager_ms = (time.perf_counter() - t0) / reps * 1e3
        graph, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
        with torch.cuda.graph(graph, stream=side):
            mh.minhash_signatures(rp, col, D, w.k, w.b, family, params, **dict(call, stream=None))
        out.zero_()
        graph.replay()
        torch.cuda.synchronize()
        same = bool(torch.equal(out, eager))
        t0 = time.perf_counter()
        for _ in range(reps):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) / reps * 1e3
        graph_rec = {"calls": reps, "eager_ms_per_step": eager_ms, "graph_replay_ms_per_step": graph_ms,
                     "replay_equals_eager": same}
        del graph, eager

    # ---- parity of the sampled rows
    parity = None
    if sample is not None:
        got = out[torch.from_numpy(sample).to(dev)].cpu().numpy()
        if family == W.FAMILY_PERM:
            # only the table rows the sample touches travel to the host, in the sample's CSR order
            take = torch.from_numpy(np.concatenate([np.arange(rp_np[r], rp_np[r + 1]) for r in sample])).to(dev)
            assert np.array_equal(col[take].cpu().numpy().view(np.uint32), s_col), "host and device generators disagree"
            table_rows = params[col[take].long(), :w.k].cpu().numpy().view(np.uint32)
            want, dt_o, used = pool.signatures(s_rp, s_col, D, w.k, w.b, family, None, table_rows=table_rows)
            s_evals = float(s_rp[-1]) * w.k
            cpu_rec = {"value": s_evals / dt_o, "unit": "gather-evals/s", "cores": used, "kind": "oracle",
                       "sample": "%d rows (%s), %d nonzeros, %.3g %% of the batch, in %.1f s on %d processes; each process "
                                 "gets the table rows of its nonzeros as a dense slice, so this is not a gather rate"
                                 % (cover["rows"], cover["rule"], cover["nonzeros"], cover["pct_of_evaluations"], dt_o, used)}
            del take, table_rows
        parity = bool(np.array_equal(got, want)) and status == 0

    # ---- dominant kernel alone, HIP events on the launch stream.  The profiled call waits for the stream, so a
    # loop of them alone would start every kernel on an idle device; each one follows a plain call without a gap
    # instead, and its kernel runs under the clocks of the timed loop above.
    kms = []
    for _ in range(args.steps):
        mh.minhash_signatures(rp, col, D, w.k, w.b, family, params, **call)
        _, ms = mh.minhash_signatures_profiled(rp, col, D, w.k, w.b, family, params, **call)
        kms.append(ms)
    k_ms = float(np.mean(kms))
    if family == W.FAMILY_PERM:
        alg_bytes = float(total_nnz) * (4.0 * w.k + 4.0) + 8.0 * (n_rows + 1) + float(n_rows) * sig_bytes
        roof = {"bound": "hbm", "achieved": alg_bytes / (k_ms * 1e-3) / 1e9, "peak": HBM_PEAK / 1e9, "unit": "GB/s",
                "traffic": None, "kernel": "mh_perm_kernel", "kernel_ms": k_ms,
                "model": "4k+4 bytes per nonzero (one table row + the index) + row_ptr + packed output"}
        try:
            from paper_1205_2958_amd import probe
            gen = torch.Generator(device=dev)
            gen.manual_seed(99)
            rows_i = torch.randint(0, params.shape[0], (1 << 22,), generator=gen, device=dev, dtype=torch.int32)
            roof["measured_ceilings_GBps"] = {
                "stream_read": probe.stream_read(params),
                "gather_%dB_rows" % (4 * w.k): probe.gather_rows(params, (4 * w.k + 15) // 16 * 16, rows_i),
                "what": "plain coalesced read of the whole table; whole table rows at 4M uniformly random row numbers, "
                        "one row per wavefront and load, 8 rows in flight (libminhash_probe.so)"}
            del rows_i
        except (FileNotFoundError, RuntimeError, AssertionError) as e:
            roof["measured_ceilings_GBps"] = {"error": str(e)}
    else:
        mix = issue_mix_for(family, D)
        slots = issue_slots(mix)
        roof = {"bound": "alu", "achieved": evals * slots / (k_ms * 1e-3) / 1e12, "peak": ALU_PEAK_SLOTS / 1e12,
                "unit": "TOP/s", "traffic": None, "kernel": "mh_hash_kernel", "kernel_ms": k_ms,
                "model": "%.2f issue slots per hash evaluation = multiply + max(full, (full + simple) / 2) with %.1f "
                         "multiplies (nothing issues beside them), %.1f other full-issue and %.1f simple instructions; "
                         "peak = 256 CU x 4 SIMD x 16 lanes x 2.4 GHz full-issue lane-slots/s, simple instructions "
                         "issuing at twice that rate and beside full-issue ones; evidence: %s"
                         % (slots, mix[0], mix[1], mix[2], ISSUE_MODEL_EVIDENCE)}
    roof["frac"] = roof["achieved"] / roof["peak"]
    if not rows_limit and not universe and not flags and w.name in PROFILED_TRAFFIC:
        roof["traffic"], roof["traffic_source"] = PROFILED_TRAFFIC[w.name]

    rec = {
        "value": evals / (dt / args.steps), "unit": "hash-evals/s", "ms_per_step": ms_per_step, "kernel_ms": k_ms,
        "rows_per_s": n_rows / (dt / args.steps),
        "config": {"workload": w.name, "n_rows": n_rows, "nnz": total_nnz, "D": D, "k": w.k, "b": w.b, "family": family,
                   "setup_s": round(gen_s, 2)},
        "roofline": roof, "cpu_baseline": cpu_rec,
        "parity_sample_rows": cover["rows"] if parity is not None else 0,
        "parity_sample_pct_of_evaluations": cover["pct_of_evaluations"] if parity is not None else 0.0,
        "parity_sample_ok": parity,
    }
    if graph_rec is not None:
        rec["hip_graph"] = graph_rec
    del col, rp, params, out, ws
    torch.cuda.empty_cache()
    return rec


def probe_mode(args) -> int:
    """Runs the device-side probes and prints one JSON line with their table."""
    import torch
    from paper_1205_2958_amd import probe

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    scratch = torch.zeros(4096, dtype=torch.int32, device=dev)
    names = probe.kinds()
    issue = {}
    for wps in (4, 5):
        for ki, name in enumerate(names):
            row = {}
            for ns in probe.N_SIMPLE:
                _, plain = probe.issue(ki, ns, False, wps, scratch)
                row["+%d" % ns] = round(plain, 3)
                if ns:
                    _, pr = probe.issue(ki, ns, True, wps, scratch)
                    row["+%d prio" % ns] = round(pr, 3)
            issue["%s, %d waves/SIMD" % (name, wps)] = row
    buf = torch.empty(1 << 30, dtype=torch.int32, device=dev)          # 4 GiB
    buf.fill_(1)
    mem = {"stream_read_GBps_4GiB": {"%d blocks/CU" % b: round(probe.stream_read(buf, blocks_per_cu=b), 1) for b in (4, 8, 16)}}
    dst = torch.empty(1 << 28, dtype=torch.int32, device=dev)
    ms = probe.copy(buf[: 1 << 28], dst, reps=3)
    mem["copy_1GiB_GBps_read_plus_write"] = round(2.0 * (1 << 30) / (ms * 1e-3) / 1e9, 1)
    del dst
    gen = torch.Generator(device=dev)
    gen.manual_seed(7)
    gathers = {}
    for row_bytes, pitch in ((800, 800), (800, 896), (896, 896), (1024, 1024), (512, 512), (256, 256)):
        n_rows = (1 << 32) // pitch // 64 * 64                         # a table of about 4 GiB
        table = buf[: n_rows * pitch // 4].view(n_rows, pitch // 4)
        rows_i = torch.randint(0, n_rows, (1 << 22,), generator=gen, device=dev, dtype=torch.int32)
        for fl in (8, 16):
            gathers["%d-byte rows, pitch %d, %d in flight" % (row_bytes, pitch, fl)] = round(
                probe.gather_rows(table, row_bytes, rows_i, in_flight=fl), 1)
    mem["gather_rows_GBps_4GiB_table"] = gathers
    print(json.dumps({"probe": "issue slots per (1 probed + n simple v_add_u32) instructions per SIMD at 2.4 GHz nominal, one "
                               "slot = one 64-lane instruction at 16 lanes per clock; 8 independent probed instructions then "
                               "n x 8 independent adds per group; 'prio' = probed run at wave priority 1, adds at 0",
                      "issue_slots": issue, "memory": mem}))
    return 0


def stream_mode(args, w, params_np, pool) -> int:
    rec = stream_record(args, w, params_np, pool, args.batches or w.n_batches(), args.packed, args.cpu_seconds)
    if pool is not None:
        pool.close()
    print(json.dumps(rec))
    return 0 if rec["parity_sample_ok"] in (None, True) else 1


def stream_record(args, w, params_np, pool, n_batches: int, packed: bool, cpu_seconds: float):
    """The heavy-tailed workload end to end: batches resident in pinned host memory,
    H2D copy / kernels / D2H copy overlapped on three streams.  Sampled rows of the
    first and of the last batch are compared with the oracle."""
    import torch
    from paper_1205_2958_amd import minhash as mh

    dev = torch.device("cuda:0")
    params = torch.from_numpy(params_np.view(np.int64)).to(dev)
    batches, total_nnz, total_rows, max_nnz = [], 0, 0, 0
    batch_nnz, batch_bytes = [], []
    t0 = time.perf_counter()
    # Pinned host memory on the GPU machine is capped near 64 GiB, less than the 80 GB of
    # indices of all ten batches: the first `distinct` batches are staged, later ones
    # re-send the staged bytes of batch (i mod distinct).  Rates are unaffected.
    distinct = min(n_batches, 10 if packed and args.distinct_batches == 7 else args.distinct_batches)
    data_of = [bi if bi < distinct else bi % distinct for bi in range(n_batches)]    # whose rows batch bi carries
    piece = 1 << 28                         # 1 GiB pieces: the pinned allocator rounds sizes up to powers of two
    max_words, sent_bytes = 0, 0.0

    def pinned_pieces(t):
        out = []
        for at in range(0, t.numel(), piece):
            h = torch.empty(min(piece, t.numel() - at), dtype=torch.int32, pin_memory=True)
            h.copy_(t[at: at + h.numel()])
            out.append(h)
        return out

    for bi in range(n_batches):
        if bi >= distinct:
            batches.append(batches[data_of[bi]])
            total_nnz += batch_nnz[data_of[bi]]
            total_rows += batches[bi][0].numel() - 1
            sent_bytes += batch_bytes[data_of[bi]]
            continue
        nnz = w.nnz(bi)
        rp_np = W.row_ptr_from_nnz(nnz)
        col = W.csr_indices_torch(nnz, w.D, w.data_seed + bi, dev)
        rp_h = torch.from_numpy(rp_np).pin_memory()
        if packed:
            width, word_ptr, words = mh.pack_indices(rp_h.to(dev), col)
            del col
            batches.append((rp_h, width.cpu().pin_memory(), word_ptr.cpu().pin_memory(), pinned_pieces(words)))
            max_words = max(max_words, words.numel())
            nbytes = 4.0 * words.numel() + 20.0 * len(nnz)
            del words
        else:
            batches.append((rp_h, pinned_pieces(col)))
            nbytes = 4.0 * col.numel() + 8.0 * len(nnz)
            del col
        batch_nnz.append(int(rp_np[-1]))
        batch_bytes.append(nbytes)
        sent_bytes += nbytes
        total_nnz += int(rp_np[-1])
        total_rows += len(nnz)
        max_nnz = max(max_nnz, int(rp_np[-1]))
        print("batch %d staged in pinned host memory: %d rows, %d nonzeros, %.2f GB to send" % (bi, len(nnz), int(rp_np[-1]), nbytes / 1e9),
              file=sys.stderr, flush=True)
    torch.cuda.synchronize()
    gen_s = time.perf_counter() - t0

    def run(bs):
        if packed:
            return mh.stream_batches_packed(bs, w.D, w.k, w.b, w.family, params, w.batch_rows, max_nnz, max_words,
                                            edge_slices=args.edge_slices)
        return mh.stream_batches(bs, w.D, w.k, w.b, w.family, params, w.batch_rows, max_nnz, edge_slices=args.edge_slices)

    run(batches[:1])                        # warm-up
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    outs = run(batches)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    evals = float(total_nnz) * w.k
    parity, n_cmp, cpu_rec, covers = None, 0, None, []
    if pool is not None and cpu_seconds > 0:
        parity = True
        budget = ORACLE_RATE_GUESS[w.family] * cpu_seconds * pool.procs / 2.0
        for bi in sorted({0, n_batches - 1}):
            src = data_of[bi]
            nnz = w.nnz(src)
            sample, cover = W.stratified_rows(nnz, w.k, budget, seed=4000 + w.data_seed + src, split=SPLIT,
                                              max_row_evals=budget / 4, heavy_from=100_000)
            s_rp = W.row_ptr_from_nnz(nnz[sample])
            s_col = W.csr_indices_np(nnz[sample], w.D, w.data_seed + src, rows=sample)
            want, dt_o, used = pool.signatures(s_rp, s_col, w.D, w.k, w.b, w.family, params_np)
            parity = parity and bool(np.array_equal(outs[bi][torch.from_numpy(sample)].numpy(), want))
            n_cmp += cover["rows"]
            covers.append("batch %d (rows of batch %d): %d rows, %d nonzeros, longest %d" % (bi, src, cover["rows"],
                                                                                          cover["nonzeros"], cover["longest_row"]))
            cpu_rec = {"value": float(s_rp[-1]) * w.k / dt_o, "unit": "hash-evals/s", "cores": used, "kind": "oracle",
                       "sample": "; ".join(covers) + "; " + cover["rule"]}
    rec = {
        "metric": "hash-evals/sec (nnz*k), host-resident batches streamed over PCIe" + (" as packed index rows" if packed else ""),
        "value": evals / dt, "unit": "hash-evals/s", "n_gpus": 1, "steps": 1, "warmup": 1, "ms_per_step": dt * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u32/u64 integer",
        "data": "synthetic (seeded; stands in for the paper's expanded rcv1 shape)",
        "config": {"workload": w.name + (" streamed as tiles of differences, decoded on the device" if packed else " streamed"), "n_rows": total_rows, "nnz": total_nnz, "D": w.D, "k": w.k, "b": w.b,
                   "family": w.family, "batches": n_batches, "distinct_batches_in_pinned_memory": distinct,
                   "setup_s": round(gen_s, 1)},
        "rows_per_s": total_rows / dt,
        "h2d_GBps_sustained": sent_bytes / dt / 1e9, "h2d_GB": sent_bytes / 1e9, "bits_per_index_sent": 8.0 * sent_bytes / total_nnz,
        "roofline": None, "cpu_baseline": cpu_rec,
        "parity_sample_rows": n_cmp, "parity_sample_ok": parity,
    }
    del batches, outs, params
    torch.cuda.empty_cache()
    return rec


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
    ap.add_argument("--workload", default="all", choices=["all", "tiny_2u", "large_2u", "large_4u", "perm_table",
                                                           "huge_2u_m61", "large_2u_ms32", "short_rows_2u", "large_4u_m61", "consumers"],
                    help="all (default): large_2u as the headline plus the other configurations as sub-records")
    ap.add_argument("--pairs", type=int, default=20_000_000, help="consumers: number of random row pairs")
    ap.add_argument("--rows", type=int, default=0, help="use only the first ROWS rows (debugging; invalidates the metric)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0,
                    help="oracle work per core for the CPU baseline of the headline workload (0: skip); the other "
                         "configurations of the default run get a fifth of it each")
    ap.add_argument("--perm-ld", type=int, default=0)
    ap.add_argument("--stream", action="store_true",
                    help="huge_2u_m61 only: all 10 batches of 200 000 rows start in pinned host memory and are streamed "
                         "host-to-device, hashed and copied back with copies and kernels overlapped; the timed region "
                         "runs from the first copy to the last signature on the host (PCIe-inclusive, reported apart)")
    ap.add_argument("--packed", action="store_true",
                    help="with --stream: the batches cross the host link as tiles of differences (about 17 bits per index "
                         "instead of 32) and are decoded on the device; all ten batches then fit pinned host memory")
    ap.add_argument("--batches", type=int, default=0, help="with --stream: number of batches (default: all)")
    ap.add_argument("--edge-slices", type=int, default=4,
                    help="with --stream: slices of rows the first and the last batch are copied and hashed in")
    ap.add_argument("--distinct-batches", type=int, default=7,
                    help="with --stream: batches held in pinned host memory (8 GB each)")
    ap.add_argument("--generic-mod", action="store_true",
                    help="ablation: hash with the plain %% operator instead of the Mersenne reduction (2U/4U, p = 2^31-1)")
    ap.add_argument("--exact-fold", action="store_true",
                    help="ablation (large_2u, large_4u, huge_2u_m61): the form of the reduction that needs no second look "
                         "at any value instead of the shorter form")
    ap.add_argument("--universe", type=int, default=0,
                    help="hash families with p = 2^31-1: run with this universe size D instead of the workload's power of "
                         "two (indices are folded into [0, D); a larger D leaves them as they are), e.g. 16609143 or "
                         "1010017424, to time the paths for other D")
    ap.add_argument("--calib", action="store_true",
                    help="also launch one plain copy kernel of known size (reads 1 GiB, writes 1 GiB) so that "
                         "FETCH_SIZE / WRITE_SIZE counters of a profiler run can be scaled")
    ap.add_argument("--probe", action="store_true", help="run the instruction-issue and memory probes instead of a workload")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this path runs on one GPU; rows are independent, so more GPUs would each take a slice of "
              "rows with no exchange, but nothing here launches a second rank (--gpus must be 1)", file=sys.stderr)
        return 2

    if args.probe:
        import torch
        if not torch.cuda.is_available():
            print("bench.py needs a GPU", file=sys.stderr)
            return 2
        return probe_mode(args)
    if args.workload == "consumers":
        return consumers_mode(args)
    headline = "large_2u" if args.workload == "all" else args.workload
    w = W.WORKLOADS[headline]
    family = w.family
    if args.universe and family in (W.FAMILY_2U_M61, W.FAMILY_4U_M61) and not args.stream and 3 <= args.universe <= (1 << 32) // 3:
        pass                                # huge_2u_m61 with another D: served in 32-bit steps up to 2^32 / 3
    elif args.universe and (family not in ISSUE_MIX_OTHER_D or args.stream or args.generic_mod
                            or not 1 <= args.universe < (1 << 31) - 1):
        print("bench.py: --universe needs a 2U/4U workload with p = 2^31-1 and a D below the prime, or huge_2u_m61 and a D of "
              "at most 2^32 / 3", file=sys.stderr)
        return 2
    flags = 0
    if args.generic_mod:
        flags |= 2
    if args.exact_fold:
        if family not in (W.FAMILY_2U_M31, W.FAMILY_2U_M61, W.FAMILY_4U_M31) or args.stream:
            print("bench.py: --exact-fold needs the large_2u, large_4u or huge_2u_m61 workload, not streamed", file=sys.stderr)
            return 2
        flags |= 4

    # ---- the oracle's worker pool is forked before this process touches the GPU
    pool = None
    if args.cpu_seconds > 0:
        from oracle.pool import OraclePool          # the cpu_baseline leg (and the parity samples it doubles as)
        pool = OraclePool(max(1, min(16, os.cpu_count() or 1)))

    import torch
    from paper_1205_2958_amd import minhash as mh  # noqa: F401  (fails loudly here if the library is missing)

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.stream:
        return stream_mode(args, w, W.coefficients(w.k, family, w.param_seed), pool)

    if args.calib:
        from paper_1205_2958_amd import probe
        src = torch.zeros(1 << 28, dtype=torch.int32, device=dev)
        dst = torch.empty_like(src)
        probe.copy(src, dst)                # one kernel: 2^30 bytes in, 2^30 bytes out (launched twice: once untimed)
        torch.cuda.synchronize()
        del src, dst

    head = measure(w, args, pool, dev, args.cpu_seconds, universe=args.universe, flags=flags, perm_ld_arg=args.perm_ld,
                   rows_limit=args.rows, per_core=True)
    ok = head["parity_sample_ok"] in (None, True)
    rec = {
        "metric": "hash-evals/sec (nnz*k)",
        "value": head["value"],
        "unit": "hash-evals/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u32/u64 integer" if family != W.FAMILY_PERM else "u32",
        "data": "synthetic (seeded; stands in for the paper's webspam / rcv1 shapes)",
        "config": dict(head["config"], workload=w.name + (" (generic % ablation)" if args.generic_mod else "")
                       + (" (form of the reduction that needs no second look, on every row)" if args.exact_fold else "")
                       + (" with indices folded into D = %d" % args.universe if args.universe else "")),
        "rows_per_s": head["rows_per_s"],
        "roofline": head["roofline"],
        "cpu_baseline": head["cpu_baseline"],
        "parity_sample_rows": head["parity_sample_rows"],
        "parity_sample_pct_of_evaluations": head["parity_sample_pct_of_evaluations"],
        "parity_sample_ok": head["parity_sample_ok"],
    }
    if "hip_graph" in head:
        rec["hip_graph"] = head["hip_graph"]
        ok = ok and head["hip_graph"]["replay_equals_eager"]
    if args.workload == "all":
        subs = {}
        # (a sub-record that fails says so in its place and in the exit status; the headline is printed regardless)
        for name in SUB_WORKLOADS:
            try:
                sub = measure(W.WORKLOADS[name], args, pool, dev, args.cpu_seconds / 5.0)
            except Exception as e:          # noqa: BLE001
                subs[name] = {"error": repr(e)}
                ok = False
                torch.cuda.empty_cache()
                continue
            ok = ok and sub["parity_sample_ok"] in (None, True) and sub.get("hip_graph", {}).get("replay_equals_eager", True)
            subs[name] = sub
            print("bench.py: %s done, %.3f ms per step" % (name, sub["ms_per_step"]), file=sys.stderr, flush=True)
        # the same workload from pinned host memory, as packed index rows (a few batches: what a default run has time for)
        hw = W.WORKLOADS["huge_2u_m61"]
        try:
            sub = stream_record(args, hw, W.coefficients(hw.k, hw.family, hw.param_seed), pool, STREAMED_BATCHES, True,
                                args.cpu_seconds / 5.0)
            ok = ok and sub["parity_sample_ok"] in (None, True)
            print("bench.py: huge_2u_m61 streamed, %d batches in %.1f ms" % (STREAMED_BATCHES, sub["ms_per_step"]), file=sys.stderr,
                  flush=True)
        except Exception as e:              # noqa: BLE001
            sub = {"error": repr(e)}
            ok = False
        subs["huge_2u_m61_streamed_packed"] = sub
        rec["workloads"] = subs
    if pool is not None:
        pool.close()
    print(json.dumps(rec))
    return 0 if ok else 1


if __name__ == "__main__":
    sys.exit(main())
