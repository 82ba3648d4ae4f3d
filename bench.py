#!/usr/bin/env python3
"""Benchmark of the fused MaxSim hot path on one MI355X.

A "step" is one forward pass over the ColBERT-style reranking workload (64 queries of 32
tokens against 100 000 ragged documents, fp16, packed corpus) through the C ABI; the other
workloads of the path (the single-query streaming slice, ColPali page-as-query, the
contrastive training step with backward, int8 scoring of a 400K-page corpus) are timed as
extra legs and reported in the same JSON line.  Inputs are synthetic, seeded, and resident
in HBM before any timed region starts.  The CPU oracle is timed beside it on a bounded
sample (and checks the GPU scores of that sample on the way).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--legs c2_nq1,c3,c4,c5] [--no-cpu]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# MI355X published peaks used as roofline denominators
PEAK_HBM_GBS = 8000.0
PEAK_MFMA_16BIT_TFLOPS = 2500.0
PEAK_MFMA_I8_TOPS = 5000.0
D_MODEL = 128


def forward_flops(n_q, l_q, tokens):
    """Multiply-adds of Q D^T counted as 2 flops: 2 * N_q * L_q * (sum of L_d) * d."""
    return 2.0 * n_q * l_q * tokens * D_MODEL


def forward_bytes(n_q, l_q, tokens, n_docs, elem_bytes, ragged, scale_bytes=0):
    """Algorithmic HBM bytes of the forward: D read once, Q once, scores written once."""
    b = tokens * D_MODEL * elem_bytes + tokens * scale_bytes
    b += n_q * l_q * (D_MODEL * elem_bytes + scale_bytes)
    b += n_q * n_docs * 4
    if ragged:
        b += (n_docs + 1) * 4
    return float(b)


def backward_bytes(n_q, l_q, n_docs, l_d, elem_bytes):
    """Floor of the backward: read A and g, read Q and D once, write dQ and dD once."""
    return float(n_q * n_docs * l_q * 4 + n_q * n_docs * 4 + (n_q * l_q + n_docs * l_d) * D_MODEL * elem_bytes
                 + (n_q * l_q + n_docs * l_d) * D_MODEL * 4)


def read_traffic(key):
    """HBM bytes per launch measured with rocprofv3 --pmc, kept as 'key value' lines in profiles/traffic.txt."""
    path = os.path.join(ROOT, "profiles", "traffic.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        tok = line.split()
        if len(tok) >= 2 and tok[0] == key:
            try:
                return float(tok[1])
            except ValueError:
                return None
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--legs", default="c1,c2_nq1,c2_i8,c2_train,c3,c3_host,wide_d,c4,c5,ceilings")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--cpu-docs", type=int, default=8192, help="documents in the oracle's sample")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (--gpus %d is not supported); "
              "the path shards by documents with no communication between GPUs" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2605_29517_amd import binding as M
    from paper_2605_29517_amd import probe as P
    from paper_2605_29517_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    M.load()
    dev = "cuda:0"
    legs = [x for x in args.legs.split(",") if x]

    flush_buf = []

    def time_launches(fn, steps, warmup, cold=False):
        """W untimed steps, then K timed steps between synchronisations; one event pair per launch.
        cold=True: 512 MB are written before every timed launch (outside its event pair) so that a working set
        small enough for the L2s and the 256 MB Infinity Cache is read from HBM, as in the paper's method;
        the returned wall time is then the mean of the event times.  cold="read": the 512 MB are read instead, which
        also empties the caches of the operands but leaves no modified lines behind whose write-back the timed kernel
        would have to wait for.
        Returns (ms per step, average, median, minimum) of the event times; the last call's full statistics
        (with the interquartile range) are kept in `last_stats`."""
        if cold and not flush_buf:
            flush_buf.append(torch.empty(512 << 20, dtype=torch.uint8, device=dev))
            flush_buf[0].fill_(1)
            flush_buf.append(torch.zeros(1, dtype=torch.float32, device=dev))
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        t0 = time.perf_counter()
        for a, b in ev:
            if cold == "read":
                P.maxsim_probe_read(flush_buf[0], flush_buf[1])
            elif cold:
                flush_buf[0].fill_(1)
            a.record()
            fn()
            b.record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3 / steps
        k = sorted(a.elapsed_time(b) for a, b in ev)
        avg = sum(k) / len(k)
        q1, q3 = k[len(k) // 4], k[(3 * len(k)) // 4]
        last_stats.clear()
        last_stats.update({"avg": round(avg, 4), "median": round(k[len(k) // 2], 4), "min": round(k[0], 4),
                           "iqr": round(q3 - q1, 4), "timed": steps, "warmup": warmup,
                           "cold": "read-flush" if cold == "read" else bool(cold)})
        return (avg if cold else wall_ms), avg, k[len(k) // 2], k[0]

    last_stats = {}

    def stats():
        return dict(last_stats)

    def read_shader_clock():
        """Current shader clock in MHz from the driver's sysfs table (the line rocm-smi marks as active), or None.
        Read from a file: no child process is started from this GPU-initialised process."""
        import glob
        import re
        best = None
        for path in sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk")):
            try:
                for line in open(path):
                    if line.rstrip().endswith("*"):
                        m = re.search(r"(\d+)\s*mhz", line, re.I)
                        if m:
                            best = max(best or 0, int(m.group(1)))
            except OSError:
                pass
        return best

    def clock_under_load(fn, seconds=1.0):
        """Shader clock (MHz) read while `fn` is launched back to back for about `seconds` (None if the driver does
        not expose it)."""
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        fn()
        torch.cuda.synchronize()
        per = max(time.perf_counter() - t0, 1e-5)
        n = max(4, min(20000, int(seconds / per)))
        for _ in range(n):
            fn()
        time.sleep(min(0.5 * seconds, 0.5 * n * per))    # the queue is still draining when the clock is read
        mhz = read_shader_clock()
        torch.cuda.synchronize()
        return mhz

    def roof(bound, work, avg_ms, peak, unit, key):
        achieved = work / (avg_ms * 1e-3) / (1e9 if unit == "GB/s" else 1e12)
        t = read_traffic(key)
        return {"bound": bound, "achieved": round(achieved, 2), "peak": peak, "unit": unit,
                "frac": round(achieved / peak, 4), "traffic": t,
                "traffic_source": ("profiles/traffic.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run of this "
                                   "command; fabric traffic of the L2s, not measured in this run)") if t is not None else None}

    # ---------------- headline: config 2, ragged ColBERT rerank, 64 queries ----------------
    n_q, l_q, n_docs = 64, 32, 100_000
    Q, Dp, off, lens = W.colbert_rerank(n_q=n_q, l_q=l_q, n_docs=n_docs, device=dev)
    T = int(Dp.shape[0])
    scores = torch.empty(n_q, n_docs, dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    wall_ms, avg_ms, med_ms, min_ms = time_launches(
        lambda: M.maxsim_forward_ragged(Q, Dp, off, total_tokens=T, scores=scores), args.steps, args.warmup)
    pairs_per_s = n_q * n_docs / (wall_ms * 1e-3)
    out = {
        "metric": "docs scored/sec per query + % MFMA peak (L_q=1024) / % HBM BW (L_q=32)",
        "value": round(pairs_per_s, 1),
        "unit": "docs/s (each query's documents counted: N_q*B/t)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(wall_ms, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16",
        "data": "synthetic",
        "config": {"workload": "configs[1]: ColBERT-style rerank, N_q=64, L_q=32, d=128, B=100000 ragged L_d~U[64,300] "
                               "(packed, int32 offsets), fp16 unit-norm rows, fp32 accumulate, scores [64,100000]",
                   "total_tokens": T, "entry_point": "maxsim_forward_ragged"},
        "docs_per_s_per_query": round(n_docs / (wall_ms * 1e-3), 1),
        "kernel_ms": stats(),
        "roofline": roof("mfma", forward_flops(n_q, l_q, T), avg_ms, PEAK_MFMA_16BIT_TFLOPS, "TFLOP/s", "c2_nq64"),
        "hbm_frac_same_launch": round(forward_bytes(n_q, l_q, T, n_docs, 2, True) / (avg_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
    }
    extra = []
    out["shader_clock_mhz_under_load"] = clock_under_load(lambda: M.maxsim_forward_ragged(Q, Dp, off, total_tokens=T, scores=scores))
    out["peaks"] = {"hbm_GB_per_s": PEAK_HBM_GBS, "mfma_16bit_TFLOP_per_s": PEAK_MFMA_16BIT_TFLOPS, "mfma_i8_TOP_per_s": PEAK_MFMA_I8_TOPS,
                    "at_shader_clock_mhz": 2400,
                    "note": "published figures (256 CUs at 2.4 GHz); shader_clock_mhz_under_load beside a leg is what rocm-smi "
                            "reports while that leg's kernel runs back to back (the part lowers its clock under matrix load)"}

    # ---------------- CPU oracle on a bounded sample of the same workload ----------------
    if not args.no_cpu:
        from oracle import cpu_oracle as O
        ns = min(args.cpu_docs, n_docs)
        g = torch.Generator().manual_seed(1234)
        pick = torch.sort(torch.randperm(n_docs, generator=g)[:ns]).values
        pick[0], pick[-1] = 0, n_docs - 1
        pick = torch.unique(pick)
        lens_c, off_c = lens.cpu().long(), off.cpu().long()
        sub_len = lens_c[pick]
        sub_off = torch.zeros(len(pick) + 1, dtype=torch.int64)
        sub_off[1:] = torch.cumsum(sub_len, 0)
        rows = torch.cat([torch.arange(int(off_c[d]), int(off_c[d + 1])) for d in pick.tolist()])
        Dsub = Dp[rows.to(dev)].cpu()
        threads = max(1, min(os.cpu_count() or 1, 16))
        t0 = time.perf_counter()
        ref, _, _ = O.forward(W.to_raw_numpy(Q), W.to_raw_numpy(Dsub), "f16", offsets=sub_off.numpy().astype(np.int32),
                              want_argmax=False, want_margin=False, threads=threads)
        cpu_s = time.perf_counter() - t0
        got = scores[:, pick.to(dev)].cpu().numpy().astype(np.float64)
        rel = float(np.max(np.abs(got - ref) / np.abs(ref)))
        out["cpu_baseline"] = {"value": round(n_q * len(pick) / cpu_s, 1), "unit": out["unit"], "cores": threads,
                               "kind": "oracle", "seconds": round(cpu_s, 2),
                               "sample": "all 64 queries x %d documents drawn from the same corpus (incl. first and last)" % len(pick)}
        out["parity_on_sample"] = {"max_rel_err": rel, "tolerance": 2e-3, "ok": bool(rel <= 2e-3)}
    del scores

    # ---------------- extra legs ----------------
    if "c2_nq1" in legs:
        Q1 = Q[:1].contiguous()
        s1 = torch.empty(1, n_docs, dtype=torch.float32, device=dev)
        w, a, m, mn = time_launches(lambda: M.maxsim_forward_ragged(Q1, Dp, off, total_tokens=T, scores=s1), 50, 5)
        leg_nq1 = {"leg": "c2_nq1", "workload": "configs[1] single-query slice (N_q=1): the streaming, HBM-bound regime",
                   "kernel_ms": stats(), "ms": round(w, 4), "docs_per_s": round(n_docs / (w * 1e-3), 1), "kernel_ms_avg": round(a, 4),
                   "roofline": roof("hbm", forward_bytes(1, l_q, T, n_docs, 2, True), a, PEAK_HBM_GBS, "GB/s", "c2_nq1")}
        del s1
        # between the two regimes: the same corpus at 2 .. 24 queries (both fractions of every point: neither roof binds alone)
        sweep = []
        for nq in (2, 4, 8, 16, 24): # (not 32: that is the headline's kernel instantiation, whose profiler average it would dilute)
            if nq > Q.shape[0]:
                break
            Qn = Q[:nq].contiguous()
            sn = torch.empty(nq, n_docs, dtype=torch.float32, device=dev)
            w, a, m, mn = time_launches(lambda: M.maxsim_forward_ragged(Qn, Dp, off, total_tokens=T, scores=sn), 20, 3)
            sweep.append({"n_q": nq, "ms": round(a, 4), "hbm_frac": round(forward_bytes(nq, l_q, T, n_docs, 2, True) / (a * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                          "mfma_frac": round(2.0 * nq * l_q * T * D_MODEL / (a * 1e-3) / 1e12 / PEAK_MFMA_16BIT_TFLOPS, 4)})
            del Qn, sn
        leg_nq1["query_count_sweep"] = sweep
        extra.append(leg_nq1)
    if "c1" in legs:
        # config 1 (the parity case): 1 x 32 query tokens, 1000 x 128 document tokens, fp32 with argmax; 65.7 MB,
        # timed cold (it would sit in the Infinity Cache otherwise); report only
        Qt1, Dt1 = W.tiny_forward()
        Qt1, Dt1 = Qt1.to(dev), Dt1.to(dev)
        st1 = torch.empty(1, 1000, dtype=torch.float32, device=dev)
        at1 = torch.empty(1, 1000, 32, dtype=torch.int32, device=dev)
        w, a, m, mn = time_launches(lambda: M.maxsim_forward(Qt1, Dt1, scores=st1, argmax=at1), 50, 5, cold=True)
        by1 = forward_bytes(1, 32, 1000 * 128, 1000, 4, False) + 1000 * 32 * 4
        c1_stats = stats()
        c1_oracle = None
        if not args.no_cpu:
            # the oracle on all of config 1 (also checks the GPU's scores and argmax of this leg)
            from oracle import cpu_oracle as O
            threads = max(1, min(os.cpu_count() or 1, 16))
            t0 = time.perf_counter()
            r1, ra1, rm1 = O.forward(W.to_raw_numpy(Qt1), W.to_raw_numpy(Dt1), "f32", threads=threads)
            cs = time.perf_counter() - t0
            torch.cuda.synchronize()
            rel1 = float(np.max(np.abs(st1.cpu().numpy().astype(np.float64) - r1) / np.abs(r1)))
            clear = rm1 > 1e-3
            c1_oracle = {"docs_per_s": round(1000 / cs, 1), "seconds": round(cs, 3), "cores": threads, "sample": "all 1000 documents",
                         "max_rel_err_gpu": rel1, "argmax_equal_where_margin_clear": bool(np.array_equal(at1.cpu().numpy()[clear], ra1[clear]))}
        extra.append({"leg": "c1", "workload": "configs[0]: tiny forward with argmax, 1 x 32 x 128 fp32 query, 1000 x 128 x 128 fp32 corpus (cold)",
                      "kernel_ms": c1_stats, "cpu_oracle": c1_oracle, "ms": round(w, 4), "docs_per_s": round(1000 / (w * 1e-3), 1),
                      "roofline": roof("hbm", by1, a, PEAK_HBM_GBS, "GB/s", "c1")})
        del Qt1, Dt1, st1, at1
    if "c2_i8" in legs:
        # the same ragged corpus quantised to int8 (offline), one query quantised on the fly: streaming regime
        D8p, dsp = M.maxsim_quantize_rows_i8(Dp)
        Q1h = Q[:1].contiguous()
        q8 = torch.empty(1, l_q, D_MODEL, dtype=torch.int8, device=dev)
        qs8 = torch.empty(1, l_q, dtype=torch.float32, device=dev)
        s8 = torch.empty(1, n_docs, dtype=torch.float32, device=dev)

        def step_i8r():
            M.maxsim_quantize_rows_i8(Q1h, X_i8=q8, scale=qs8)
            M.maxsim_forward_i8_ragged(q8, qs8, D8p, dsp, off, total_tokens=T, scores=s8)
        w, a, m, mn = time_launches(step_i8r, 50, 5)
        extra.append({"leg": "c2_i8", "workload": "configs[1] corpus as int8 + fp32 scales, ragged (maxsim_forward_i8_ragged), N_q=1",
                      "ms": round(w, 4), "docs_per_s": round(n_docs / (w * 1e-3), 1), "kernel_ms_avg": round(a, 4),
                      "roofline": roof("hbm", forward_bytes(1, l_q, T, n_docs, 1, True, scale_bytes=4), a, PEAK_HBM_GBS, "GB/s", "c2_i8")})
        del D8p, dsp, s8
    if "c2_train" in legs:
        # ragged training step on a slice of the corpus: 256 queries x the first 256 documents
        nt = 256
        Tt = int(off[nt])
        Qt, Dt, offt = Q.repeat(4, 1, 1)[:nt].contiguous(), Dp[:Tt].contiguous(), off[:nt + 1].contiguous()
        st = torch.empty(nt, nt, dtype=torch.float32, device=dev)
        at = torch.empty(nt, nt, l_q, dtype=torch.int32, device=dev)
        gt = torch.empty(nt, nt, dtype=torch.float32, device=dev)
        dQt = torch.empty(nt, l_q, D_MODEL, dtype=torch.float32, device=dev)
        dDt = torch.empty(Tt, D_MODEL, dtype=torch.float32, device=dev)

        def step_rt():
            M.maxsim_forward_ragged(Qt, Dt, offt, total_tokens=Tt, scores=st, argmax=at)
            M.maxsim_ce_grad(st, 0.02, g=gt)
            M.maxsim_backward_ragged(Qt, Dt, offt, at, gt, total_tokens=Tt, dQ=dQt, dD=dDt)
        w, _, _, _ = time_launches(step_rt, 50, 5, cold=True)
        wb, ab, _, _ = time_launches(lambda: M.maxsim_backward_ragged(Qt, Dt, offt, at, gt, total_tokens=Tt, dQ=dQt, dD=dDt), 50, 5, cold=True)
        # the same step replayed from a HIP graph (its five kernels are short enough for launch gaps to count): captured
        # on a side stream after an eager call, timed back to back
        graph_ms = None
        try:
            M.maxsim_init()
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                step_rt()
                side.synchronize()
                with torch.cuda.graph(graph, stream=side):
                    step_rt()
            torch.cuda.synchronize()
            wg, _, _, _ = time_launches(graph.replay, 50, 5)
            we, _, _, _ = time_launches(step_rt, 50, 5)
            graph_ms = {"graph_replay_ms": round(wg, 4), "eager_back_to_back_ms": round(we, 4)}
            del graph
        except Exception as e:  # a capture problem must not cost the bench line
            graph_ms = {"error": repr(e)[:200]}
        extra.append({"leg": "c2_train", "workload": "ragged training step: 256 queries (L_q=32) x 256 ragged documents (%d tokens), fp16, "
                                                     "forward+argmax, CE, maxsim_backward_ragged" % Tt,
                      "step_ms": round(w, 4), "backward_ms": round(wb, 4), "pairs_per_s": round(nt * nt / (w * 1e-3), 1),
                      "hip_graph": graph_ms})
        del Qt, Dt, st, at, gt, dQt, dDt
    del Dp, Q

    if "wide_d" in legs:
        # wider embeddings (the paper's fat-embedding extension, App. "split-d"): ColPali-shaped pages, bf16;
        # d = 256 keeps the queries in registers, every wider row streams both operands in slabs of d
        wide = []
        for dw, ndw in ((256, 2000), (512, 1000), (768, 700), (1024, 500), (2048, 250)):
            Qw = W.unit_rows((4, 1024, dw), "bf16", 91, dev)
            Dw = W.unit_rows((ndw, 1024, dw), "bf16", 92, dev)
            sw = torch.empty(4, ndw, dtype=torch.float32, device=dev)
            w, a, m, mn = time_launches(lambda: M.maxsim_forward(Qw, Dw, scores=sw), 50, 5)
            fl = 2.0 * 4 * 1024 * ndw * 1024 * dw
            wide.append({"d": dw, "n_docs": ndw, "ms": round(w, 4), "kernel_ms": stats(), "TFLOP_per_s": round(fl / (a * 1e-3) / 1e12, 1),
                         "mfma_frac": round(fl / (a * 1e-3) / 1e12 / PEAK_MFMA_16BIT_TFLOPS, 4)})
            del Qw, Dw, sw
        # the shape of the paper's split-d table: one query page against 128 document pages
        small = []
        for dw in (768, 1024, 2048):
            Qw = W.unit_rows((1, 1024, dw), "bf16", 93, dev)
            Dw = W.unit_rows((128, 1024, dw), "bf16", 94, dev)
            sw = torch.empty(1, 128, dtype=torch.float32, device=dev)
            w, a, m, mn = time_launches(lambda: M.maxsim_forward(Qw, Dw, scores=sw), 50, 5)
            small.append({"d": dw, "ms": round(w, 4), "kernel_ms": stats()})
            del Qw, Dw, sw
        # int8 at the same widths and page counts (the slab kernel with i8 MFMAs; d = 128 is config 5)
        wide8 = []
        for dw, ndw in ((256, 2000), (512, 1000), (1024, 500), (2048, 250)):
            q8w, qsw = M.maxsim_quantize_rows_i8(W.unit_rows((4, 1024, dw), "f16", 95, dev))
            d8w, dsw = M.maxsim_quantize_rows_i8(W.unit_rows((ndw, 1024, dw), "bf16", 96, dev))
            sw = torch.empty(4, ndw, dtype=torch.float32, device=dev)
            w, a, m, mn = time_launches(lambda: M.maxsim_forward_i8(q8w, qsw, d8w, dsw, scores=sw), 50, 5)
            ops = 2.0 * 4 * 1024 * ndw * 1024 * dw
            wide8.append({"d": dw, "n_docs": ndw, "ms": round(w, 4), "kernel_ms": stats(), "TOP_per_s": round(ops / (a * 1e-3) / 1e12, 1),
                          "mfma_frac": round(ops / (a * 1e-3) / 1e12 / PEAK_MFMA_I8_TOPS, 4)})
            del q8w, qsw, d8w, dsw, sw
        extra.append({"leg": "wide_d", "workload": "N_q=4, L_q=L_d=1024, bf16, d=256 .. 2048 at about 2 GB of documents each; "
                                                   "and B=128, N_q=1 (the paper's split-d table); int8 at d=256 .. 2048",
                      "results": wide, "b128_single_query": small, "int8": wide8,
                      "paper_context": {"split_d_ms_A100": {"768": 2.43, "1024": 2.60, "2048": 4.91},
                                        "split_d_ms_H100": {"768": 0.76, "1024": 1.07, "2048": 2.06}}})

    if "c3" in legs or "c3_host" in legs:
        nq3, nd3, l3 = 4, 10_000, 1024
        Q3, D3 = W.colpali_page_as_query(n_q=nq3, n_docs=nd3, l=l3, device=dev)
        s3 = torch.empty(nq3, nd3, dtype=torch.float32, device=dev)
        if "c3" in legs:
            w, a, m, mn = time_launches(lambda: M.maxsim_forward(Q3, D3, scores=s3), 50, 5)
            c3_stats = stats()
            c3_clock = clock_under_load(lambda: M.maxsim_forward(Q3, D3, scores=s3))
            c3_oracle = None
            if not args.no_cpu:
                # the oracle on 4 queries x 64 documents of config 3 (first, last and 62 drawn ones); checks the GPU's scores
                from oracle import cpu_oracle as O
                g3 = torch.Generator().manual_seed(333)
                pick3 = torch.unique(torch.cat([torch.tensor([0, nd3 - 1]), torch.randperm(nd3, generator=g3)[:62]]))
                threads = max(1, min(os.cpu_count() or 1, 16))
                D3s = D3[pick3.to(dev)].cpu()
                t0 = time.perf_counter()
                r3, _, _ = O.forward(W.to_raw_numpy(Q3), W.to_raw_numpy(D3s), "bf16", want_argmax=False, want_margin=False, threads=threads)
                cs = time.perf_counter() - t0
                rel3 = float(np.max(np.abs(s3[:, pick3.to(dev)].cpu().numpy().astype(np.float64) - r3) / np.abs(r3)))
                c3_oracle = {"pairs_per_s": round(nq3 * len(pick3) / cs, 2), "seconds": round(cs, 2), "cores": threads,
                             "sample": "4 queries x %d documents" % len(pick3), "max_rel_err_gpu": rel3, "ok": bool(rel3 <= 2e-3)}
            extra.append({"leg": "c3", "workload": "configs[2]: ColPali page-as-query, N_q=4, L_q=L_d=1024, B=10000, bf16",
                          "kernel_ms": c3_stats, "shader_clock_mhz_under_load": c3_clock, "cpu_oracle": c3_oracle, "ms": round(w, 4), "pairs_per_s": round(nq3 * nd3 / (w * 1e-3), 1), "kernel_ms_avg": round(a, 4),
                          "roofline": roof("mfma", forward_flops(nq3, l3, nd3 * l3), a, PEAK_MFMA_16BIT_TFLOPS, "TFLOP/s", "c3")})
        if "c3_host" in legs:
            # the same corpus kept in page-locked host memory and streamed through a two-block device buffer
            # (out-of-core path): PCIe-inclusive, reported beside the resident figure, never as `value`
            blk = 1000
            D3h = torch.empty(D3.shape, dtype=D3.dtype, pin_memory=True)
            D3h.copy_(D3)
            stage = torch.empty(2 * blk, l3, D_MODEL, dtype=D3.dtype, device=dev)
            w, a, m, mn = time_launches(lambda: M.maxsim_forward_streamed(Q3, D3h, blk, staging=stage, scores=s3), 5, 2)
            nbytes = D3.numel() * 2
            extra.append({"leg": "c3_host", "workload": "configs[2] with the corpus in page-locked HOST memory, streamed in blocks of "
                                                        "%d documents (maxsim_forward_streamed)" % blk,
                          "ms": round(w, 3), "pairs_per_s": round(nq3 * nd3 / (w * 1e-3), 1),
                          "host_to_device_GB_per_s": round(nbytes / (w * 1e-3) / 1e9, 1)})
            del D3h, stage
        del Q3, D3, s3

    if "c4" in legs:
        n4, lq4, ld4, tau = 256, 32, 1024, 0.02
        Q4, D4 = W.contrastive_batch(n4, lq4, ld4, device=dev)
        s4 = torch.empty(n4, n4, dtype=torch.float32, device=dev)
        a4 = torch.empty(n4, n4, lq4, dtype=torch.int32, device=dev)
        g4 = torch.empty(n4, n4, dtype=torch.float32, device=dev)
        loss4 = torch.empty(1, dtype=torch.float32, device=dev)
        dQ4 = torch.empty(n4, lq4, D_MODEL, dtype=torch.float32, device=dev)
        dD4 = torch.empty(n4, ld4, D_MODEL, dtype=torch.float32, device=dev)
        # the whole working set (67 MB of D, 134 MB of dD) would sit in the Infinity Cache: timed cold (flushed)
        wf, af, _, _ = time_launches(lambda: M.maxsim_forward(Q4, D4, scores=s4, argmax=a4), 50, 5, cold=True)
        c4_fwd_stats = stats()
        wc, ac, _, _ = time_launches(lambda: M.maxsim_ce_grad(s4, tau, g=g4, loss=loss4), 50, 5, cold=True)
        wb, ab, _, _ = time_launches(lambda: M.maxsim_backward(Q4, D4, a4, g4, dQ=dQ4, dD=dD4), 50, 5, cold=True)
        c4_bwd_stats = stats()
        c4_oracle = None
        if not args.no_cpu:
            # the oracle on the whole of config 4: forward with argmax, cross-entropy gradient, backward through the
            # GPU's argmax and gradient (so both sides add the same edges); checks the GPU's scores and gradients
            from oracle import cpu_oracle as O
            threads = max(1, min(os.cpu_count() or 1, 16))
            t0 = time.perf_counter()
            r4, _, _ = O.forward(W.to_raw_numpy(Q4), W.to_raw_numpy(D4), "f16", want_argmax=True, want_margin=False, threads=threads)
            t_f = time.perf_counter() - t0
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            rQ4, rD4 = O.backward(W.to_raw_numpy(Q4), W.to_raw_numpy(D4), "f16", a4.cpu().numpy(), g4.cpu().numpy().astype(np.float64))
            t_b = time.perf_counter() - t0
            rel4 = float(np.max(np.abs(s4.cpu().numpy().astype(np.float64) - r4) / np.abs(r4)))
            eq = float(np.abs(dQ4.cpu().numpy() - rQ4).max() / np.abs(rQ4).max())
            ed = float(np.abs(dD4.cpu().numpy() - rD4).max() / np.abs(rD4).max())
            c4_oracle = {"forward_pairs_per_s": round(n4 * n4 / t_f, 1), "forward_seconds": round(t_f, 2), "backward_seconds": round(t_b, 2),
                         "cores_forward": threads, "cores_backward": 1, "sample": "all 256 x 256 pairs",
                         "max_rel_err_scores_gpu": rel4, "max_err_dQ_over_max": eq, "max_err_dD_over_max": ed,
                         "ok": bool(rel4 <= 2e-3 and eq <= 1e-4 and ed <= 1e-4)}
        wbw, _, _, _ = time_launches(lambda: M.maxsim_backward(Q4, D4, a4, g4, dQ=dQ4, dD=dD4), 50, 5)
        wbr, _, _, _ = time_launches(lambda: M.maxsim_backward(Q4, D4, a4, g4, dQ=dQ4, dD=dD4), 50, 5, cold="read")
        # the same backward with dD through the explicit CSR (Alg. 2), and the CSR build alone
        rp4 = torch.empty(n4 * ld4 + 1, dtype=torch.int32, device=dev)
        ci4 = torch.empty(n4 * n4 * lq4, dtype=torch.int32, device=dev)
        wcsr, _, _, _ = time_launches(lambda: M.maxsim_backward_csr(Q4, D4, a4, g4, row_ptr=rp4, col_idx=ci4, dQ=dQ4, dD=dD4),
                                      50, 5, cold=True)
        wcb, _, _, _ = time_launches(lambda: M.maxsim_csr_build(a4, ld4, row_ptr=rp4, col_idx=ci4), 50, 5, cold=True)
        # real argmax distributions are skewed (a few tokens win for many queries): a quarter of the edges moved to the
        # first four tokens of every document
        gen4 = torch.Generator(dev).manual_seed(44)
        hot = torch.rand(a4.shape, device=dev, generator=gen4) < 0.25
        a4h = torch.where(hot, torch.randint(0, 4, a4.shape, device=dev, generator=gen4, dtype=torch.int32), a4).contiguous()
        wsk, _, _, _ = time_launches(lambda: M.maxsim_backward(Q4, D4, a4h, g4, dQ=dQ4, dD=dD4), 50, 5, cold=True)
        del hot, a4h

        def step4():
            M.maxsim_forward(Q4, D4, scores=s4, argmax=a4)
            M.maxsim_ce_grad(s4, tau, g=g4, loss=loss4)
            M.maxsim_backward(Q4, D4, a4, g4, dQ=dQ4, dD=dD4)
        ws, _, _, _ = time_launches(step4, 50, 5, cold=True)
        wsw, _, _, _ = time_launches(step4, 50, 5)
        extra.append({"leg": "c4", "workload": "configs[3]: contrastive step, 256 queries (L_q=32) x 256 docs (L_d=1024), fp16, "
                                               "forward+argmax, CE tau=0.02, backward dQ/dD",
                      "timing": "cold: 512 MB written before every timed launch; *_cold_read_flush_ms: 512 MB read instead "
                                "(operands evicted, no modified lines left to write back); *_warm_ms: back to back, operands in cache",
                      "forward_kernel_ms": c4_fwd_stats, "backward_kernel_ms": c4_bwd_stats, "cpu_oracle": c4_oracle,
                      "step_ms": round(ws, 4), "forward_ms": round(wf, 4), "ce_ms": round(wc, 4), "backward_ms": round(wb, 4),
                      "step_warm_ms": round(wsw, 4), "backward_warm_ms": round(wbw, 4), "backward_cold_read_flush_ms": round(wbr, 4),
                      # every edge gathers one row of D (dQ) and one row of Q (dD) through the L2: the traffic that
                      # bounds this formulation, next to the `l2_gather_*` ceilings
                      "backward_gathered_bytes": 2 * n4 * n4 * lq4 * D_MODEL * 2,
                      "backward_gather_TB_per_s": round(2 * n4 * n4 * lq4 * D_MODEL * 2 / (ab * 1e-3) / 1e12, 2),
                      "backward_csr_ms": round(wcsr, 4), "csr_build_ms": round(wcb, 4),
                      "backward_skewed_argmax_ms": round(wsk, 4),
                      "pairs_per_s": round(n4 * n4 / (ws * 1e-3), 1),
                      "roofline_forward": roof("mfma", forward_flops(n4, lq4, n4 * ld4), af, PEAK_MFMA_16BIT_TFLOPS, "TFLOP/s", "c4_fwd"),
                      "roofline_backward": roof("hbm", backward_bytes(n4, lq4, n4, ld4, 2), ab, PEAK_HBM_GBS, "GB/s", "c4_bwd")})
        del Q4, D4, s4, a4, g4, dQ4, dD4, rp4, ci4

    if "c5" in legs:
        nd5, l5, chunk = 400_000, 1024, 10_000
        Qh = W.int8_query(l5, device=dev)
        D8 = torch.empty(nd5, l5, D_MODEL, dtype=torch.int8, device=dev)
        ds = torch.empty(nd5, l5, dtype=torch.float32, device=dev)
        qev = []
        for ci in range(nd5 // chunk):  # corpus quantised offline (index time), outside the step's timed region
            X = W.int8_corpus_chunk(ci, chunk, l5, device=dev)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            M.maxsim_quantize_rows_i8(X, X_i8=D8[ci * chunk:(ci + 1) * chunk], scale=ds[ci * chunk:(ci + 1) * chunk])
            e1.record()
            qev.append((e0, e1))
            del X
        torch.cuda.synchronize()
        qms = sorted(a.elapsed_time(b) for a, b in qev[1:])
        quant_ms = sum(qms) / len(qms)   # one chunk: 10.24 M fp32 rows read (512 B), codes + scale written (132 B)
        Q8 = torch.empty(1, l5, D_MODEL, dtype=torch.int8, device=dev)
        qs = torch.empty(1, l5, dtype=torch.float32, device=dev)
        s5 = torch.empty(1, nd5, dtype=torch.float32, device=dev)
        torch.cuda.synchronize()

        def step5():  # the query is quantised on the fly, inside the timed call
            M.maxsim_quantize_rows_i8(Qh, X_i8=Q8, scale=qs)
            M.maxsim_forward_i8(Q8, qs, D8, ds, scores=s5)
        w, a, m, mn = time_launches(step5, 50, 5)
        c5_stats = stats()
        c5_clock = clock_under_load(step5)
        c5_oracle = None
        if not args.no_cpu:
            # the oracle on 256 documents of config 5 (first, last, 254 drawn ones), from the GPU's codes and scales
            # (whose bit-equality with the oracle's quantiser is what tests/test_gpu_int8.py establishes): bit-exact
            from oracle import cpu_oracle as O
            g5 = torch.Generator().manual_seed(555)
            pick5 = torch.unique(torch.cat([torch.tensor([0, nd5 - 1]), torch.randperm(nd5, generator=g5)[:254]]))
            threads = max(1, min(os.cpu_count() or 1, 16))
            d8s, dss = D8[pick5.to(dev)].cpu().numpy(), ds[pick5.to(dev)].cpu().numpy()
            t0 = time.perf_counter()
            r5 = O.forward_i8(Q8.cpu().numpy(), qs.cpu().numpy(), d8s, dss, threads=threads)
            cs = time.perf_counter() - t0
            same = bool(np.array_equal(s5[:, pick5.to(dev)].cpu().numpy().view(np.uint32), r5.view(np.uint32)))
            c5_oracle = {"docs_per_s": round(len(pick5) / cs, 2), "seconds": round(cs, 2), "cores": threads,
                         "sample": "%d documents" % len(pick5), "bit_exact_gpu": same}
        extra.append({"leg": "c5", "kernel_ms": c5_stats, "shader_clock_mhz_under_load": c5_clock, "cpu_oracle": c5_oracle, "workload": "configs[4]: int8 corpus, 1 query L_q=1024 quantised on the fly, B=400000 docs "
                                               "L_d=1024 int8 + fp32 per-token scales (%.1f GB resident)" % ((D8.numel() + ds.numel() * 4) / 1e9),
                      "ms": round(w, 4), "docs_per_s": round(nd5 / (w * 1e-3), 1), "kernel_ms_avg": round(a, 4),
                      "roofline": roof("mfma", forward_flops(1, l5, nd5 * l5), a, PEAK_MFMA_I8_TOPS, "TOP/s", "c5"),
                      "quantiser": {"workload": "one corpus chunk at index time: %d fp32 rows of 128 -> int8 codes + fp32 scale" % (chunk * l5),
                                    "ms": round(quant_ms, 4),
                                    "roofline": roof("hbm", chunk * l5 * (D_MODEL * 4 + D_MODEL + 4), quant_ms, PEAK_HBM_GBS, "GB/s", "c5_quant")}})
        del D8, ds

    if "ceilings" in legs:
        # what the part sustains: register-only MFMA loops on realistic operand bits (unit-norm rows),
        # a plain read stream (a reference rate, not an upper bound: the library's streaming kernels match or pass it),
        # and a copy of known size (the calibration kernel for profiler byte counters)
        sink = torch.zeros(1, dtype=torch.float32, device=dev)
        ceil = {}
        rows16 = W.unit_rows((8192, D_MODEL), "f16", 77, dev)       # 2 MiB of fp16 operand bits
        rowsbf = W.unit_rows((8192, D_MODEL), "bf16", 78, dev)
        rows8 = torch.randint(-127, 128, (1 << 21,), dtype=torch.int8, device=dev, generator=torch.Generator(dev).manual_seed(79))
        zeros = torch.zeros(1 << 20, dtype=torch.float16, device=dev)
        for name, kind, ops, iters in (("mfma_f16_unit_norm_operands", 0, rows16, 60000), ("mfma_bf16_unit_norm_operands", 1, rowsbf, 60000),
                                       ("mfma_i8_random_operands", 2, rows8, 60000), ("mfma_f16_zero_operands", 0, zeros, 60000)):
            n_ops = P.PROBE_MFMA_OPS_PER_ITER[kind] * iters
            w, a, m, mn = time_launches(lambda: P.maxsim_probe_mfma(kind, ops, iters, sink), 8, 3)
            ceil[name] = {"ms": round(a, 3), "tera_ops_per_s": round(n_ops / (a * 1e-3) / 1e12, 1),
                          "shader_clock_mhz_under_load": clock_under_load(lambda: P.maxsim_probe_mfma(kind, ops, iters, sink))}
        big = torch.empty(1 << 30, dtype=torch.int32, device=dev)   # 4 GiB
        big.fill_(1)
        dst = torch.empty(1 << 28, dtype=torch.int32, device=dev)   # 1 GiB
        w, a, m, mn = time_launches(lambda: P.maxsim_probe_read(big, sink), 10, 3)
        ceil["hbm_read_stream_reference"] = {"ms": round(a, 3), "GB_per_s": round(big.numel() * 4 / (a * 1e-3) / 1e9, 1)}
        # the same stream with non-temporal loads (the hint slows the scoring kernels, whose load instructions take 32 bytes
        # of each of 32 lines and rely on the caches to merge them; whole-line streams gain from it)
        w, a, m, mn = time_launches(lambda: P.maxsim_probe_read(big, sink, streaming=True), 10, 3)
        ceil["hbm_read_stream_non_temporal"] = {"ms": round(a, 3), "GB_per_s": round(big.numel() * 4 / (a * 1e-3) / 1e9, 1)}
        w, a, m, mn = time_launches(lambda: P.maxsim_probe_copy(big[:1 << 28], dst), 10, 3)
        ceil["hbm_copy_1GiB"] = {"ms": round(a, 3), "GB_per_s_read_plus_write": round(2 * dst.numel() * 4 / (a * 1e-3) / 1e9, 1),
                                 "bytes_read": dst.numel() * 4, "bytes_written": dst.numel() * 4}
        # random gathers of whole 256-byte rows (the backward's access pattern: a row of D or Q per edge) from a table
        # that fits every XCD's L2 (2 MiB, the size of config 4's Q), one as large as config 4's D (64 MiB) and one
        # far beyond the caches (1 GiB): one row per load instruction (dD's walk) and four (dQ's gather)
        for label, nbytes in (("2MiB", 2 << 20), ("64MiB", 64 << 20), ("1GiB", 1 << 30)):
            table = big[:nbytes // 4]
            for kind, name in ((0, "row_per_load"), (1, "four_rows_per_load")):
                iters = 64 if kind == 0 else 32
                gathered = [0]

                def gather():
                    gathered[0] = P.maxsim_probe_gather(kind, table, iters, sink)
                w, a, m, mn = time_launches(gather, 10, 3)
                ceil["l2_gather_256B_rows_%s_table_%s" % (label, name)] = {"ms": round(a, 4), "TB_per_s": round(gathered[0] / (a * 1e-3) / 1e12, 2)}
        out["ceilings"] = ceil
        del big, dst

    out["legs"] = extra
    # the two fractions the metric names, lifted out of the legs: % of MFMA peak at L_q = L_d = 1024 (config 3)
    # and % of HBM bandwidth at L_q = 32 (single-query slice of config 2)
    by_leg = {l["leg"]: l for l in extra}
    out["metric_fractions"] = {
        "mfma_frac_lq1024": by_leg["c3"]["roofline"]["frac"] if "c3" in by_leg else None,
        "hbm_frac_lq32": by_leg["c2_nq1"]["roofline"]["frac"] if "c2_nq1" in by_leg else None,
    }
    # the same legs against what this box sustained in this run (the register-only MFMA loops and the read probe of
    # the ceilings leg): the part lowers its clock under matrix load by an amount that differs between boxes and hours
    ceil = out.get("ceilings")
    if ceil:
        def of_probe(leg, key, probe, unit):
            if leg is None or probe not in ceil:
                return None
            return round(leg["roofline"]["achieved"] / ceil[probe][unit], 4)
        out["fractions_of_this_box_probes"] = {
            "headline_of_fp16_mfma_probe": round(out["roofline"]["achieved"] / ceil["mfma_f16_unit_norm_operands"]["tera_ops_per_s"], 4)
            if "mfma_f16_unit_norm_operands" in ceil else None,
            "c3_of_bf16_mfma_probe": of_probe(by_leg.get("c3"), "c3", "mfma_bf16_unit_norm_operands", "tera_ops_per_s"),
            "c5_of_i8_mfma_probe": of_probe(by_leg.get("c5"), "c5", "mfma_i8_random_operands", "tera_ops_per_s"),
            "c2_nq1_of_read_probe": of_probe(by_leg.get("c2_nq1"), "c2_nq1", "hbm_read_stream_non_temporal", "GB_per_s"),
        }
    # context only (another machine, the authors' Triton kernels): figures the paper prints for an A100-40GB
    # (Tab. "mem", Fig. 1 caption, Sec. 1) and for the ColPali shape on an A100-80GB (Tab. "fwd_abs", inference frontier)
    out["paper_context"] = {
        "a100_40gb_peak_memory_gb_colpali_1024x1024": {"fused_B10K": 2.9, "fused_B20K": 5.2, "fused_B50K": 13.1, "fused_B100K": 26.2,
                                                       "naive_fp16_B10K": 23.9, "naive_fp16_B20K": "OOM"},
        "a100_40gb_largest_dense_corpus_docs": 175000,
        "unfused_similarity_tensor_gb_per_query_B10K": {"fp16": 21, "fp32": 42},
        "a100_80gb_fused_ms_colpali_B10K_one_query": 16.2,
        "here_device_memory_gb_config3": round((10_000 * 1024 * 128 * 2 + 4 * 1024 * 128 * 2 + 4 * 10_000 * 4) / 1e9, 2),
        "note": "the library allocates nothing: device memory is the caller's inputs and outputs",
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
