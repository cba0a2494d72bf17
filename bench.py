#!/usr/bin/env python3
"""Benchmark of the verifier hot path on one MI355X.

A step is one llm42_verify_window + llm42_commit_rollback over one batch of
synthetic input, with weights, KV cache and inputs already resident in HBM,
replayed as a HIP graph.  The model is the Llama-3.1-8B shape (32 layers, d 4096,
32 q / 8 kv heads of 128, FFN 14336, vocab 128256) with random-init bf16 weights.

Headline workload (N = 1), `c5`: the largest single-GPU configuration - 128
sequences with contexts uniform in 1024..8192, verification window 32 (4096 rows
and about 77 GB of KV per pass).  The same run then times the 32-sequence
configuration (`c3`, window 64, 2048 rows) and the single-sequence one (`c2`, 512-token
prompt, window 32) and reports them under "other_workloads".

Prints one JSON line: verified tokens/s; "roofline" for the dominant kernel (the
gate/up GEMM: MFMA bound at many rows, HBM bound at 32) and "roofline_attention" for
the attention launches (HBM bound: the KV stream), both timed with HIP events that
the library records around those launches on the stream they run on; the cost of the
fixed schedule against the same pass with the schedule lifted; and the CPU checker
timed on the host cores on sequences of the same workload, reading the same KV bytes.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0       # MI355X HBM3E
MFMA_PEAK_TFLOPS = 2500.0   # MI355X dense bf16
PMC_FILE = os.path.join(ROOT, "profiles", "pmc_traffic.txt")
WORKLOADS = {
    # name: (num_seqs, window, replacement rate, description)
    "c2": (1, 32, 0.02, "llama-3.1-8B shape random-init, 1 sequence, 512-token prompt (KV by the library's own "
                        "prefill), window 32, candidates = greedy continuation with 2% replaced"),
    # large-batch configurations: the contexts' KV is seeded noise instead of a prefill, candidates are random ids
    # (every pass commits 1 token per sequence); the verifier's work depends on neither
    "c3": (32, 64, 0.01, "llama-3.1-8B shape, 32 sequences, contexts lognormal(6.0,1.0)+lognormal(5.3,0.9) clipped "
                         "to [17, 6144], block 16, window 64; KV = seeded noise, candidates random"),
    "c5": (128, 32, 0.01, "llama-3.1-8B shape, 128 sequences, contexts uniform 1024-8192, block 16, window 32; "
                          "KV = seeded noise, candidates random"),
}
SEED, PROMPT_LEN = 42, 512


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def pmc_traffic(workload, kernel):
    """HBM-side bytes per launch from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs summarised in profiles/
    (written by `python -m paper_2601_17768_amd.pmc_traffic`).  The file records a digest of the kernel sources it
    was measured on; a figure measured on other kernels than the ones being timed is not reported (None)."""
    from paper_2601_17768_amd.build import kernel_sources_digest
    if not os.path.exists(PMC_FILE):
        return None
    entries = {}
    for line in open(PMC_FILE):
        if "=" in line and not line.lstrip().startswith("#"):
            k, v = line.split("=", 1)
            entries[k.strip()] = v.strip()
    if entries.get("kernel_sources_sha256") != kernel_sources_digest():
        return None
    v = entries.get(f"{workload}.{kernel}")
    return None if v is None else int(float(v))


def contexts_of(workload, wl, rng, num_seqs):
    import numpy as np
    if workload == "c2":
        return np.full(num_seqs, PROMPT_LEN, dtype=np.int32)
    if workload == "c3":
        return (wl.lognormal_lengths(rng, num_seqs, 6.0, 1.0, 16, 4096) +
                wl.lognormal_lengths(rng, num_seqs, 5.3, 0.9, 1, 2048)).astype(np.int32)
    return wl.uniform_lengths(rng, num_seqs, 1024, 8192)


def build_candidates(sess, kv, bt, seq_lens, first, window, rate, shape, rng):
    """Greedy continuation by iterating the verifier to its fixed point (every pass
    fixes at least one more position), then seeded random replacements."""
    import torch
    from paper_2601_17768_amd import workloads as wl
    n = seq_lens.numel()
    cand = torch.zeros((n, window), dtype=torch.int32, device=sess.device)
    cand[:, 0] = first
    for _ in range(window):
        out, _, _ = sess.verify(kv, bt, seq_lens, cand)
        new = cand.clone()
        new[:, 1:] = out[:, :-1]
        if torch.equal(new, cand):
            break
        cand = new
    host = wl.replace_candidates(rng, cand.cpu().numpy(), rate, shape.vocab)
    return torch.as_tensor(host, device=sess.device)


def cpu_baseline(shape, weights, kv, bt, contexts, cand, window, budget_s=12.0, max_seqs=4):
    """The CPU checker, as it stands, on sequences of the timed workload: each sequence's cached K and V are read
    back from the paged cache (the very bytes the timed pass read) and its window is replayed by the float64
    checker, followed by the accept rule.  Sequences are taken in order until `budget_s` seconds of checker time
    have been spent (at most `max_seqs`).  Returns the JSON object."""
    import torch
    from oracle import llm42_oracle as orc
    from paper_2601_17768_amd import kv_layout
    cfg = orc.OracleConfig(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                           shape.d_ffn, shape.vocab, shape.rope_theta, shape.rms_eps)
    cand_host = cand.cpu().numpy()
    spent, rows, used = 0.0, 0, []
    for s in range(min(max_seqs, len(contexts))):
        L = int(contexts[s])
        k, v = kv_layout.read_tokens(kv, bt[s], L, shape.head_dim)
        okv = orc.OracleKV(cfg, L + window)
        okv.k[:, :L] = k.float().cpu().double()
        okv.v[:, :L] = v.float().cpu().double()
        del k, v
        t0 = time.time()
        out, _ = orc.verify_window(cfg, weights, [okv], [L], [cand_host[s]])
        orc.commit_rollback(cand_host[s], out[0], window)
        spent += time.time() - t0
        rows += window
        used.append(L)
        del okv
        if spent >= budget_s:
            break
    return {"value": rows / spent, "unit": "verified tokens/s", "cores": torch.get_num_threads(), "kind": "oracle",
            "sample": f"{len(used)} of the workload's {len(contexts)} sequences (contexts {used}), window {window}, all "
                      f"{shape.n_layers} layers, float64 checker on the KV bytes the timed pass reads, {spent:.1f} s"}


def vendor_gemm_tflops(torch, m, n, k, reps=20):
    """torch.matmul (hipBLASLt / rocBLAS) on bf16 operands drawn like the workload's: a yardstick only."""
    a = torch.randn(m, k, device="cuda").to(torch.bfloat16)
    b = (torch.randn(n, k, device="cuda") * 0.02).to(torch.bfloat16)
    for _ in range(3):
        c = a @ b.t()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        c = a @ b.t()
    e1.record()
    torch.cuda.synchronize()
    del c
    return 2.0 * m * n * k / (e0.elapsed_time(e1) / reps * 1e-3) / 1e12


def padded_rows(rows):
    return 16 if rows <= 16 else 32 if rows <= 32 else 64 if rows <= 64 else \
        (rows + 127) // 128 * 128 if rows <= 256 else 512 if rows <= 512 else (rows + 255) // 256 * 256


def run_workload(name, sess, shape, weights, args, with_cpu_baseline):
    """Set one workload up, time it, and return its part of the JSON line."""
    import numpy as np
    import torch
    from paper_2601_17768_amd import binding as B
    from paper_2601_17768_amd import workloads as wl

    num_seqs, window, rate, desc = WORKLOADS[name]
    dev = sess.device
    t0 = time.time()
    rng = wl.rng_for(SEED, 2, 1000)
    contexts = contexts_of(name, wl, rng, num_seqs)
    max_context = int(contexts.max()) + window
    table, num_blocks = wl.make_block_table(rng, contexts + window, 16, spare_blocks=8)
    bt = torch.as_tensor(table, device=dev)
    kv = sess.kv_cache(num_blocks)
    seq_lens0 = torch.as_tensor(contexts, device=dev)
    if name == "c2":
        prompts = [wl.random_tokens(wl.rng_for(SEED, 2, s), PROMPT_LEN, shape.vocab) for s in range(num_seqs)]
        first = sess.prefill(kv, bt, prompts, window=window)
        cand = build_candidates(sess, kv, bt, seq_lens0, first, window, rate, shape, rng)
    else:
        kv.normal_(generator=torch.Generator(device=dev).manual_seed(SEED))
        cand = torch.as_tensor(wl.random_tokens(rng, num_seqs * window, shape.vocab).reshape(num_seqs, window),
                               device=dev)
    torch.cuda.synchronize()
    log(f"{name}: KV + candidates ready after {time.time() - t0:.1f}s; {int(contexts.sum())} context tokens")

    ws = sess.workspace(num_seqs, window, max_context)
    out = torch.empty((num_seqs, window), dtype=torch.int32, device=dev)
    counts = torch.empty(num_seqs, dtype=torch.int32, device=dev)
    ctoks = torch.empty((num_seqs, window), dtype=torch.int32, device=dev)
    rolled = torch.empty(num_seqs, dtype=torch.int32, device=dev)
    lens_work = seq_lens0.clone()
    steps, layers = args.steps, shape.n_layers

    def step(batch_chosen=False):
        lens_work.copy_(seq_lens0)          # the commit advances the lengths: start every step from the same state
        B.llm42_verify_window(sess.model, kv, num_blocks, bt, lens_work, cand, window, None, max_context, out,
                              ws, None, None, None, None, batch_chosen=batch_chosen)
        B.llm42_commit_rollback(cand, out, None, lens_work, counts, ctoks, rolled, None)

    def timed(fn, warm):
        """ms per step of `fn`, as a HIP graph replay unless --no-graph.  Returns (ms, the outputs of the run)."""
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        eager = out.clone()
        run = fn
        if not args.no_graph:
            # the hot calls allocate nothing and never synchronise, so a step can be captured once and
            # replayed as a HIP graph: this removes the host's per-launch cost (about 260 launches)
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                fn()
            for _ in range(2):
                graph.replay()
            torch.cuda.synchronize()
            assert args.no_check or torch.equal(out, eager), "graph replay differs from the eager step"
            run = graph.replay
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(steps):
            run()
        torch.cuda.synchronize()
        return (time.perf_counter() - t1) * 1e3 / steps, eager

    ms_per_step, eager_out = timed(step, max(1, args.warmup))
    rows = num_seqs * window
    committed = int(counts.sum())

    def launches_of(kind):
        """The same steps once more, launched one by one, with HIP events around every launch of one kernel class
        on the stream it runs on (events cannot be read back from a replayed graph).  Returns the durations in ms."""
        B.llm42_profile_enable(kind, steps * layers)
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        got = [ms for _, ms in B.llm42_profile_collect(steps * layers)]
        assert args.no_check or torch.equal(out, eager_out)
        return got

    # roofline of the gate/up GEMM, the largest kernel of the pass.  Few rows: HBM bound, algorithmic bytes per
    # launch = packed gate+up weights, read once, + the activation operand in + the SwiGLU output out.  Many rows:
    # MFMA bound, algorithmic flops per launch = 2 * rows * d_model * 2 d_ffn.
    gu = launches_of("gate_up")
    gu_ms = float(np.mean(gu))
    m_pad = padded_rows(rows)
    traffic = None if args.layers is not None else pmc_traffic(name, "gate_up")
    if rows <= 64:
        gu_bytes = 2 * shape.d_model * shape.d_ffn * 2 + m_pad * shape.d_model * 2 + m_pad * shape.d_ffn * 2
        achieved = gu_bytes / (gu_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": "gate/up GEMM + SwiGLU (gemm_xshare_kernel)",
                    "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                    "bytes_per_launch": gu_bytes, "avg_launch_ms": round(gu_ms, 5), "launches_timed": len(gu)}
    else:
        gu_flops = 2.0 * rows * shape.d_model * 2 * shape.d_ffn
        achieved = gu_flops / (gu_ms * 1e-3) / 1e12
        roofline = {"bound": "mfma", "kernel": "gate/up GEMM + SwiGLU (gemm_tiled_kernel)",
                    "achieved": round(achieved, 1), "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(achieved / MFMA_PEAK_TFLOPS, 4), "traffic": traffic,
                    "flops_per_launch": gu_flops, "avg_launch_ms": round(gu_ms, 5), "launches_timed": len(gu)}
        if with_cpu_baseline or args.vendor_gemm:
            # context, not part of the path: the vendor library's plain GEMM of the same shape and value
            # distribution on this machine (no SwiGLU), timed the same way - what this GPU sustains on real data
            roofline["vendor_gemm_same_shape_TFLOPs"] = round(vendor_gemm_tflops(torch, m_pad, 2 * shape.d_ffn, shape.d_model), 1)
    # roofline of the attention launches (one per layer: the streaming kernel, plus the merge pass where the call
    # has one): HBM bound.  Algorithmic bytes per launch = every cached K and V byte of the call's contexts and
    # windows once (the 4 query heads of a kv head share its tiles), + the query operand in + the output out.
    at = launches_of("attention")
    at_ms = float(np.mean(at))
    kv_layer = (int(contexts.sum()) + rows) * shape.kv_bytes_per_token // shape.n_layers
    at_bytes = kv_layer + 2 * rows * shape.n_q_heads * shape.head_dim * 2
    at_achieved = at_bytes / (at_ms * 1e-3) / 1e9
    roofline_attention = {"bound": "hbm", "kernel": "window attention over the paged KV cache (attention_stream_kernel / "
                          "attention_kernel + merge)", "achieved": round(at_achieved, 1), "peak": HBM_PEAK_GBS,
                          "unit": "GB/s", "frac": round(at_achieved / HBM_PEAK_GBS, 4),
                          "traffic": None if args.layers is not None else pmc_traffic(name, "attention"),
                          "bytes_per_launch": at_bytes, "avg_launch_ms": round(at_ms, 5), "launches_timed": len(at)}

    # The cost of the fixed schedule (many rows only; with few rows the two plans coincide): the same steps through
    # llm42_measure_verify_window_batch_chosen - residual projections unsplit, attention supers accumulated
    # straight through - timed the same way.  Same tile kernels both ways: a lower bound on what an engine with
    # freely chosen splits would gain.
    overhead = None
    if rows > 64:
        free_ms, free_out = timed(lambda: step(True), 1)
        step()                                  # the scheduled outputs again
        torch.cuda.synchronize()
        assert args.no_check or torch.equal(out, eager_out)
        overhead = {"fixed_schedule_ms_per_step": round(ms_per_step, 4), "batch_chosen_ms_per_step": round(free_ms, 4),
                    "overhead_frac": round(ms_per_step / free_ms - 1.0, 4),
                    "rows_with_a_different_token": int((free_out != eager_out).sum()),
                    "what": "same tile kernels both ways (a lower bound on the cost against freely chosen splits): "
                            "residual projections unsplit above 16 rows, attention supers without chunk partials "
                            "(where the work items are supers, not whole sequences)"}

    # per-class breakdown of one more (untimed) step
    B.llm42_profile_enable(None, 32 * layers)
    step()
    torch.cuda.synchronize()
    per_class = {}
    for cls, ms in B.llm42_profile_collect(32 * layers):
        per_class[cls] = per_class.get(cls, 0.0) + ms
    log(f"{name}: {ms_per_step:.3f} ms per step; kernel classes, ms per step: " +
        ", ".join(f"{k} {v:.3f}" for k, v in per_class.items()) + f"; sum {sum(per_class.values()):.3f}")
    if args.pmc_calibration:
        # one plain kernel of known HBM traffic for scaling the FETCH_SIZE / WRITE_SIZE counters: reads 256 MiB, writes 256 MiB
        cal_in = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device=dev)
        cal_out = torch.empty_like(cal_in)
        torch.cuda.synchronize()
        torch.add(cal_in, 1.0, out=cal_out)
        torch.cuda.synchronize()
        del cal_in, cal_out

    weight_bytes = shape.gemm_params * 2
    result = {
        "value": round(rows / (ms_per_step * 1e-3), 1), "unit": "tokens/s", "ms_per_step": round(ms_per_step, 4),
        "config": {"workload": f"{name}: {desc}", "num_seqs": num_seqs, "window": window,
                   "context_tokens_total": int(contexts.sum()), "max_context": max_context, "rows_per_step": rows,
                   "n_layers": layers, "committed_tokens_per_step": committed},
        "roofline": roofline, "roofline_attention": roofline_attention,
        # whole-pass view: every weight byte is streamed once per step; every row costs 2 flops per weight
        "pass_weight_stream_GBps": round(weight_bytes / (ms_per_step * 1e-3) / 1e9, 1),
        "pass_weight_stream_frac_of_hbm_peak": round(weight_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "pass_gemm_TFLOPs": round(2.0 * rows * shape.gemm_params / (ms_per_step * 1e-3) / 1e12, 1),
        "launch_mode": "eager" if args.no_graph else "hip graph replay",
        "kernel_ms_per_step": {k: round(v, 4) for k, v in per_class.items()},
    }
    if overhead is not None:
        result["determinism_overhead"] = overhead
    if with_cpu_baseline:
        log("timing the CPU checker on the host cores ...")
        result["cpu_baseline"] = cpu_baseline(shape, weights, kv, bt, contexts, cand, window)
    del kv, ws
    sess._ws = None
    torch.cuda.empty_cache()
    return result


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c5", choices=sorted(WORKLOADS), help="the headline workload of the line")
    ap.add_argument("--no-others", action="store_true", help="time the headline workload only")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--vendor-gemm", action="store_true", help="time the vendor GEMM yardstick for every workload")
    ap.add_argument("--no-graph", action="store_true", help="launch every step kernel by kernel instead of replaying a HIP graph")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run one plain elementwise kernel of known traffic (reads 256 MiB, writes 256 MiB) so "
                         "that a rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE run can be scaled to bytes")
    ap.add_argument("--layers", type=int, default=None, help="debug only: fewer layers (invalid as a result)")
    ap.add_argument("--no-check", action="store_true", help="debug only: do not compare the timed steps' outputs")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no sharding, no collectives); use --gpus 1")

    import torch
    from paper_2601_17768_amd import binding as B
    from paper_2601_17768_amd import workloads as wl
    from paper_2601_17768_amd.session import VerifierSession

    shape = wl.LLAMA_8B if args.layers is None else wl.LLAMA_8B.replace(n_layers=args.layers)
    t0 = time.time()
    weights = wl.make_weights(shape, seed=SEED)
    log(f"weights generated in {time.time() - t0:.1f}s")
    sess = VerifierSession(shape, weights, max_position=8192 + 2 * 64, device="cuda:0")
    log(f"model on device after {time.time() - t0:.1f}s; {B.llm42_schedule_info()}")

    head = run_workload(args.workload, sess, shape, weights, args, with_cpu_baseline=not args.no_cpu_baseline)
    result = {
        "metric": "verified tokens/s at 8B shape on 1 MI355X", "value": head.pop("value"), "unit": head.pop("unit"),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head.pop("ms_per_step"),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
    }
    result.update(head)
    if not args.no_others:
        result["other_workloads"] = {}
        for name in sorted(WORKLOADS, reverse=True):
            if name != args.workload:
                result["other_workloads"][name] = run_workload(name, sess, shape, weights, args, with_cpu_baseline=False)
    sess.close()
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
