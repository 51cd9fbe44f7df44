#!/usr/bin/env python3
"""Throughput of the bounded self-speculative decode path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input: the
decode phase (draft steps + verification rounds) that generates the workload's
gen_len tokens at batch 1 from a prefilled prompt, with the forced exit /
acceptance schedule of the configuration.  Weights, prompt and KV cache are
resident in HBM when the timed region starts.  Prints one JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C2]
"""
import argparse
import json
import os
import re
import sys
import time

import numpy as np

HBM_PEAK_GBS = 8000.0
ROOT = os.path.dirname(os.path.abspath(__file__))
# Where the counter-measured HBM traffic of the dominant kernel is kept: a rocprofv3 --pmc
# summary (FETCH_SIZE / WRITE_SIZE scaled by the same counters' readings on the plain copy
# kernel).  The bench line quotes the figure from that file and names it; null without it.
TRAFFIC_PROFILE = {"C2": "profiles/c2_projection_hbm_traffic.txt"}
KERNEL_PROFILE = {"C2": "profiles/c2_bench_kernel_trace.txt"}


def measured_traffic(config):
    """(bytes per launch, file) from the line 'traffic_bytes_per_launch = <number>' of the profile summary."""
    rel = TRAFFIC_PROFILE.get(config)
    if not rel:
        return None, None
    try:
        m = re.search(r"^traffic_bytes_per_launch\s*=\s*([0-9.eE+]+)", open(os.path.join(ROOT, rel)).read(), re.M)
    except OSError:
        return None, None
    return (float(m.group(1)), rel) if m else (None, None)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="C2", help="C1..C5 (sb_inputs.CONFIGS)")
    ap.add_argument("--gen", type=int, default=0, help="override the number of generated tokens")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-table", action="store_true")
    ap.add_argument("--proj", default="auto", choices=["auto", "valu", "mfma"])
    ap.add_argument("--head-mask", default="0",
                    help="variant: evaluate exit heads only at the layers of this bit mask (bit l-1 = layer l, e.g. "
                         "0xAA = even layers); forced exit layers move up to the next layer of the mask.  0 = the "
                         "paper's rule, a head after every layer (the workload the headline number is quoted on)")
    ap.add_argument("--batch", default="", help="also measure batches of these sizes (e.g. 2,4): aggregate tokens/s of B "
                    "sequences decoded together, greedy and speculative (w_max = 8 / B); reported under 'batch', not the headline")
    ap.add_argument("--copy-probe", action="store_true",
                    help="only run the plain copy kernel on 1 GiB (a yardstick of known traffic for "
                         "calibrating profiler counters) and exit")
    ap.add_argument("--head-probe", action="store_true",
                    help="only run the head projection alone (sb_op_head: RMSNorm-folded [V x d] sweep with the Eq. 2 "
                         "epilogue, then the merge) at the 7B / 32000 and the 8B / 128256 shapes, rotating over several "
                         "matrices so that no sweep finds its weights in a cache, and exit")
    ap.add_argument("--sampling-probe", action="store_true",
                    help="only time a round with greedy verification against a round with sampling-mode verification "
                         "(temperature 1.0, top-p 0.9; Sec. 4.3) on --config's shape and forced exit schedule, and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (the decode path is one sequence at batch 1); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2604_12247_amd as sb
    import sb_inputs as si

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.copy_probe:
        copy_probe(torch, sb)
        return
    if args.head_probe:
        head_probe(torch, sb)
        return
    if args.sampling_probe:
        sampling_probe(torch, sb, si, args.config)
        return
    wl = si.CONFIGS[args.config]
    shape = wl.shape
    gen_len = args.gen or wl.gen_len
    P = wl.prompt_len
    max_seq = (P + gen_len + 4 * wl.w_max + 16 + 15) // 16 * 16

    t0 = time.time()
    weights = si.make_weights(shape, wl.weight_seed)
    log(f"[bench] {wl.name}: weights generated in {time.time() - t0:.1f}s")
    t0 = time.time()
    proj = {"auto": sb.PROJ_AUTO, "valu": sb.PROJ_VALU, "mfma": sb.PROJ_MFMA}[args.proj]
    log(f"[bench] uploading the weights and packing the projections ...")
    model = sb.Model(shape, weights, max_seq, device="cuda:0", proj_kernel=proj)
    sess = model.session()
    torch.cuda.synchronize()
    log(f"[bench] uploaded and packed in {time.time() - t0:.1f}s")
    prompt = si.make_prompt(shape.vocab, P, wl.prompt_seed)
    T = wl.temperatures()

    # ---- prefill (reported separately, not part of a step)
    log(f"[bench] prefill of {P} tokens ...")
    t0 = time.perf_counter()
    first = sess.prefill(prompt)
    prefill_first_ms = (time.perf_counter() - t0) * 1e3   # includes one-off kernel loading
    warm = model.session()                                # the same prompt again, on a session of its own
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    assert warm.prefill(prompt) == first
    prefill_ms = (time.perf_counter() - t0) * 1e3
    del warm
    log(f"[bench] prefill {P} tokens: {prefill_ms:.1f} ms ({prefill_first_ms:.1f} ms the first time in the process)")

    # ---- the library's own greedy decoding: baseline and source of the continuation
    p_ar = sb.Params(0, 1, [], wl.threshold)
    n_ar = gen_len + 2 * wl.w_max
    ar_ms = []
    for i in range(2):
        sess.rewind(P, first)
        G, st = sess.decode(n_ar, p_ar)
        ar_ms.append(st["decode_ms"] / n_ar)
    ar_tok_s = 1e3 / min(ar_ms)
    ar_bytes_per_tok = (st["weight_bytes"] + st["kv_bytes"]) / n_ar
    log(f"[bench] greedy AR: {ar_tok_s:.1f} tok/s ({ar_bytes_per_tok / 1e9:.2f} GB/token, "
        f"{ar_tok_s * ar_bytes_per_tok / 1e9:.0f} GB/s algorithmic)")
    greedy = [first] + G.tolist()

    def kernel_table(allp, pair_us):
        out = {}
        for k, v in allp.items():
            raw = v["total_ms"] * 1e3 / v["launches"]
            us = max(raw - pair_us, 0.1)
            gbs = v["bytes"] / v["launches"] / us / 1e3
            out[k] = {"launches": v["launches"], "avg_us": round(us, 2), "avg_us_events_raw": round(raw, 2),
                      "GB/s": round(gbs, 1), "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4)}
        return out

    # per-kernel table of the greedy decoder: one stream, one row, nothing runs beside a kernel
    kernels_greedy = None
    if not args.no_kernel_table:
        sess.rewind(P, first)
        sess.profile_begin(None, max_launches=1 << 18)
        sess.decode(min(n_ar, 128), p_ar)
        kernels_greedy = kernel_table(sess.profile_end(), sess.empty_pair_ms * 1e3)
        for k, v in kernels_greedy.items():
            log(f"[bench]   greedy {k:12s} {v['launches']:7d} launches  {v['avg_us']:8.2f} us  {v['GB/s']:8.1f} GB/s")

    # ---- forced schedule: exit layer ~ U{exit_lo..d_max}, emitted tokens per round ~ U{1..w_max},
    # realised by draft injection so that verification is real and the output stays greedy
    accepts = si.accept_schedule(wl.sched_seed, 2 * gen_len, wl.w_max)
    fd, rounds = si.injection_schedule(greedy, accepts, wl.w_max, shape.vocab)
    fe = si.forced_exit_schedule(wl.sched_seed, len(fd), wl.exit_lo, wl.d_max)
    head_mask = int(args.head_mask, 0)
    if head_mask:
        assert (head_mask >> (wl.d_max - 1)) & 1, "the mask must contain layer d_max"
        fe = [next(l for l in range(e, wl.d_max + 1) if (head_mask >> (l - 1)) & 1) if e else 0 for e in fe]
    p_spec = sb.Params(wl.d_max, wl.w_max, T, wl.threshold, forced_exit=fe, forced_draft=fd, head_mask=head_mask)

    def step():
        sess.rewind(P, first)
        out, st = sess.decode(gen_len, p_spec)
        return out, st

    for _ in range(args.warmup):
        out, st = step()
        assert out.tolist() == greedy[1:gen_len + 1], "speculative output differs from greedy decoding"
    # dominant kernel (gate/up projection) timed live with HIP events on the library's stream
    # (every 16th launch: an event pair idles the GPU for several microseconds)
    sess.profile_begin(["gate_up"], max_launches=1 << 16, sample_every=16)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        out, st = step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    prof = sess.profile_end()
    assert out.tolist() == greedy[1:gen_len + 1], "speculative output differs from greedy decoding"
    ms_per_step = elapsed * 1e3 / args.steps
    tok_s = gen_len / (ms_per_step / 1e3)
    log(f"[bench] speculative: {tok_s:.1f} tok/s, {st['rounds']} rounds, "
        f"{st['emitted'] / st['rounds']:.2f} tokens/round, speedup {tok_s / ar_tok_s:.3f}x")

    gu = prof["gate_up"]
    # an event pair with nothing in between already reads a few microseconds: that is
    # the bracket's own cost, measured when the timing began, and is taken off
    pair_us = sess.empty_pair_ms * 1e3
    gu_raw_us = gu["total_ms"] * 1e3 / gu["launches"]
    gu_us = gu_raw_us - pair_us
    gu_bytes = gu["bytes"] / gu["launches"]
    traffic, traffic_file = measured_traffic(args.config) if not (args.gen or head_mask) else (None, None)
    # `avg_us` is what the events read minus what an empty event pair reads (the bracket's own
    # cost): the figure that agrees with rocprofv3's kernel duration in the named profile.  The
    # unsubtracted reading and the fraction it would give stand beside it.
    roofline = {"bound": "hbm", "kernel": "gate_up projection + SwiGLU (gemv_mfma_kernel<2,SWIGLU,4,packed>)",
                "achieved": round(gu_bytes / gu_us / 1e3, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(gu_bytes / gu_us / 1e3 / HBM_PEAK_GBS, 4),
                "frac_from_raw_event_time": round(gu_bytes / gu_raw_us / 1e3 / HBM_PEAK_GBS, 4),
                "traffic": traffic, "traffic_source": traffic_file,
                "traffic_note": "HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE, each scaled by "
                                "the same counter's reading on the plain copy kernel (file named in traffic_source); "
                                "null when that file does not cover this workload",
                "rocprofv3_summary": KERNEL_PROFILE.get(args.config),
                "bytes_per_launch": int(gu_bytes), "avg_us": round(gu_us, 2), "avg_us_events_raw": round(gu_raw_us, 2),
                "empty_event_pair_us": round(pair_us, 2), "timed_launches": gu["launches"],
                "timing": "HIP events on the library's stream around every 16th launch inside the timed steps; "
                          "avg_us = raw reading minus the reading of an empty event pair"}

    kernels = phases = None
    if not args.no_kernel_table:
        sess.profile_begin(None, max_launches=1 << 18)
        step()
        kernels = kernel_table(sess.profile_end(), sess.empty_pair_ms * 1e3)
        for k, v in kernels.items():
            log(f"[bench]   {k:12s} {v['launches']:7d} launches  {v['avg_us']:8.2f} us  {v['GB/s']:8.1f} GB/s")
        # time account of one more step, phase by phase (events at the phase boundaries of every round)
        sess.phase_timing(True)
        _, pst = step()
        sess.phase_timing(False)
        phases = {}
        for ph in ("draft", "align", "verify"):
            ms, by = pst[f"gpu_{ph}_ms"], pst[f"{ph}_bytes"]
            phases[ph] = {"gpu_ms": round(ms, 2), "algorithmic_GB": round(by / 1e9, 2),
                          "GB/s": round(by / 1e6 / ms, 1) if ms > 0 else None,
                          "frac_of_hbm_peak": round(by / 1e6 / ms / HBM_PEAK_GBS, 4) if ms > 0 else None}
        phases["readback_gpu_ms"] = round(pst["gpu_readback_ms"], 2)
        phases["host_enqueue_draft_ms"] = round(pst["host_draft_ms"], 2)
        phases["host_enqueue_verify_ms"] = round(pst["host_verify_ms"], 2)
        phases["host_wait_ms"] = round(pst["host_wait_ms"], 2)
        phases["note"] = ("draft: layers and exit heads of all draft steps of a round, the exit heads beside the following "
                          "layer on a second stream (bytes of both / time of the phase); verify: remaining layers + final head")
        log("[bench]   phases: " + ", ".join(f"{k} {v['gpu_ms']} ms {v['GB/s']} GB/s" for k, v in phases.items() if isinstance(v, dict)))

    # the same schedule with every exit decision read back from the device after each head, as the host
    # has to do when exits are computed rather than forced (no head beside the next layer, one wait per layer)
    readback_tok_s = None
    if not args.no_kernel_table:
        p_rb = sb.Params(wl.d_max, wl.w_max, T, wl.threshold, forced_exit=fe, forced_draft=fd, head_mask=head_mask,
                         exit_readback=True)
        best = None
        for _ in range(2):
            sess.rewind(P, first)
            out_rb, st_rb = sess.decode(gen_len, p_rb)
            best = st_rb["decode_ms"] if best is None else min(best, st_rb["decode_ms"])
        assert out_rb.tolist() == greedy[1:gen_len + 1]
        readback_tok_s = gen_len / best * 1e3
        log(f"[bench] exit decisions read back per layer: {readback_tok_s:.1f} tok/s ({readback_tok_s / tok_s:.3f} of the headline)")

    batch = None
    if args.batch:
        batch = batch_runs(sb, si, model, wl, [int(x) for x in args.batch.split(",")], min(gen_len, 256), ar_tok_s, tok_s)

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(shape, weights, prompt, wl)

    spec_bytes = st["weight_bytes"] + st["kv_bytes"]
    line = {
        "metric": "batch1_generated_tokens_per_s", "value": round(tok_s, 2), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if shape.weight_dtype == si.configs.BF16 else "f32",
        "arithmetic": ("bf16 weights x activations carried as bf16 high + low parts on the matrix cores, fp32 accumulation, "
                       "bf16 KV cache" if shape.weight_dtype == si.configs.BF16 else "fp32 on the vector ALUs"),
        "data": "synthetic",
        "config": {"workload": wl.name, "prompt_len": P, "gen_len": gen_len, "d_max": wl.d_max,
                   "w_max": wl.w_max, "threshold": wl.threshold, "T": [round(t, 4) for t in T],
                   "schedule": f"forced exit layer U[{wl.exit_lo},{wl.d_max}], tokens per round U[1,{wl.w_max}] "
                               "by draft injection; output checked equal to greedy decoding",
                   "batch": 1, **({"variant": f"exit heads only at the layers of mask {head_mask:#x}; forced exit layers "
                                              "moved up to the next such layer"} if head_mask else {})},
        "greedy_ar_tokens_per_s": round(ar_tok_s, 2), "speedup_vs_greedy_ar": round(tok_s / ar_tok_s, 4),
        "tokens_per_s_with_exit_decisions_read_back_per_layer": None if readback_tok_s is None else round(readback_tok_s, 2),
        "tokens_per_round": round(st["emitted"] / st["rounds"], 3), "prefill_ms": round(prefill_ms, 1), "prefill_first_call_ms": round(prefill_first_ms, 1),
        "algorithmic_GB_per_step": round(spec_bytes / 1e9, 2),
        "algorithmic_GBps_whole_path": round(spec_bytes / 1e6 / ms_per_step, 1),
        "greedy_algorithmic_GBps_whole_path": round(ar_tok_s * ar_bytes_per_tok / 1e9, 1),
        "batch": batch, "roofline": roofline, "kernels": kernels, "kernels_greedy": kernels_greedy, "phases": phases, "cpu_baseline": cpu,
    }
    print(json.dumps(line), flush=True)


def batch_runs(sb, si, model, wl, sizes, gen, ar1, spec1):
    """B sequences (different prompts) decoded together: aggregate generated tokens/s."""
    import torch
    shape, P = wl.shape, wl.prompt_len
    out = {}
    for B in sizes:
        w_max = max(1, min(wl.w_max, sb.SB_MAX_W // B))
        sess = [model.session() for _ in range(B)]
        prompts = [si.make_prompt(shape.vocab, P, wl.prompt_seed + 17 * (b + 1)) for b in range(B)]
        firsts = [s.prefill(p) for s, p in zip(sess, prompts)]
        bt = sb.Batch(sess)
        p_ar = sb.Params(0, 1, [], wl.threshold)
        n_ar = gen + 2 * w_max
        best = None
        for _ in range(2):
            for s, f in zip(sess, firsts):
                s.rewind(P, f)
            torch.cuda.synchronize(); t0 = time.perf_counter()
            G = bt.decode(n_ar, [p_ar] * B)
            torch.cuda.synchronize(); dt = time.perf_counter() - t0
            best = dt if best is None else min(best, dt)
        ar = B * n_ar / best
        params = []
        for b in range(B):
            greedy = [firsts[b]] + G[b].tolist()
            acc = si.accept_schedule(wl.sched_seed + b, 2 * gen, w_max)
            fd, _ = si.injection_schedule(greedy, acc, w_max, shape.vocab)
            fe = si.forced_exit_schedule(wl.sched_seed + b, len(fd), wl.exit_lo, wl.d_max)
            params.append(sb.Params(wl.d_max, w_max, wl.temperatures(), wl.threshold, forced_exit=fe, forced_draft=fd))
        best = None
        for _ in range(2):
            for s, f in zip(sess, firsts):
                s.rewind(P, f)
            torch.cuda.synchronize(); t0 = time.perf_counter()
            O = bt.decode(gen, params)
            torch.cuda.synchronize(); dt = time.perf_counter() - t0
            best = dt if best is None else min(best, dt)
        for b in range(B):
            assert O[b].tolist() == G[b].tolist()[:gen], "batched speculative output differs from greedy decoding"
        spec = B * gen / best
        out[str(B)] = {"w_max": w_max, "greedy_tokens_per_s": round(ar, 1), "speculative_tokens_per_s": round(spec, 1),
                       "greedy_vs_batch1": round(ar / ar1, 3), "speculative_vs_batch1": round(spec / spec1, 3)}
        log(f"[bench] batch {B} (w_max {w_max}): greedy {ar:.1f} tok/s ({ar / ar1:.2f}x batch 1), speculative {spec:.1f} tok/s "
            f"({spec / spec1:.2f}x batch 1's {spec1:.1f})")
        del bt, sess
    return out


def head_probe(torch, sb):
    """The exit / final head by itself (Sec. 3.2, Eq. 2): activation split + [V x d] projection + merge per call."""
    import ctypes as C
    from paper_2604_12247_amd import binding as B
    L = sb.lib()
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    for V, d in ((32000, 4096), (128256, 4096)):
        n_mat = max(2, min(6, (3 << 30) // (V * d * 2)))
        Ws = [sb.op_repack(torch.randint(-2000, 2000, (V, d), dtype=torch.int16, device="cuda")) for _ in range(n_mat)]
        for M in (1, 6):
            x = torch.randn(M, d, device="cuda")
            am = torch.empty(8, dtype=torch.int32, device="cuda")
            cf = torch.empty(8, dtype=torch.float32, device="cuda")
            scratch = torch.zeros(L.sb_op_head_scratch_bytes(M, V, d), dtype=torch.uint8, device="cuda")

            def run(W):
                B.check(L.sb_op_head(W.data_ptr(), 1, V, d, x.data_ptr(), M, 1.5, 3, am.data_ptr(), cf.data_ptr(), None,
                                     scratch.data_ptr(), st))
            for i in range(3):
                run(Ws[i % n_mat])
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(20):
                run(Ws[i % n_mat])
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / 20
            print(json.dumps({"op": "sb_op_head", "V": V, "d": d, "rows": M, "weight_bytes": V * d * 2,
                              "avg_us_three_kernels": round(us, 1),
                              "GB/s_three_kernels": round(V * d * 2 / us / 1e3, 1),
                              "frac_of_hbm_peak_three_kernels": round(V * d * 2 / us / 1e3 / HBM_PEAK_GBS, 4)}), flush=True)
        del Ws


def sampling_probe(torch, sb, si, config):
    """Cost of the sampling-mode acceptance kernel per round (Sec. 4.3): the same forced exit schedule decoded with
    greedy and with sampled verification.  Random-init exit heads propose tokens the full model gives almost no
    mass, so every round rejects its first draft and emits one drawn token: rounds of equal shape in both modes,
    whose difference is the acceptance kernel (nucleus search + draw over one row) and the logits it reads."""
    import numpy as np
    wl = si.CONFIGS[config]
    shape, P, gen = wl.shape, min(wl.prompt_len, 512), 128
    model = sb.Model(shape, si.make_weights(shape, wl.weight_seed), (P + 4 * gen + 64) // 16 * 16)
    sess = model.session()
    first = sess.prefill(si.make_prompt(shape.vocab, P, wl.prompt_seed))
    T = wl.temperatures()
    fe = si.forced_exit_schedule(wl.sched_seed, 8 * gen, wl.exit_lo, wl.d_max)
    U = np.random.default_rng(1).random(2 * (P + 4 * gen + 64)).astype(np.float32)
    res = {}
    for name, kw in (("greedy", {}), ("sampled", dict(sample_temperature=1.0, top_p=0.9, sample_u=U))):
        p = sb.Params(wl.d_max, wl.w_max, T, wl.threshold, forced_exit=fe, **kw)
        for _ in range(2):
            sess.rewind(P, first)
            _, st = sess.decode(gen, p)
        res[name] = st["decode_ms"] * 1e3 / st["rounds"]
        res[name + "_rounds"] = st["rounds"]
        res[name + "_drafts_per_round"] = st["drafts"] / st["rounds"]
    print(json.dumps({"probe": "sampling-mode verification", "workload": wl.name, "vocab": shape.vocab, "prompt": P,
                      "generated": gen, "temperature": 1.0, "top_p": 0.9,
                      "us_per_round_greedy_verification": round(res["greedy"], 1),
                      "us_per_round_sampled_verification": round(res["sampled"], 1),
                      "added_us_per_round": round(res["sampled"] - res["greedy"], 1),
                      "rounds": [res["greedy_rounds"], res["sampled_rounds"]],
                      "drafts_per_round": [round(res["greedy_drafts_per_round"], 2), round(res["sampled_drafts_per_round"], 2)]}),
          flush=True)


def copy_probe(torch, sb):
    n = 1 << 30
    src = torch.randint(0, 255, (n,), dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(2):
        sb.op_copy(dst, src)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        sb.op_copy(dst, src)
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / 5
    print(json.dumps({"kernel": "copy_kernel", "bytes_read": n, "bytes_written": n, "avg_us": round(us, 1),
                      "GB/s": round(2 * n / us / 1e3, 1)}), flush=True)


def cpu_baseline(shape, weights, prompt, wl):
    """The oracle's greedy decoding on the host cores, on a bounded sample: the double build
    (the parity reference) and the float build."""
    from oracle import Oracle, num_threads
    n_prompt = 4
    res = {}
    for bits in (64, 32):
        om = Oracle(shape, weights, 64, bits=bits)
        s = om.session()
        t0 = time.perf_counter()
        s.prefill(prompt[:n_prompt])
        per_tok = (time.perf_counter() - t0) / n_prompt
        n = int(max(2, min(24, 8.0 / max(per_tok, 1e-3))))
        t0 = time.perf_counter()
        tok = 0
        for _ in range(n):
            tok, _ = s.step(tok, want_logits=False)
        dt = time.perf_counter() - t0
        res[bits] = (n, n / dt)
        log(f"[bench] oracle ({'double' if bits == 64 else 'float'}): {n / dt:.2f} tok/s on {num_threads()} threads")
        del s, om
    return {"value": round(res[64][1], 3), "unit": "tokens/s", "cores": num_threads(), "kind": "oracle",
            "float_build_value": round(res[32][1], 3),
            "sample": f"greedy decoding of {res[64][0]} tokens after a {n_prompt}-token prompt at the {wl.name} shape, "
                      "teacher-forced: `value` is the double-precision build of the oracle (the parity reference), "
                      f"`float_build_value` its float build ({res[32][0]} tokens)"}


if __name__ == "__main__":
    main()
