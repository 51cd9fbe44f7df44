#!/usr/bin/env python3
"""Sensitivity of computed-exit decoding to its four parameters, on one GPU.

The paper's ablation (Sec. 4.3) varies the exit threshold, the annealing
coefficient of Eq. 1, the depth bound d_max and the width bound w_max one at a time
and reports wall-clock speed-up and compression rate.  Trained exit heads are not
available here, so the sweep runs on a structured synthetic model
(sb_inputs.easy_token_weights: exit heads aliased to the final head with a peaked
soft-max, more so the deeper the head; deep layers fading out), on which the Annealed
Confidence Threshold really decides every exit.  Only the shape of the curves carries over, not their values.

Every setting decodes the same continuation with exits computed on the device, is
checked token by token against the library's own greedy decoding, and is timed
against it (same prefilled state, sb_rewind + sb_decode).

    python -m paper_2604_12247_amd.sweep [--config C2] [--gen 256] [--decay 0.5 --head-scale 24 --ramp 1]
"""
import argparse
import json
import sys
import time


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="C2", help="shape and prompt of this workload (sb_inputs.CONFIGS)")
    ap.add_argument("--gen", type=int, default=256, help="tokens decoded per setting")
    ap.add_argument("--decay", type=float, default=0.5, help="per-layer fading of the output projections")
    ap.add_argument("--head-scale", type=float, default=24.0, help="gain factor of the aliased exit heads")
    ap.add_argument("--ramp", type=float, default=1.0,
                    help="0: all exit heads equally peaked; 1: peakedness grows linearly with depth")
    ap.add_argument("--threshold", type=float, default=0.5, help="centre value of the exit threshold")
    ap.add_argument("--alpha", type=float, default=0.2, help="centre value of the annealing coefficient")
    ap.add_argument("--d-max", type=int, default=0, help="centre value of the depth bound (0: the workload's)")
    ap.add_argument("--w-max", type=int, default=0, help="centre value of the width bound (0: the workload's)")
    ap.add_argument("--json", default="", help="also write the rows to this file")
    args = ap.parse_args()

    import torch
    import paper_2604_12247_amd as sb
    import sb_inputs as si

    assert torch.cuda.is_available(), "the sweep needs a GPU"
    wl = si.CONFIGS[args.config]
    shape = wl.shape
    d0 = args.d_max or wl.d_max
    w0 = args.w_max or wl.w_max
    P, gen = wl.prompt_len, args.gen
    max_seq = (P + gen + 4 * sb.SB_MAX_W + 16 + 15) // 16 * 16

    t0 = time.time()
    weights = si.easy_token_weights(shape, si.make_weights(shape, wl.weight_seed), args.decay, args.head_scale,
                                    args.ramp)
    model = sb.Model(shape, weights, max_seq, device="cuda:0")
    sess = model.session()
    log(f"[sweep] {wl.name}: structured weights (decay {args.decay}, head scale {args.head_scale}, ramp {args.ramp}) "
        f"ready in {time.time() - t0:.1f}s")
    prompt = si.make_prompt(shape.vocab, P, wl.prompt_seed)
    first = sess.prefill(prompt)

    p_ar = sb.Params(0, 1, [], 0.5)
    ar_ms = []
    for _ in range(2):
        sess.rewind(P, first)
        greedy, st = sess.decode(gen, p_ar)
        ar_ms.append(st["decode_ms"])
    ar_tok_s = gen / (min(ar_ms) / 1e3)
    greedy = greedy.tolist()
    log(f"[sweep] greedy decoding: {ar_tok_s:.1f} tokens/s")

    def run(tau, alpha, d_max, w_max):
        T = sb.temperature_schedule(alpha, shape.n_layers, d_max) if d_max else []
        p = sb.Params(d_max, w_max, T, tau)
        best = None
        for _ in range(2):
            sess.rewind(P, first)
            out, st = sess.decode(gen, p)
            assert out.tolist() == greedy, "computed-exit output differs from greedy decoding"
            if best is None or st["decode_ms"] < best["decode_ms"]:
                best = st
        st = best
        drafts, acc = st["drafts"], st["emitted"] - st["rounds"]
        return {"threshold": tau, "alpha": alpha, "d_max": d_max, "w_max": w_max,
                "tokens_per_s": round(gen / (st["decode_ms"] / 1e3), 1),
                "speedup": round(gen / (st["decode_ms"] / 1e3) / ar_tok_s, 3),
                "tokens_per_round": round(st["emitted"] / st["rounds"], 3),
                "drafts": drafts, "accepted_frac": round(acc / drafts, 3) if drafts else None,
                "mean_exit_layer": round(sum(l * n for l, n in enumerate(st["exit_hist"])) / max(1, drafts), 2),
                "layer_sweeps": st["layer_sweeps"], "head_evals": st["head_evals"]}

    grids = [("threshold", [0.1, 0.2, 0.3, 0.4, 0.5, 0.6, 0.7, 0.8, 0.9, 0.97]),
             ("alpha", [0.0, 0.1, 0.2, 0.5, 1.0, 2.0, 4.0]),
             ("d_max", [d for d in (1, 2, 3, 4, 6, 8, 10) if d <= min(shape.n_exit_heads, shape.n_layers - 1)]),
             ("w_max", [1, 2, 3, 4, 6, 8])]
    centre = {"threshold": args.threshold, "alpha": args.alpha, "d_max": d0, "w_max": w0}
    rows = []
    hdr = f"{'varied':10s} {'thr':>5s} {'alpha':>5s} {'d_max':>5s} {'w_max':>5s} {'tok/s':>8s} {'speedup':>8s} " \
          f"{'tok/round':>9s} {'drafts':>7s} {'accepted':>8s} {'exit layer':>10s} {'sweeps':>7s}"
    print(f"# {wl.name}, {gen} tokens per setting, greedy decoding {ar_tok_s:.1f} tokens/s; "
          f"structured weights: decay {args.decay}, head scale {args.head_scale}, ramp {args.ramp}")
    print(hdr)
    for name, values in grids:
        for v in values:
            s = dict(centre)
            s[name] = v
            r = run(s["threshold"], s["alpha"], s["d_max"], s["w_max"])
            r["varied"] = name
            rows.append(r)
            acc = "-" if r["accepted_frac"] is None else f"{r['accepted_frac']:.3f}"
            print(f"{name:10s} {r['threshold']:5.2f} {r['alpha']:5.2f} {r['d_max']:5d} {r['w_max']:5d} "
                  f"{r['tokens_per_s']:8.1f} {r['speedup']:8.3f} {r['tokens_per_round']:9.3f} {r['drafts']:7d} "
                  f"{acc:>8s} {r['mean_exit_layer']:10.2f} {r['layer_sweeps']:7d}", flush=True)
    if args.json:
        with open(args.json, "w") as f:
            json.dump({"workload": wl.name, "gen": gen, "greedy_tokens_per_s": ar_tok_s, "decay": args.decay,
                       "head_scale": args.head_scale, "ramp": args.ramp, "rows": rows}, f, indent=1)


if __name__ == "__main__":
    main()
