"""Writes the stored expected values under tests/golden/ for the full-size workload configurations.

Calls ONLY oracle/ (the CPU oracle) and workloads/ (seeded inputs); nothing here touches the HIP path.
For every sequence of a configuration it stores, as JSON:
  * the oracle's token-by-token greedy output ("target") and each step's top-1/top-2 margin: the sequence
    the synthetic drafts are derived from;
  * for each verification round of SpecDecode over the seeded corrupted draft (paper Section 3.2, Eq. 8-12):
    draft offset, k, alpha, bonus, the model's top-1 token at every row, every row's top-1/top-2 margin, and
    every row's four largest logits with their token ids (the set of near-maximal tokens);
  * "storage_noise": the error model of a decoder that keeps its activations in bf16: the logit deviation between
    the oracle as it is (nothing rounded) and the same oracle with every stored activation rounded to bf16, on a
    small probe (the tests size their floating-point bars for deep bf16 models from its RMS);
    "noise_floor": the deviation between two rounded evaluations that differ only in summation precision;
  * for a few rows of rounds 1-3 and of every fourth round after them, the logits at a seeded sample of
    vocabulary columns (256 of them in rounds 1-3, 32 later) plus each row's top-8 (value, index) pairs, for the element-wise logit comparison.

Every stored value comes from the oracle in its plain form (act_dtype=None: fp64, nothing rounded).

Usage:  python tests/golden/make_golden.py --config 1 [--procs 4] [--max-rounds N] [--gzip]
        python tests/golden/make_golden.py --config 4 --trim cfg4_full.json --max-rounds 16 --gzip
        python tests/golden/make_golden.py --config 3 --seqs 0:2 --greedy-head 64 --later-round 1:4096 --max-rounds 1 --gzip
The second form cuts a file this script wrote earlier down to its first N rounds per sequence (rounds are
computed one after the other, so the result equals a fresh run with --max-rounds N) without repeating hours of
CPU work.  The third form is for the long-document shape, whose token-by-token greedy target would take hours of
oracle time per page: the draft is the oracle's greedy continuation for its first G tokens (corrupted like the
configuration says) followed by seeded random tokens, and "--later-round s:C" places sequence s in a later round
of its page: C seeded random tokens stand for what earlier rounds committed (they are part of the context; the
last of them is the pending token) and the draft is the remaining draft_len - C tokens.
"""
import argparse
import gzip
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle as O          # noqa: E402
import workloads as W       # noqa: E402

N_SAMPLE_ROWS = 4
N_SAMPLE_COLS = 256


def draft_for(cfg_index, desc, seed, sp, target):
    fn = W.corrupt_draft_forced if sp.forced_different else W.corrupt_draft
    return fn(target, sp.corrupt_p, desc.vocab, seed, f"cfg{cfg_index}.{sp.seq_id}")[0]


def sample_positions(seed, cfg_index, seq_id, n_rows, vocab, rnd=0):
    g = np.random.default_rng([seed, cfg_index, seq_id] + ([rnd] if rnd else []))
    rows = np.unique(np.concatenate([[0, n_rows - 1], g.integers(0, n_rows, size=N_SAMPLE_ROWS - 2)]))
    cols = np.sort(g.choice(vocab, size=N_SAMPLE_COLS, replace=False))
    return rows, cols


def one_sequence(args):
    cfg_index, seed, sp, max_rounds, threads = args
    try:
        from threadpoolctl import threadpool_limits
        threadpool_limits(threads)
    except Exception:
        pass
    t0 = time.time()
    desc = W.CONFIGS[cfg_index].model
    weights = _WEIGHTS
    vis, prompt = W.make_prefix(desc, seed, sp.seq_id, sp.n_visual, sp.n_prompt)
    cache, pending = O.prefill(desc, weights, vis, prompt)          # the oracle as it is: nothing rounded
    n_ctx = LATER_ROUND.get(sp.seq_id, 0)
    context = None
    draft_len = sp.draft_len - n_ctx
    if n_ctx:
        # a later round of this page: n_ctx seeded random tokens stand for what earlier rounds committed
        context = np.random.default_rng([seed, cfg_index, sp.seq_id, 11]).integers(0, desc.vocab, size=n_ctx)
        feed = np.concatenate([[pending], context[:-1]])
        O.decoder_forward(desc, weights, O.embed_tokens(weights, feed), cache, want_logits=False)
        pending = int(context[-1])
    base_len = len(cache)
    explicit_draft = False
    if GREEDY_HEAD:
        # long-document shapes: the full greedy target costs hours of oracle time per page.  The draft's first
        # GREEDY_HEAD tokens are the oracle's greedy continuation, corrupted as the configuration says (a real
        # accepted run); the rest are seeded random tokens, which still exercise every row of the full-size pass
        head, hmargin = O.greedy_decode(desc, weights, cache, pending, GREEDY_HEAD, return_margins=True)
        cache.truncate(base_len)
        tail = np.random.default_rng([seed, cfg_index, sp.seq_id, 7]).integers(0, desc.vocab, size=draft_len - GREEDY_HEAD)
        target = np.concatenate([head, tail]).astype(np.int32)
        tmargin = np.concatenate([hmargin, np.zeros(len(tail))])
        draft = np.concatenate([draft_for(cfg_index, desc, seed, sp, head), tail]).astype(np.int32)
        explicit_draft = True
    else:
        target, tmargin = O.greedy_decode(desc, weights, cache, pending, draft_len, return_margins=True)
        cache.truncate(base_len)
        draft = draft_for(cfg_index, desc, seed, sp, target)
    t1 = time.time()
    rounds, committed = [], 0
    pend = pending
    while committed < draft_len and (max_rounds is None or len(rounds) < max_rounds):
        rest = draft[committed:]
        base = len(cache)
        alpha, bonus, u_hat, logits = O.verify_block(desc, weights, cache, pend, rest)
        cache.truncate(base + 1 + alpha)
        margin = O.top2_margin(logits)
        top4 = np.argpartition(-logits, 4, axis=1)[:, :4]
        order = np.argsort(-np.take_along_axis(logits, top4, axis=1), axis=1, kind="stable")
        top4 = np.take_along_axis(top4, order, axis=1)
        rec = {"offset": committed, "k": int(len(rest)), "alpha": int(alpha), "bonus": int(bonus),
               "u_hat": u_hat.tolist(), "margin": [float(f"{m:.6g}") for m in margin],
               "top4_idx": top4.tolist(),
               "top4_val": [[float(f"{x:.6g}") for x in row] for row in np.take_along_axis(logits, top4, axis=1)]}
        r = len(rounds)
        if r < 3 or r % 4 == 0:
            rows, cols = sample_positions(seed, cfg_index, sp.seq_id, logits.shape[0], desc.vocab, r)
            if r >= 3:
                cols = cols[::8]          # later rounds: every eighth of the drawn columns keeps the files small
            top_idx = np.argsort(-logits[rows], axis=1)[:, :8]
            rec["logit_samples"] = {
                "rows": rows.tolist(), "cols": cols.tolist(),
                "values": [[float(f"{x:.9g}") for x in logits[q, cols]] for q in rows],
                "top8_idx": top_idx.tolist(),
                "top8_val": [[float(f"{logits[q, j]:.9g}") for j in top_idx[i]] for i, q in enumerate(rows)]}
        rounds.append(rec)
        committed += alpha + 1
        pend = bonus
    print(f"  cfg{cfg_index} seq {sp.seq_id}: S={base_len} k={draft_len} greedy {t1 - t0:.0f}s rounds {len(rounds)} "
          f"total {time.time() - t0:.0f}s", flush=True)
    out = {"seq_id": sp.seq_id, "n_visual": sp.n_visual, "n_prompt": sp.n_prompt, "draft_len": draft_len,
           "cached_len": base_len, "pending": int(pending), "target": target.tolist(),
           "target_margin": [float(f"{m:.6g}") for m in tmargin], "rounds": rounds,
           "complete": committed >= draft_len}
    if explicit_draft:
        out["draft"] = draft.tolist()
        out["greedy_head"] = GREEDY_HEAD
    if context is not None:
        out["context_tokens"] = context.tolist()
    return out


def noise_probe(cfg_index, seed):
    """Error model of bf16 activation storage, measured by the oracle alone on a probe (256 visual rows + 64
    random draft tokens of sequence 0).  Returns (storage_noise, noise_floor):
    storage_noise = deviation of the logits when every stored activation is rounded to bf16 (the oracle's
    diagnostic act_dtype="bf16" form) from the plain fp64 oracle: what any decoder that keeps activations in bf16
    must be expected to deviate by;  noise_floor = deviation between two such rounded evaluations that differ only
    in the precision of their sums (fp64 vs fp32)."""
    desc = W.CONFIGS[cfg_index].model
    if desc.dtype != "bf16":
        z = {"rows": 65, "rms": 0.0, "max_abs": 0.0}
        return z, z
    vis, _ = W.make_prefix(desc, seed, 0, 256, 0)
    draft = np.random.default_rng([seed, cfg_index, 999]).integers(0, desc.vocab, size=64)
    out = []
    for dt, act in ((np.float64, None), (np.float64, "bf16"), (np.float32, "bf16")):
        cache, pending = O.prefill(desc, _WEIGHTS, vis, [], dt, act_dtype=act)
        out.append(O.verify_block(desc, _WEIGHTS, cache, pending, draft, dt, act_dtype=act)[3].astype(np.float64))

    def dev(d):
        return {"rows": 65, "rms": float(f"{np.sqrt((d ** 2).mean()):.4g}"), "max_abs": float(f"{np.abs(d).max():.4g}")}
    return dev(out[0] - out[1]), dev(out[1] - out[2])


_WEIGHTS = None
GREEDY_HEAD = 0
LATER_ROUND = {}


def main():
    global _WEIGHTS, GREEDY_HEAD, LATER_ROUND
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, required=True)
    ap.add_argument("--procs", type=int, default=1)
    ap.add_argument("--max-rounds", type=int, default=None)
    ap.add_argument("--seqs", type=str, default=None, help="a:b slice of the configuration's sequences")
    ap.add_argument("--out", type=str, default=None)
    ap.add_argument("--gzip", action="store_true", help="write cfgN.json.gz")
    ap.add_argument("--greedy-head", type=int, default=0,
                    help="draft = corrupted greedy continuation for this many tokens, then seeded random tokens")
    ap.add_argument("--later-round", type=str, default="",
                    help="s:C[,s:C...]: sequence s starts after C committed tokens (seeded random context)")
    ap.add_argument("--threads", type=int, default=0, help="BLAS threads per process (default: cores / procs)")
    ap.add_argument("--trim", type=str, default=None, help="existing output of this script to cut to --max-rounds")
    args = ap.parse_args()
    here = os.path.dirname(os.path.abspath(__file__))
    path = args.out or os.path.join(here, f"cfg{args.config}.json" + (".gz" if args.gzip else ""))
    if args.trim:
        with (gzip.open if args.trim.endswith(".gz") else open)(args.trim, "rt") as f:
            out = json.load(f)
        assert out["config"] == args.config and args.max_rounds
        for sq in out["sequences"]:
            if len(sq["rounds"]) > args.max_rounds:
                sq["rounds"] = sq["rounds"][: args.max_rounds]
                sq["complete"] = False
        write_out(out, path)
        return
    seed = W.SEED_BASE
    GREEDY_HEAD = args.greedy_head
    LATER_ROUND = {int(a): int(b) for a, b in (x.split(":") for x in args.later_round.split(",") if x)}
    desc = W.CONFIGS[args.config].model
    specs = W.draw_sequences(args.config, seed)
    if args.seqs:
        a, b = args.seqs.split(":")
        specs = specs[int(a):int(b)]
    _WEIGHTS = W.make_weights(desc, seed)
    O.hsd_oracle._cast_weights(_WEIGHTS, np.float64)     # cast once, before forking
    storage_noise, noise = noise_probe(args.config, seed)
    print("storage noise (plain vs bf16-rounded activations):", storage_noise, flush=True)
    print("noise floor (rounded, fp64 vs fp32 sums):", noise, flush=True)
    threads = args.threads or max(1, (os.cpu_count() or 8) // args.procs)
    jobs = [(args.config, seed, sp, args.max_rounds, threads) for sp in specs]
    t0 = time.time()
    if args.procs > 1:
        import multiprocessing as mp
        with mp.get_context("fork").Pool(args.procs) as pool:
            seqs = pool.map(one_sequence, jobs, chunksize=1)
    else:
        seqs = [one_sequence(j) for j in jobs]
    out = {"config": args.config, "seed": seed, "oracle_dtype": "float64",
           "oracle_act_dtype": None, "generator": "tests/golden/make_golden.py",
           "storage_noise": storage_noise, "noise_floor": noise, "sequences": seqs}
    write_out(out, path)
    print(f"done in {time.time() - t0:.0f}s")


def write_out(out, path):
    with (gzip.open(path, "wt", compresslevel=9) if path.endswith(".gz") else open(path, "w")) as f:
        json.dump(out, f, separators=(",", ":"))
    print(f"wrote {path} ({os.path.getsize(path) / 1e6:.2f} MB)")


if __name__ == "__main__":
    main()
