"""Benchmark of the HSD verification hot path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input: the round-1 verification of a
workload configuration: batch metadata already in HBM -> verify (KV reservation, 24-layer decoder forward over
every draft row with KV append, LM-head arg-max, acceptance scan) -> KV commit/rollback -> read back
(alpha, bonus).  Prefix prefill, weight upload and the generation of the greedy target sequence the drafts derive
from are outside the timed region (the paper's T_decode excludes prefill, Section 4.2).

The headline (`value`, `ms_per_step`, `config`) is the region-level workload, configs[1] (16 regions, 1024 visual +
32 prompt tokens of prefix each, draft lengths U[16,256], 5 % of the draft tokens corrupted).  The page-level,
long-document and ragged workloads (configs[2], [3], [4]) are timed the same way in the same run and reported
under "configs", each with the roofline of its dominant kernel; their drafts, too, derive from the model's own
greedy continuation.

Prints ONE JSON line.  `value` = verified draft tokens per second (draft rows scored / time).
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBPS = 8000.0
# Bytes that crossed the L2 <-> fabric boundary per launch of the kernel on configs[1] (fetch + write), taken
# from two rocprofv3 --pmc runs (FETCH_SIZE, then WRITE_SIZE) scaled by what the same counters read for a plain
# 2 GiB device copy; the runs and the scaling are recorded in profiles/bench_cfg1_region_verify_hbm_traffic.md.
# The counters cannot be read from inside this script; None for kernels not profiled that way.
MEASURED_TRAFFIC_BYTES = {(1, "gate_up"): 63_512_576}

WORKLOAD_TEXT = {
    1: "configs[1] region-level verify, round 1: 16 regions x (1055 cached + pending + draft U[16,256]), "
       "24-layer d1024 16q/4kv x64 FFN4096 vocab 32768, paged KV 16-token blocks",
    2: "configs[2] page-level verify, round 1: 1 page x (4127 cached + pending + 2048-token draft), same model",
    3: "configs[3] long-document verify, round 1: 4 pages x (8192 cached + pending + 8192-token draft), same model",
    4: "configs[4] ragged region verify, round 1: 64 regions x (U[512,2048] cached + pending + draft "
       "lognormal(4.5,0.8) in [8,1024]), same model",
}
DOMINANT = {1: "gate_up", 2: "attention", 3: "attention", 4: "gate_up"}


def build_workload(cfg_index, seed):
    import workloads as W
    specs = W.draw_sequences(cfg_index, seed)
    desc = W.CONFIGS[cfg_index].model
    weights = W.make_weights(desc, seed)
    return W, desc, weights, specs


def prefix_inputs(W, desc, seed, sp):
    vis, prompt = W.make_prefix(desc, seed, sp.seq_id, sp.n_visual, sp.n_prompt)
    if sp.n_prompt == 0:
        return np.full(sp.n_visual, -1, np.int32), vis, 0
    tok = np.concatenate([np.full(sp.n_visual, -1, np.int32), prompt[:-1]]).astype(np.int32)
    emb = np.concatenate([vis, np.zeros((sp.n_prompt - 1, desc.d_model), np.float32)], axis=0)
    return tok, emb, int(prompt[-1])


def cpu_baseline(W, desc, weights, seed, specs, drafts, pendings, n_sample):
    """The oracle as it stands, timed on this machine's host cores on round 1 of the first n_sample sequences
    (prefill of their prefixes is done first and not timed, as on the GPU side)."""
    import oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count()
    caches = []
    for sp in specs[:n_sample]:
        vis, prompt = W.make_prefix(desc, seed, sp.seq_id, sp.n_visual, sp.n_prompt)
        caches.append(O.prefill(desc, weights, vis, prompt)[0])
    t0 = time.perf_counter()
    rows = 0
    for i in range(n_sample):
        O.verify_block(desc, weights, caches[i], pendings[i], drafts[i])
        rows += len(drafts[i])
    dt = time.perf_counter() - t0
    return {"value": rows / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"round-1 verification of the first {n_sample} of {len(specs)} regions "
                      f"({rows} draft tokens, fp64 numpy, {dt:.1f} s; prefix prefill not timed)"}


def attention_work(desc, prefix_len, q_len):
    """Algorithmic flops and bytes of one attention launch (one layer): every (query, visible key) pair, each
    sequence's K/V read once, Q read and O written once."""
    flops = sum(4.0 * desc.n_q_heads * desc.head_dim * (l * s_ + l * (l + 1) / 2) for s_, l in zip(prefix_len, q_len))
    kv_bytes = sum((s_ + l) * desc.n_kv_heads * desc.head_dim * 2 * 2 for s_, l in zip(prefix_len, q_len))
    qo_bytes = 2 * sum(q_len) * desc.q_dim * 2
    return flops, kv_bytes + qo_bytes


def run_config(cfg_index, args, weights_cache):
    """Round 1 of one workload configuration: set-up (untimed), W warm-up steps, K timed steps, then extra steps
    in which single kernel classes are bracketed by events.  Returns (result dict, state for the headline extras)."""
    import torch
    from paper_2602_12957_amd.runtime import Engine
    import paper_2602_12957_amd.binding as B
    import workloads as W

    seed = args.seed or W.SEED_BASE
    desc = W.CONFIGS[cfg_index].model
    specs = W.draw_sequences(cfg_index, seed)
    if "w" not in weights_cache:
        weights_cache["w"] = W.make_weights(desc, seed)
    weights = weights_cache["w"]
    mode = W.CONFIGS[cfg_index].kind        # "region" or "page": the entry point
    n = len(specs)
    k_max = max(sp.draft_len for sp in specs)
    # room for every sequence to grow by the longest draft: the untimed greedy generation advances all in lock step
    maxb = max((sp.n_visual + sp.n_prompt + k_max + 1 + 15) // 16 + 1 for sp in specs)
    n_blocks = sum((sp.n_visual + sp.n_prompt + k_max + 1 + 15) // 16 + 1 for sp in specs) + 8
    total_q = sum(sp.draft_len + 1 for sp in specs)
    prefix_len = [sp.n_visual + max(sp.n_prompt - 1, 0) for sp in specs]
    # workspace rows: one verification block, or (configs[1]) all prefixes at once for the prefill figure
    ws_rows = max(total_q, sum(prefix_len) if cfg_index == 1 else 8192)
    steps = args.steps if cfg_index in (1, args.profile_config) else max(3, min(args.steps, args.other_steps))
    debug = None
    if args.debug_knobs:       # experiments only: "name=value,..." with gemm_cfg=q:o:g:d:l
        debug = {}
        for item in args.debug_knobs.split(","):
            k, v = item.split("=")
            debug[k] = tuple(int(x) for x in v.split(":")) if k == "gemm_cfg" else int(v)
    # one long draft of one sequence (configs[2]) gives the attention launch 132 workgroups for 256 compute units:
    # that is the case the library's key split (hsd_model_desc.attn_key_chunk, fixed cut points) is there for
    key_chunk = args.attn_key_chunk if args.attn_key_chunk >= 0 else (1024 if cfg_index == 2 else 0)
    eng = Engine(desc, weights, n_blocks, n, maxb, ws_rows, max_dump=total_q if cfg_index == 1 else 0,
                 attn_key_chunk=key_chunk, debug=debug)
    slots = list(range(n))
    toks, embs, pend = [], [], []
    for sp in specs:
        t, e, p = prefix_inputs(W, desc, seed, sp)
        toks.append(t), embs.append(e), pend.append(p)

    # --- set-up (untimed): prefix prefill, greedy target generation on the GPU path itself, prefill again
    eng.prefill(slots, toks, embs)
    if args.random_target:
        target = np.random.default_rng(seed).integers(0, desc.vocab, size=(n, k_max)).astype(np.int32)
    else:
        target = eng.greedy_decode(slots, pend, k_max, mode)
        eng.reset()
        eng.prefill(slots, toks, embs)
    torch.cuda.synchronize()
    corrupt = W.corrupt_draft_forced if specs[0].forced_different else W.corrupt_draft
    drafts = [corrupt(target[i][:sp.draft_len], sp.corrupt_p, desc.vocab, seed, f"cfg{cfg_index}.{sp.seq_id}")[0]
              for i, sp in enumerate(specs)]
    blocks = [np.concatenate([[pend[i]], drafts[i]]).astype(np.int32) for i in range(n)]
    log_tau = 0.0 if args.tau >= 1.0 else float(np.log(args.tau))
    batch = eng.prepare(slots, blocks, log_tau=log_tau)
    eng.snapshot()
    torch.cuda.synchronize()

    def step():
        eng.restore()                       # bookkeeping back to "prefix cached" (one small device copy)
        eng.verify_prepared(batch, mode)
        eng.commit()
        return eng.read_acceptance(n)       # synchronises: the host needs alpha to slice the next round

    for _ in range(args.warmup):
        alpha, bonus, status = step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        alpha, bonus, status = step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    assert status == 0, f"device status {status}"

    verified = sum(sp.draft_len for sp in specs)
    accepted = int(alpha.sum())
    ms_step = dt / steps * 1e3
    d, F, V = desc.d_model, desc.d_ffn, desc.vocab
    qd, kvd = desc.q_dim, desc.kv_dim
    flops_per_launch = {"gate_up": 2.0 * total_q * d * 2 * F, "qkv": 2.0 * total_q * d * (qd + 2 * kvd),
                        "o": 2.0 * total_q * qd * d, "down": 2.0 * total_q * F * d, "lm_head": 2.0 * total_q * d * V}
    prof_map = {"gate_up": B.HSD_PROF_GEMM_GATE_UP, "qkv": B.HSD_PROF_GEMM_QKV, "attention": B.HSD_PROF_ATTENTION,
                "o": B.HSD_PROF_GEMM_O, "down": B.HSD_PROF_GEMM_DOWN, "lm_head": B.HSD_PROF_GEMM_LM_HEAD,
                "rmsnorm": B.HSD_PROF_RMSNORM}

    def time_kernel(name, n_steps=3):
        """Average launch duration of one kernel class over extra steps (HIP events on the launch stream, recorded
        by the library around each launch); never inside the timed region above."""
        eng.profile(prof_map[name], 3 * desc.n_layers * n_steps + 8)
        for _ in range(n_steps):
            step()
        cnt, ms = eng.profile_read()
        eng.profile(B.HSD_PROF_NONE, 0)
        return (ms / cnt, cnt) if cnt > 0 else (None, 0)

    att_flops, att_bytes = attention_work(desc, prefix_len, [sp.draft_len + 1 for sp in specs])

    def roofline_of(name):
        avg_ms, cnt = time_kernel(name)
        if avg_ms is None:
            return None
        if name == "attention":
            # binding roof of this launch: the larger of its time at the HBM peak and at the MFMA peak
            t_hbm, t_mfma = att_bytes / (PEAK_HBM_GBPS * 1e9), att_flops / (PEAK_BF16_TFLOPS * 1e12)
            if t_mfma >= t_hbm:
                ach = att_flops / (avg_ms * 1e-3) / 1e12
                r = {"kernel": "k_attn_mfma", "bound": "mfma", "achieved": round(ach, 1), "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(ach / PEAK_BF16_TFLOPS, 4)}
            else:
                ach = att_bytes / (avg_ms * 1e-3) / 1e9
                r = {"kernel": "k_attn_mfma", "bound": "hbm", "achieved": round(ach, 1), "peak": PEAK_HBM_GBPS,
                     "unit": "GB/s", "frac": round(ach / PEAK_HBM_GBPS, 4)}
            r.update({"traffic": None, "avg_launch_ms": round(avg_ms, 5), "launches_timed": cnt,
                      "flops_per_launch": att_flops, "bytes_per_launch": att_bytes,
                      "achieved_TFLOPs": round(att_flops / (avg_ms * 1e-3) / 1e12, 1),
                      "achieved_GBps": round(att_bytes / (avg_ms * 1e-3) / 1e9, 1)})
            return r
        ach = flops_per_launch[name] / (avg_ms * 1e-3) / 1e12
        return {"kernel": f"k_gemm_mfma ({name})", "bound": "mfma", "achieved": round(ach, 1),
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(ach / PEAK_BF16_TFLOPS, 4),
                "traffic": MEASURED_TRAFFIC_BYTES.get((cfg_index, name)), "avg_launch_ms": round(avg_ms, 5),
                "launches_timed": cnt, "flops_per_launch": flops_per_launch[name]}

    dominant = args.profile_kernel if (cfg_index == 1 and args.profile_kernel != "auto") else DOMINANT[cfg_index]
    gemm_flops_step = 2.0 * desc.gemm_params * total_q
    all_flops_step = gemm_flops_step + desc.n_layers * att_flops
    res = {
        "workload": WORKLOAD_TEXT[cfg_index] + (" (random drafts)" if args.random_target else ""),
        "attn_key_chunk": key_chunk,
        "entry_point": "hsd_verify_region_batch" if mode == "region" else "hsd_verify_page",
        "n_seq": n, "rows_per_step": total_q, "draft_tokens_per_step": verified, "steps": steps,
        "ms_per_step": round(ms_step, 4),
        "verified_tokens_per_s": round(verified / (ms_step * 1e-3), 1),
        "accepted_tokens_per_s": round(accepted / (ms_step * 1e-3), 1),
        "committed_tokens_per_s": round((accepted + n) / (ms_step * 1e-3), 1),
        "aal": round(accepted / n, 3),
        "gemm_tflops_whole_step": round(gemm_flops_step / (ms_step * 1e-3) / 1e12, 1),
        "whole_step_frac_of_mfma_peak": round(all_flops_step / (ms_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
        "roofline": roofline_of(dominant) if dominant != "none" else None,
    }
    if dominant != "attention" and dominant != "none":
        att = roofline_of("attention")
        res["attention"] = att
    if args.breakdown:
        bd = {}
        for name in prof_map:
            avg_ms, cnt = time_kernel(name)
            if avg_ms is not None:
                bd[name] = {"launches_per_step": cnt // 3, "avg_us": round(avg_ms * 1e3, 2),
                            "us_per_step": round(avg_ms * cnt / 3 * 1e3, 1)}
        res["breakdown"] = bd
    state = dict(eng=eng, step=step, specs=specs, drafts=drafts, pend=pend, target=target, toks=toks, embs=embs,
                 slots=slots, total_q=total_q, log_tau=log_tau, desc=desc, weights=weights, seed=seed, W=W, n=n)
    return res, state


def headline_extras(out, st, args):
    """Figures beside the headline, all on configs[1] and all outside its timed region."""
    import torch
    eng, specs, drafts, pend, target = st["eng"], st["specs"], st["drafts"], st["pend"], st["target"]
    slots, n, log_tau, desc, seed, total_q = st["slots"], st["n"], st["log_tau"], st["desc"], st["seed"], st["total_q"]
    if args.calibration_copy_mb > 0:
        src = torch.ones(args.calibration_copy_mb * (1 << 20) // 4, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if args.random_target:
        return
    # --- the same workload to completion: verify -> commit -> read (alpha, bonus) -> slice the next blocks on the
    # host -> upload them, until every draft is consumed (not part of `value`)

    def to_completion():
        eng.restore()
        pending, offset = list(pend), [0] * n
        rounds = rows = acc = 0
        while True:
            active = [i for i in range(n) if offset[i] < len(drafts[i])]
            if not active:
                break
            blks = [np.concatenate([[pending[i]], drafts[i][offset[i]:]]).astype(np.int32) for i in active]
            eng.verify(active, blks, "region", log_tau=log_tau)
            eng.commit()
            a, b, st_ = eng.read_acceptance(len(active))
            assert st_ == 0
            for j, i in enumerate(active):
                rows += len(blks[j]) - 1
                acc += int(a[j])
                offset[i] += int(a[j]) + 1
                pending[i] = int(b[j])
            rounds += 1
        return rounds, rows, acc
    to_completion()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    rounds, rows, acc = to_completion()
    torch.cuda.synchronize()
    dtc = time.perf_counter() - t0
    out["to_completion"] = {"rounds": rounds, "ms_total": round(dtc * 1e3, 3), "draft_rows_scored": rows,
                            "accepted_tokens": acc, "verified_tokens_per_s": round(rows / dtc, 1),
                            "committed_tokens_per_s": round(sum(len(d_) for d_ in drafts) / dtc, 1),
                            "note": "includes host slicing and the upload of each round's batch"}
    # --- the same model decoding the same sequences one token per pass (Lq = 1 for every region): the
    # autoregressive baseline of the paper's decode-time speedup ratio (Section 4.2), on this GPU and this library
    eng.restore()
    n_ar = 32
    eng.greedy_decode(slots, pend, 4)
    eng.restore()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    eng.greedy_decode(slots, pend, n_ar)
    torch.cuda.synchronize()
    dar = time.perf_counter() - t0
    ar_rate = n * n_ar / dar
    weight_bytes = 2.0 * desc.gemm_params
    out["ar_decode_baseline"] = {
        "tokens_per_s": round(ar_rate, 1), "ms_per_token_step": round(dar / n_ar * 1e3, 4), "steps_timed": n_ar,
        "batch": n, "weight_stream_frac_of_hbm_peak": round(weight_bytes / (dar / n_ar) / (PEAK_HBM_GBPS * 1e9), 4),
        "speedup_to_completion": round(out["to_completion"]["committed_tokens_per_s"] / ar_rate, 2),
        "note": "same library, one token per sequence and pass; a pass over 16 rows is bound by per-launch latency, "
                "not by streaming the weights, so the ratio flatters verification (see weight_stream_frac_of_hbm_peak)"}
    # --- relaxed acceptance (paper Section 3.2, Eq. 11; operating point tau = 0.75, Section 4.1) on near-miss drafts:
    # the greedy target with 15 % of its tokens replaced by the model's own second choice at that position
    eng.restore()
    tblocks = [np.concatenate([[pend[i]], target[i][:sp.draft_len]]).astype(np.int32) for i, sp in enumerate(specs)]
    o = eng.verify(slots, tblocks, "region", dump_rows=np.arange(total_q))
    logits = o.logits.cpu().numpy()                       # the library's logit dump; the ranking is host work
    second = np.argpartition(-logits, 1, axis=1)[:, :2]
    second = np.where(second[:, 0] == logits.argmax(axis=1), second[:, 1], second[:, 0])
    del logits
    rng = np.random.default_rng(seed + 1)
    nm_blocks = []
    for i, sp in enumerate(specs):
        lo = int(o.cu_q[i])
        d = target[i][:sp.draft_len].copy()
        hit = rng.random(sp.draft_len) < 0.15
        d[hit] = second[lo:lo + sp.draft_len][hit]
        nm_blocks.append(np.concatenate([[pend[i]], d]).astype(np.int32))
    curve = {}
    for tau in (1.0, 0.9, 0.75, 0.5, 0.25):
        eng.restore()
        eng.verify(slots, nm_blocks, "region", log_tau=0.0 if tau >= 1.0 else float(np.log(tau)))
        a, _, st_ = eng.read_acceptance(n)
        assert st_ == 0
        curve[str(tau)] = round(float(a.mean()), 3)
    out["aal_vs_tau_near_miss"] = curve
    eng.restore()
    # --- prefix prefill of the same 16 regions (excluded from the decode metric, reported for the end-to-end
    # picture): with the visual embedding rows already on the device, as a vision encoder leaves them, and with
    # their upload from pageable host memory
    toks, embs = st["toks"], st["embs"]
    n_prefill = sum(len(t) for t in toks)
    dev_embs = [torch.from_numpy(e).to("cuda:0") for e in embs]
    pf = {}
    for key, src in (("ms", dev_embs), ("ms_with_upload", embs)):
        eng.reset()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        eng.prefill(slots, toks, src)
        torch.cuda.synchronize()
        pf[key] = time.perf_counter() - t0
    flops_pf = 2.0 * (desc.gemm_params - desc.d_model * desc.vocab) * n_prefill
    out["prefill"] = {"rows": n_prefill, "ms": round(pf["ms"] * 1e3, 3),
                      "rows_per_s": round(n_prefill / pf["ms"], 1),
                      "gemm_frac_of_mfma_peak": round(flops_pf / pf["ms"] / 1e12 / PEAK_BF16_TFLOPS, 4),
                      "ms_with_upload": round(pf["ms_with_upload"] * 1e3, 3),
                      "note": "visual embedding rows resident on the device; ms_with_upload adds their copy from "
                              "host memory"}
    del dev_embs


def hw_probe(yardstick: bool):
    """What this chip sustains, measured with the library's probe kernels (hsd_probe_launch): the matrix pipes with
    every compute unit busy and with a few, a compute unit's load path from L2, its LDS.  With `yardstick` also the
    vendor library's plain bf16 GEMM (torch.matmul) on the projection shapes of configurations 1 and 3, operands
    rotated through copies so that they come from HBM as they do inside a pass."""
    import torch
    from paper_2602_12957_amd import binding as B
    dev = torch.device("cuda:0")
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    scratch = torch.zeros(16 << 20, dtype=torch.uint8, device=dev)      # 8 regions of 2 MiB: L2 resident
    stream = torch.cuda.current_stream().cuda_stream

    def timed(kind, n_wg, iters, arg=0):
        B.hsd_probe_launch(stream, kind, n_wg, max(1, iters // 50), arg, scratch.data_ptr(), scratch.numel())
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        B.hsd_probe_launch(stream, kind, n_wg, iters, arg, scratch.data_ptr(), scratch.numel())
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3

    out = {"probe": "hardware", "compute_units": n_cu, "peak_bf16_tflops_datasheet": PEAK_BF16_TFLOPS}
    mf = {}
    for n_wg in (8, n_cu // 4, n_cu):
        iters = 20000
        dt = timed(B.HSD_PROBE_MFMA, n_wg, iters)
        ns = dt * 1e9 / (iters * 16)                   # per MFMA and SIMD (one wave per SIMD)
        mf[str(n_wg)] = {"tflops": round(n_wg * 4 * iters * 16 * 32768 / dt / 1e12, 1), "ns_per_mfma": round(ns, 2),
                         "clock_ghz_at_32_cycles": round(32 / ns, 3)}
    out["mfma_32x32x16_bf16_by_busy_units"] = mf
    ld = {}
    for name, kind in (("to_registers", B.HSD_PROBE_LOAD_REG), ("to_lds", B.HSD_PROBE_LOAD_LDS)):
        iters = 2000
        dt = timed(kind, n_cu, iters)
        ld[name] = {"bytes_per_ns_per_cu": round(iters * 32768 / (dt * 1e9), 1),
                    "tb_per_s_chip": round(n_cu * iters * 32768 / dt / 1e12, 2)}
    out["load_path_from_l2"] = ld
    lds = {}
    for waves in (4, 8, 16):
        iters = 4000
        dt = timed(B.HSD_PROBE_LDS_READ, n_cu, iters, waves)
        lds[str(waves)] = round(iters * 8192 * waves / (dt * 1e9), 1)
    out["lds_read_b128_bytes_per_ns_per_cu_by_waves"] = lds
    if yardstick:
        ys = {}
        shapes = [("cfg1 gate/up", 1856, 8192, 1024), ("cfg1 down", 1856, 1024, 4096), ("cfg1 qkv", 1856, 1536, 1024),
                  ("cfg1 o", 1856, 1024, 1024), ("cfg1 lm_head", 1856, 32768, 1024), ("cfg3 gate/up", 32772, 8192, 1024),
                  ("cfg3 down", 32772, 1024, 4096), ("cfg3 lm_head", 32772, 32768, 1024), ("square 8192", 8192, 8192, 8192)]
        for name, M, N, K in shapes:
            nb = max(1, min(16, int(600e6 // ((M * K + N * K) * 2))))
            A = [torch.randn(M, K, device=dev, dtype=torch.bfloat16) for _ in range(nb)]
            Wt = [torch.randn(N, K, device=dev, dtype=torch.bfloat16) for _ in range(nb)]
            o = torch.empty(M, N, device=dev, dtype=torch.bfloat16)
            for i in range(3):
                torch.matmul(A[i % nb], Wt[i % nb].t(), out=o)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(20):
                torch.matmul(A[i % nb], Wt[i % nb].t(), out=o)
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / 20
            ys[name] = {"M": M, "N": N, "K": K, "us": round(us, 1), "tflops": round(2.0 * M * N * K / us * 1e-6, 0)}
            del A, Wt, o
        out["vendor_gemm_yardstick"] = ys
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--seed", type=int, default=None)
    ap.add_argument("--cpu-sample", type=int, default=16, help="sequences of the workload the oracle is timed on (0 = skip)")
    ap.add_argument("--profile-kernel", type=str, default="auto",
                    choices=["auto", "gate_up", "qkv", "attention", "o", "down", "lm_head", "rmsnorm", "none"],
                    help="kernel class of the headline's roofline object (auto: the gate/up GEMM)")
    ap.add_argument("--configs", type=str, default="1,2,3,4",
                    help="workload configurations to time; 1 is the headline and always runs")
    ap.add_argument("--other-steps", type=int, default=5, help="timed steps of configs 2-4 (at most --steps)")
    ap.add_argument("--random-target", action="store_true",
                    help="profiling aid: skip the greedy target generation and corrupt a random token sequence instead "
                         "(same shapes and kernels; acceptance lengths are then meaningless)")
    ap.add_argument("--calibration-copy-mb", type=int, default=0,
                    help="profiling aid: after the timed region run one plain device-to-device copy of this many MiB "
                         "(a kernel of known traffic against which HBM counters are scaled)")
    ap.add_argument("--tau", type=float, default=1.0,
                    help="acceptance threshold of the relaxed rule (paper default 0.75); 1.0 = exact greedy match, "
                         "the rule the headline metric is defined on")
    ap.add_argument("--attn-key-chunk", type=int, default=-1,
                    help="attention key split (hsd_model_desc.attn_key_chunk): keys per chunk, 0 = unsplit; "
                         "default: 1024 for configs[2] (one long draft of one sequence), unsplit elsewhere")
    ap.add_argument("--profile-config", type=int, default=0, choices=[0, 1, 2, 3, 4],
                    help="profiling aid: run round 1 of this one configuration only (set-up, warm-up, timed steps, "
                         "per-kernel extra steps) and print its result object instead of the headline line")
    ap.add_argument("--debug-knobs", type=str, default="",
                    help="experiments only: hsd_debug_set knobs, e.g. sync_layers=1,gemm_cfg=7:9:8:9:8")
    ap.add_argument("--breakdown", action="store_true",
                    help="after the timed region, time every kernel class in turn (extra steps) and report avg us per launch")
    ap.add_argument("--hw-probe", action="store_true",
                    help="instead of the benchmark: run the library's hardware probes (sustained MFMA rate, load path, "
                         "LDS) and print their JSON line")
    ap.add_argument("--yardstick", action="store_true",
                    help="with --hw-probe: also time the vendor library's plain GEMM on the projection shapes")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    if args.hw_probe:
        hw_probe(args.yardstick)
        return
    others = [int(c) for c in args.configs.split(",") if c.strip() and int(c) != 1]
    weights_cache = {}
    if args.profile_config:
        res, st = run_config(args.profile_config, args, weights_cache)
        if args.calibration_copy_mb > 0:
            headline_extras({}, dict(st, eng=st["eng"]), argparse.Namespace(**dict(vars(args), random_target=True)))
        st["eng"].close()
        print(json.dumps(res))
        return
    res1, st = run_config(1, args, weights_cache)
    out = {
        "metric": "verified_draft_tokens_per_s", "value": res1["verified_tokens_per_s"], "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": res1["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": res1["workload"], "n_seq": res1["n_seq"], "rows_per_step": res1["rows_per_step"],
                   "draft_tokens_per_step": res1["draft_tokens_per_step"], "corruption_p": 0.05,
                   "acceptance": "exact match (tau = 1)" if args.tau >= 1.0 else f"relaxed, tau = {args.tau}"},
        "accepted_tokens_per_s": res1["accepted_tokens_per_s"],
        "committed_tokens_per_s": res1["committed_tokens_per_s"],
        "aal": res1["aal"],
        "gemm_tflops_whole_step": res1["gemm_tflops_whole_step"],
        "whole_step_frac_of_mfma_peak": res1["whole_step_frac_of_mfma_peak"],
        "roofline": res1["roofline"],
        "attention": res1.get("attention"),
    }
    if "breakdown" in res1:
        out["breakdown"] = res1["breakdown"]
    headline_extras(out, st, args)
    if args.cpu_sample > 0:
        out["cpu_baseline"] = cpu_baseline(st["W"], st["desc"], st["weights"], st["seed"], st["specs"], st["drafts"],
                                           st["pend"], min(args.cpu_sample, st["n"]))
    st["eng"].close()
    del st
    torch.cuda.empty_cache()
    out["configs"] = {}
    for c in others:
        if c not in (2, 3, 4):
            continue
        res, st_c = run_config(c, args, weights_cache)
        st_c["eng"].close()
        del st_c
        torch.cuda.empty_cache()
        out["configs"][str(c)] = res
    print(json.dumps(out))


if __name__ == "__main__":
    main()
