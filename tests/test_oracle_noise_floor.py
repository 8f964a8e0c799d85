"""Why the floating-point bars of deep bf16 models are derived rather than taken as stated.

Two evaluations of the SAME 24-layer decoder, both storing activations in bf16 at the same points, that differ
only in the precision in which sums are formed (fp64 vs fp32), are compared.  Oracle code only, CPU only.  Their
logits deviate by far more than the stated bf16 bar (max-abs 2e-2), and arg-max decisions flip at margins above
1e-2: a rounding that falls on the other side of a bf16 boundary in an early layer is amplified by the layers
above it.  No implementation (this repository's HIP path included) can agree with the oracle more closely than two
instances of the oracle agree with each other; the GPU parity tests therefore scale their bars with this floor.
"""
import numpy as np

import oracle as O
import workloads as W


def test_bf16_storage_noise_floor_of_model_m():
    desc, seed = W.MODEL_M, W.SEED_BASE
    w = W.make_weights(desc, seed)
    vis, _ = W.make_prefix(desc, seed, 0, 48, 0)
    draft = np.random.default_rng(5).integers(0, desc.vocab, size=15)
    logits = []
    for dt in (np.float64, np.float32):
        cache, pending = O.prefill(desc, w, vis, [], dt, act_dtype="bf16")
        logits.append(O.verify_block(desc, w, cache, pending, draft, dt, act_dtype="bf16")[3].astype(np.float64))
    d = logits[0] - logits[1]
    rms, mx = float(np.sqrt((d ** 2).mean())), float(np.abs(d).max())
    flips = int((logits[0].argmax(-1) != logits[1].argmax(-1)).sum())
    print(f"noise floor: rms {rms:.4f} max {mx:.4f} arg-max flips {flips}/16")
    assert 3e-3 < rms < 3e-2          # about 1e-2: comparable to the stated max-abs bar itself
    assert mx > 2e-2                  # the stated bar is below what two oracle instances achieve
    # without bf16 storage the same two evaluations agree to fp32 accuracy
    a = O.verify_block(desc, w, O.prefill(desc, w, vis, [], np.float64)[0], 0, draft, np.float64)[3]
    b = O.verify_block(desc, w, O.prefill(desc, w, vis, [], np.float32)[0], 0, draft, np.float32)[3]
    assert np.abs(a - b).max() < 1e-4


def test_storage_noise_that_scales_the_gpu_bars():
    """The GPU parity bars of model M are multiples of sigma = RMS deviation between the plain fp64 oracle and the same
    oracle with activations stored in bf16 (what any bf16 implementation must do).  Oracle code only: sigma is about
    1.3e-2 on a fresh sample, and the value each golden file records (measured on its own sample by the script that
    wrote it) lies in the same range -- so the bars are tied to a property of the model, not to the HIP path."""
    import gzip
    import json
    import os
    desc, seed = W.MODEL_M, W.SEED_BASE
    w = W.make_weights(desc, seed)
    vis, _ = W.make_prefix(desc, seed, 1, 40, 0)
    draft = np.random.default_rng(11).integers(0, desc.vocab, size=23)
    cache, pending = O.prefill(desc, w, vis, [], np.float64)
    plain = O.verify_block(desc, w, cache, pending, draft, np.float64)[3]
    cache_r, pending_r = O.prefill(desc, w, vis, [], np.float64, act_dtype="bf16")
    assert pending_r == pending
    rounded = O.verify_block(desc, w, cache_r, pending_r, draft, np.float64, act_dtype="bf16")[3]
    d = np.asarray(plain, np.float64) - np.asarray(rounded, np.float64)
    sigma = float(np.sqrt((d ** 2).mean()))
    print(f"storage noise: rms {sigma:.4f} max {np.abs(d).max():.4f}")
    assert 7e-3 < sigma < 2.5e-2
    assert np.abs(d).max() < 8 * sigma            # the tail the 6-sigma max-abs bar of the GPU tests leans on
    here = os.path.join(os.path.dirname(__file__), "golden")
    for cfg in (1, 2, 3, 4):
        with gzip.open(os.path.join(here, f"cfg{cfg}.json.gz"), "rt") as f:
            g = json.load(f)
        assert g["oracle_act_dtype"] in (None, "none", "plain"), g["oracle_act_dtype"]
        assert 0.6 * sigma < g["storage_noise"]["rms"] < 1.6 * sigma, (cfg, g["storage_noise"], sigma)
