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
