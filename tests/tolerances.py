"""The comparison rules of the GPU parity tests, in plain numpy so that the CPU suite can
check what they reject (tests/test_tolerance_power.py plants mistakes in oracle results and
expects every rule below to fire).

Attention outputs (bf16 inputs, probabilities rounded to bf16 before the PV product, fp32
accumulation, bf16 output):
  * element rule   |gpu - ref| <= 2e-2 + 1e-2 |ref|
  * row rules      ||gpu - ref||_2 <= 2e-2 ||ref||_2  and  max |gpu - ref| <= 5e-2 rms(ref)
    The element rule alone has no power at long context: with i.i.d. N(0,1) values and a
    diffuse softmax over n keys the output itself is about 1/sqrt(n), below 2e-2 from some
    20,000 keys on.  The row rules scale with the row, whatever its size; bf16 rounding of
    the probabilities and of the output predicts a relative row error of about 4e-3.
  * lse            |gpu - ref| <= 2e-5 + 2e-5 |ref|   (fp32 exp2 / log2 / row sums)
  * structured values (v_block_classes): V[j][d] = 1 iff floor(j / 64) mod D = d, so
    out[i][d] is the probability mass of the key blocks of class d: every element is a sum
    of non-negative terms, its only errors are the bf16 roundings (relative 2^-9 each), and a
    dropped or doubled 64-key tile moves one element by the tile's share of its class.
    Rule: |gpu - ref| <= 6e-3 |ref| + 1e-6.
"""
import numpy as np

ATOL, RTOL = 2e-2, 1e-2
ROW_REL_L2 = 2e-2
ROW_MAX_OVER_RMS = 5e-2
LSE_ATOL, LSE_RTOL = 2e-5, 2e-5
CLASS_RTOL, CLASS_ATOL = 6e-3, 1e-6


def check_rows(got, ref, what=""):
    """got, ref: [..., D] fp64 (any leading shape, one attention row per leading index)."""
    got = np.asarray(got, np.float64); ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, f"{what}: shape {got.shape} vs {ref.shape}"
    err = np.abs(got - ref)
    bad = err > ATOL + RTOL * np.abs(ref)
    assert not bad.any(), (f"{what}: {bad.sum()} of {bad.size} outputs off, max err {err.max():.4g} at "
                           f"{np.unravel_index(err.argmax(), err.shape)}")
    d = ref.shape[-1]
    e2 = np.sqrt((err ** 2).sum(-1)); r2 = np.sqrt((ref ** 2).sum(-1))
    rel = np.where(r2 > 0, e2 / np.where(r2 > 0, r2, 1.0), np.where(e2 > 0, np.inf, 0.0))
    assert (rel <= ROW_REL_L2).all(), (f"{what}: row error {rel.max():.4g} of the row's norm at "
                                        f"{np.unravel_index(rel.argmax(), rel.shape)} (bound {ROW_REL_L2})")
    rms = r2 / np.sqrt(d)
    worst = err.max(-1)
    over = worst > ROW_MAX_OVER_RMS * rms
    assert not over.any(), (f"{what}: {over.sum()} rows with an element off by more than "
                            f"{ROW_MAX_OVER_RMS} of the row's rms (worst ratio "
                            f"{(worst / np.where(rms > 0, rms, 1e-300)).max():.4g})")


def check_lse(got, ref, what=""):
    got = np.asarray(got, np.float64); ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, f"{what}: lse shape {got.shape} vs {ref.shape}"
    assert np.array_equal(np.isneginf(got), np.isneginf(ref)), f"{what}: -inf pattern of lse differs"
    fin = np.isfinite(ref)
    if fin.any():
        err = np.abs(got[fin] - ref[fin])
        bad = err > LSE_ATOL + LSE_RTOL * np.abs(ref[fin])
        assert not bad.any(), f"{what}: lse off in {bad.sum()} rows, max err {err.max():.4g}"


def check_class_mass(got, ref, what=""):
    """Outputs computed with v_block_classes values."""
    got = np.asarray(got, np.float64); ref = np.asarray(ref, np.float64)
    err = np.abs(got - ref)
    bad = err > CLASS_ATOL + CLASS_RTOL * np.abs(ref)
    assert not bad.any(), (f"{what}: {bad.sum()} of {bad.size} block-class masses off, worst relative error "
                           f"{(err / np.maximum(np.abs(ref), 1e-300))[bad].max():.4g}")


def v_block_classes(n_tokens, n_kv_heads, d, block=64):
    """bf16 bit patterns (uint16) [n_tokens][Hkv][D]: 1.0 where floor(j / block) mod D == d, else 0."""
    cls = (np.arange(n_tokens) // block) % d
    v = np.zeros((n_tokens, n_kv_heads, d), np.uint16)
    v[np.arange(n_tokens), :, cls] = 0x3F80  # bf16 1.0
    return v
