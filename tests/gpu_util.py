"""Shared helpers of the GPU parity tests: tolerances and host<->device conversion."""
import numpy as np
import torch

from workloads.synth import bf16_bits_to_f32, bf16_round_bits

DEV = "cuda:0"
TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}


def rand_values(rng, shape, dtype, sigma=1.0):
    """float32 array whose entries are exactly representable in `dtype`."""
    x = (rng.standard_normal(shape) * sigma).astype(np.float32)
    if dtype == "bf16":
        x = bf16_bits_to_f32(bf16_round_bits(x))
    return x


def to_dev(x: np.ndarray, dtype: str) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(x)).to(DEV).to(TORCH_DTYPE[dtype])


def to_np64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def assert_attention_close(got: np.ndarray, want: np.ndarray, dtype: str, what: str = ""):
    """fp32 inputs: max-abs 1e-4.  bf16 inputs (fp32 accumulation, output rounded to bf16):
    max-relative 2e-2 with the denominator floored at 1e-2 of the row's largest magnitude."""
    got = np.asarray(got, np.float64); want = np.asarray(want, np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    assert np.all(np.isfinite(got)), what
    if dtype == "f32":
        err = np.abs(got - want).max() if got.size else 0.0
        assert err <= 1e-4, f"{what}: max abs err {err:.3e} > 1e-4"
    else:
        floor = 1e-2 * np.abs(want).max(axis=-1, keepdims=True)
        rel = np.abs(got - want) / np.maximum(np.abs(want), floor)
        err = rel.max() if rel.size else 0.0
        assert err <= 2e-2, f"{what}: max rel err {err:.3e} > 2e-2"


def assert_mass_close(got: np.ndarray, want: np.ndarray, what: str = ""):
    """Mass is float32 arithmetic on exactly represented inputs for either element type:
    relative 5e-5 of the entry, floored at 1e-7 of the row's largest entry."""
    got = np.asarray(got, np.float64); want = np.asarray(want, np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    if want.size == 0:
        return
    floor = 1e-7 * np.abs(want).max()
    rel = np.abs(got - want) / np.maximum(np.abs(want), floor)
    assert rel.max() <= 5e-5, f"{what}: mass max rel err {rel.max():.3e}"


def assert_selection_matches(got_ids, oracle_scores, oracle_ids, k, what=""):
    """Kept set must equal the oracle's top-k by (score desc, id asc), except that members of the
    symmetric difference may be tokens whose oracle score is within 1e-5 relative of the k-th."""
    from oracle import st3_oracle as orc
    got = set(int(x) for x in got_ids)
    assert len(got) == k, f"{what}: kept {len(got)} != {k}"
    pos = orc.select_topk(oracle_scores, oracle_ids, k)
    want = set(int(oracle_ids[p]) for p in pos)
    if got == want:
        return True
    order = orc.ranked_order(oracle_scores, oracle_ids)
    kth = float(oracle_scores[order[k - 1]])
    score_of = {int(i): float(s) for i, s in zip(oracle_ids, oracle_scores)}
    for tok in got ^ want:
        assert abs(score_of[tok] - kth) <= 1e-5 * abs(kth), \
            f"{what}: token {tok} score {score_of[tok]} vs k-th {kth} differs beyond the near-tie rule"
    return False
