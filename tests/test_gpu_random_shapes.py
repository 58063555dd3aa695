"""GPU parity on random shapes: fit+score, the unit features and apply-plan against the oracle, and the
fused features + fit+score call against the separate calls, bit for bit.  Seeded: the same cases
every run.  Rows 1..600 (units of 1..600 rows), chunks of 8..256 columns, 1..64 clip ratios, both
element types, activation scales with outliers."""
import random

import pytest
import torch

from paper_2605_26660_amd import synth
from test_gpu_parity import DEV, REL, assert_close, check_apply, check_features, check_fit_score, grid, to_np

pytestmark = pytest.mark.gpu


def same_bits(a, b):
    return torch.equal(a.contiguous().view(torch.uint8), b.contiguous().view(torch.uint8))


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_random_shapes(windq, seed):
    rng = random.Random(seed)
    for it in range(80):
        G = rng.choice([8, 16, 24, 32, 40, 64, 96, 128, 256])
        C = G * rng.randint(1, 5)
        R_u = rng.choice([1, 3, 17, 64, 65, 100, 128, 130, 200])
        nrb = rng.randint(1, 3)
        R = R_u * nrb
        unit_rows = rng.choice([0, R_u])
        if unit_rows == 0:
            R_u = R
        K = rng.choice([1, 2, 5, 6, 11, 20, 21, 40, 64])
        dtype = rng.choice([torch.bfloat16, torch.float32])
        what = f"seed {seed} case {it}: R={R} C={C} G={G} unit_rows={unit_rows} K={K} {dtype}"
        W = synth.weights_llm(R, C, seed=1000 * seed + it, device=DEV).to(dtype)
        X = synth.activations_llm(64, C, seed=5000 * seed + it, device=DEV)
        s, _ = windq.windq_calib_stats(X)
        try:
            if R_u >= 3:
                err, idx, ref = check_fit_score(windq, W, s, G, unit_rows, K)
            else:
                # a "unit" of one or two short rows: under an activation outlier a single weight carries
                # its whole error, and a single weight's residual is only good to ~1e-7 of the group's range
                # (see windq_fit_score_all_bits): gross mistakes only
                cg = grid(K)
                err, idx, ref = windq.windq_fit_score_all_bits(W, s, G, unit_rows, cg)
                torch.cuda.synchronize()
                from oracle import windq_oracle as O
                o_err, _, o_ref, _ = O.fit_score_all_bits(to_np(W), to_np(s), G, unit_rows, cg.numpy())
                assert_close(to_np(err), o_err, rel=50 * REL, what="err (few-row units)")
                assert_close(to_np(ref), o_ref, what="ref_energy")
            check_features(windq, W, s, G, unit_rows)
            f2, e2, i2, r2 = windq.windq_features_fit_score(W, s, G, unit_rows, grid(K))
            f1 = windq.windq_unit_features(W, s, G, unit_rows)
            torch.cuda.synchronize()
            assert same_bits(e2, err) and same_bits(i2, idx) and same_bits(r2, ref) and same_bits(f1, f2), "fused != separate"
            action = torch.tensor([rng.randint(0, 6) for _ in range(err.shape[0])], dtype=torch.uint8)
            check_apply(windq, W, G, unit_rows, action, idx, K)
        except AssertionError as e:
            raise AssertionError(f"{what}: {e}") from e


@pytest.mark.parametrize("seed", [11, 12])
def test_random_shapes_after_the_hot_path(windq, seed):
    """Protection (select, encode, masked fit+score and apply-plan), refinement, dequantisation and the
    product from the artefact, each against the oracle as in its own test file, on random shapes."""
    import test_gpu_dequant as DQ
    import test_gpu_refine as RF
    import test_gpu_salient as S
    rng = random.Random(seed)
    for it in range(60):
        G = rng.choice([8, 16, 24, 32, 40, 64, 96, 128, 256])
        C = G * rng.randint(1, 4)
        R_u = rng.choice([4, 17, 64, 65, 100, 128, 130])
        nrb = rng.randint(1, 3)
        R = R_u * nrb
        unit_rows = rng.choice([0, R_u])
        K = rng.choice([1, 5, 6, 20])
        ppm = rng.choice([0, 30000, 100000, 300000])
        n_iter = rng.choice([0, 1, 3])
        dtype = rng.choice([torch.bfloat16, torch.float32])
        what = f"seed {seed} case {it}: R={R} C={C} G={G} unit_rows={unit_rows} K={K} ppm={ppm} n_iter={n_iter} {dtype}"
        W = synth.weights_llm(R, C, seed=3000 * seed + it, device=DEV).to(dtype)
        X = synth.activations_llm(64, C, seed=7000 * seed + it, device=DEV)
        s, _ = windq.windq_calib_stats(X)
        try:
            if ppm:
                mask, keep = S.check_select(windq, W, s, G, unit_rows, ppm)
                S.check_encode(windq, W, s, G, unit_rows, ppm, mask, keep)
                S.check_masked_fit_and_apply(windq, W, s, G, unit_rows, ppm, K)
            RF.run_case(windq, W, s, G, unit_rows, K, n_iter, ppm)
            DQ.run_case(windq, W, s, G, unit_rows, K, ppm)
            DQ.gemv_case(windq, W, s, G, unit_rows, K, ppm)
        except AssertionError as e:
            raise AssertionError(f"{what}: {e}") from e
