"""How much of the tolerance (max |err| <= 2e-2 x per-head RMS of the oracle) the prescribed
arithmetic itself uses -- bf16 operands, exact sums, one bf16 rounding of the output
(tests/arith_model.py) -- on the kinds of inputs the GPU parity tests draw.  No GPU.

Two results.  (1) A seed sweep per width: the best possible bf16 pipeline already sits at
1.3e-2 - 2.2e-2 x RMS, so for some seeds NO implementation can meet the bar; the fraction that
can is reported.  (2) For every GPU parity test that draws generic inputs at a narrow width,
the exact seeded inputs it uses are shown to be feasible (model error below the bar with a
margin), so those tests keep their outlier channels and narrow nothing.
"""
import numpy as np
import pytest

import arith_model as am
import gpu_harness as gh

TOL = gh.TOL
KW = dict(eps=float(np.float32(1e-5)), theta=10000.0)


def sweep(d_model, n_kv, hd, n_tok, outliers, seeds=32):
    out = []
    for seed in range(seeds):
        c = gh.LayerCase(np.random.default_rng([4242, seed, d_model]), d_model, n_kv, hd, n_tok, outliers=outliers)
        out.append(am.worst_ratio(c.x, c.gamma, c.wkv, np.arange(n_tok), n_kv_heads=n_kv, head_dim=hd, **KW))
    return np.array(out)


@pytest.mark.parametrize("d_model,n_kv,hd,n_tok", [(256, 4, 64, 128), (512, 2, 128, 650),
                                                   (1024, 2, 128, 650), (2048, 2, 128, 255)])
def test_pass_fraction_of_the_prescribed_arithmetic(d_model, n_kv, hd, n_tok):
    """32 seeds per width the GPU tests use, with and without the x20 outlier channels."""
    for outliers in (True, False):
        r = sweep(d_model, n_kv, hd, n_tok, outliers)
        frac = float(np.mean(r <= TOL))
        print(f"d_model {d_model} outliers {outliers}: {frac:.3f} of 32 seeds within {TOL}; "
              f"model error min {r.min():.4f} median {np.median(r):.4f} max {r.max():.4f} x RMS_head")
        # the output rounding alone costs up to 2^-8 |y| with |y| up to ~5 RMS: never far below
        # the bar, never absurdly above it
        assert r.min() >= 0.9e-2 and r.max() <= 3.2e-2
        assert frac >= 0.5


def test_output_rounding_dominates():
    """With exact operands (no folded-gain rounding) the output rounding alone is most of it."""
    c = gh.LayerCase(np.random.default_rng([4242, 7]), 1024, 2, 128, 650)
    k, v = am.oracle.project_kv(c.x, c.gamma, c.wkv, KW["eps"], 2, 128)
    only_out = float(am.error_ratio(v, am.round_bf16(v)).max())
    both = am.worst_ratio(c.x, c.gamma, c.wkv, np.arange(650), n_kv_heads=2, head_dim=128, **KW)
    assert 1.0e-2 <= only_out <= both + 1e-3 <= 3.2e-2


MARGIN = 0.975            # feasible = model error <= 1.95e-2: room for fp32 accumulation


def feasible(x, gamma, wkv, pos, n_kv, hd, theta=10000.0, style=0):
    r = am.worst_ratio(x, gamma, wkv, pos, eps=KW["eps"], theta=float(np.float32(theta)),
                       n_kv_heads=n_kv, head_dim=hd, rope_style=style)
    return r


def test_inputs_of_the_mixed_restore_test_are_feasible():
    import test_gpu_mixed as t
    m = t.MIXED_SHAPE
    pos = m["pos_offset"] + m["tok_begin"] + np.arange(m["n_tok"])
    for l, c in enumerate(t.mixed_cases()):
        r = feasible(c.x[m["tok_begin"]:m["tok_begin"] + m["n_tok"]], c.gamma, c.wkv, pos, m["n_kv"], m["hd"])
        print(f"mixed restore layer {l}: model error {r:.4f} x RMS_head")
        assert r <= MARGIN * TOL


def test_inputs_of_the_several_contexts_test_are_feasible():
    import test_gpu_parity as t
    cases = t.several_contexts_cases()
    lengths = t.SEVERAL_LENGTHS
    pos = np.concatenate([np.arange(n) for n in lengths])
    for l in range(len(cases[0])):
        x = np.concatenate([cases[i][l].x[:lengths[i]] for i in range(len(lengths))])
        r = feasible(x, cases[0][l].gamma, cases[0][l].wkv, pos, 2, 128)
        print(f"several contexts layer {l}: model error {r:.4f} x RMS_head")
        assert r <= MARGIN * TOL


def test_inputs_of_the_shape_tests_are_feasible():
    import test_gpu_parity as t
    for d_model, n_kv, hd, n_tok, style in t.SHAPES:
        case, pos, bt, num_pages, offset = t.shape_inputs(d_model, n_kv, hd, n_tok, style)
        r = feasible(case.x, case.gamma, case.wkv, pos, n_kv, hd, theta=500000.0, style=style)
        print(f"shape {d_model}/{n_kv}/{hd}/{n_tok}/{style}: model error {r:.4f} x RMS_head")
        assert r <= TOL


def test_inputs_of_the_split_launch_tests_are_feasible():
    import test_gpu_parity as t
    import test_gpu_fullsize as tf
    for d_model, n_kv, hd, n_tok, style, _ in t.SPLIT_SHAPES:
        case, pos, bt, num_pages, offset = t.shape_inputs(d_model, n_kv, hd, n_tok, style)
        r = feasible(case.x, case.gamma, case.wkv, pos, n_kv, hd, theta=500000.0, style=style)
        print(f"split shape {d_model}/{n_kv}/{hd}/{n_tok}/{style}: model error {r:.4f} x RMS_head")
        assert r <= TOL
    for name, c in tf.SPLIT_CASES.items():
        case, pos, bt, num_pages, rows = tf.split_case_inputs(name)
        r = feasible(case.x[rows], case.gamma, case.wkv, pos[rows], c["n_kv"], c["hd"], theta=500000.0)
        print(f"whole + split tiles {name}, {len(rows)} rows checked element by element: model error {r:.4f} x RMS_head")
        assert r <= MARGIN * TOL


def test_inputs_of_the_store_restore_test_at_the_split_width_are_feasible():
    import test_gpu_parity  # noqa: F401  (the test draws LayerCase([31, layer]) at d_model 2048, tokens 30..679)
    pos = 1000 + 30 + np.arange(650)
    for l in range(5):
        c = gh.LayerCase(np.random.default_rng([31, l]), 2048, 2, 128, 700)
        r = feasible(c.x[30:680], c.gamma, c.wkv, pos, 2, 128)
        print(f"store restore at d_model 2048, layer {l}: model error {r:.4f} x RMS_head")
        assert r <= MARGIN * TOL
