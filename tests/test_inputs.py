"""The seeded input generator: determinism, storage rounding, value ranges (no GPU)."""
import numpy as np
import torch

import gfwa_inputs as gi


def test_bf16_rounding_matches_torch():
    x = np.random.default_rng(0).standard_normal(100000).astype(np.float32) * 7
    x[:4] = [0.0, -0.0, 1.00390625, 1.01171875]     # exact ties
    r = gi.round_to_bf16(x)
    t = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(r, t)
    # representable: converting again changes nothing, and the device sees the same bits
    np.testing.assert_array_equal(gi.round_to_bf16(r), r)
    bits = torch.from_numpy(r).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(bits, gi.bf16_bits(r))


def test_deterministic_and_shaped():
    wl = gi.custom("t", 2, 3, 50, 8, 7, "bf16", alpha_mu=-2.0, backward=True)
    a, b = gi.make_inputs(wl), gi.make_inputs(wl)
    for k in ("Q", "K", "V", "alpha", "dO"):
        np.testing.assert_array_equal(a[k], b[k])
    assert a["Q"].shape == (2, 3, 50, 8) and a["alpha"].shape == (2, 3, 50)
    assert a["alpha"].dtype == np.float32 and (a["alpha"] >= 0).all()
    assert not np.array_equal(a["Q"], a["K"])
    sub = gi.make_tensor(wl, "K", heads=[4, 1])
    np.testing.assert_array_equal(sub[0], a["K"][1, 1])
    np.testing.assert_array_equal(sub[1], a["K"][0, 1])


def test_named_workloads_match_the_stated_configs():
    w = gi.WORKLOADS
    assert (w["long_fwd"].B, w["long_fwd"].H, w["long_fwd"].N, w["long_fwd"].d, w["long_fwd"].w) == (1, 32, 16384, 128, 1024)
    assert w["long_fwd"].flops_fwd_nominal() == 4 * 32 * 16384 * 1024 * 128
    assert abs(w["long_fwd"].flops_fwd_exact() / 1e9 - 266.3) < 0.1
    assert w["train_bwd"].flops_bwd_nominal() == 10 * 64 * 8192 * 1024 * 128
    ge = gi.custom("ge", 1, 8, 64, 8, 16, "bf16", alpha_mu=1.0, zero_gate_heads=(0, 1, 2, 3))
    al = gi.make_tensor(ge, "alpha")
    assert (al[:, :4] == 0).all() and (al[:, 4:] > 0).all()
