"""Pins for the acceptance checker (oracle/check.py): its rounding routine
against library conversions and hand-picked ties, and the accept/reject logic
on values constructed by hand."""
import numpy as np
import torch

from oracle import rne_to_format, acceptance_bound, check_against_oracle, decode_output


def _rand(n, seed):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal(n) * np.exp(rng.standard_normal(n) * 25)).astype(np.float64)


def test_rne_bf16_matches_torch_on_float32_inputs():
    x = _rand(200000, 1).astype(np.float32)
    x = x[np.isfinite(x)]
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    got = rne_to_format(x.astype(np.float64), "bf16")
    assert (got == want).all()


def test_rne_f16_and_f32_match_numpy():
    x = _rand(200000, 2)
    with np.errstate(over="ignore"):
        assert (rne_to_format(x, "f32") == x.astype(np.float32).astype(np.float64)).all()
        x = x * 1e-20 ** 0  # same values; fp16 range is narrow so also scale some down
        y = np.concatenate([x, x * 1e-6, _rand(1000, 3) * 1e-7])
        assert (rne_to_format(y, "f16") == y.astype(np.float16).astype(np.float64)).all()


def test_rne_representable_values_are_fixed_points():
    bits = np.arange(65536, dtype=np.uint16)
    v = (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    v = v[np.isfinite(v)]
    assert (rne_to_format(v, "bf16") == v).all()
    h = bits.view(np.float16).astype(np.float64)
    h = h[np.isfinite(h)]
    assert (rne_to_format(h, "f16") == h).all()


def test_rne_ties_go_to_even():
    # bf16 spacing in [1, 2) is 2^-7
    s = 2.0 ** -7
    assert rne_to_format(np.array([1.0 + 0.5 * s]), "bf16")[0] == 1.0          # 128 even
    assert rne_to_format(np.array([1.0 + 1.5 * s]), "bf16")[0] == 1.0 + 2 * s  # 130 even
    assert rne_to_format(np.array([-(1.0 + 2.5 * s)]), "bf16")[0] == -(1.0 + 2 * s)
    assert rne_to_format(np.array([1.0 + 0.5 * s + 1e-12]), "bf16")[0] == 1.0 + s
    # fp16 subnormal spacing is 2^-24; 0.5 ulp ties to zero, 1.5 ulp ties to 2 ulp
    t = 2.0 ** -24
    assert rne_to_format(np.array([0.5 * t]), "f16")[0] == 0.0
    assert rne_to_format(np.array([1.5 * t]), "f16")[0] == 2 * t
    # overflow
    assert rne_to_format(np.array([65520.0]), "f16")[0] == np.inf
    assert rne_to_format(np.array([65519.0]), "f16")[0] == 65504.0


def test_bound_formula():
    b = acceptance_bound(np.array([0.0, 1.0, 8192.0]), 32768)
    assert b[0] == 1e-6
    assert b[1] == 2.0 ** -7 + 1e-6            # 4 * 2^15 * 2^-24 = 2^-7
    assert b[2] == 64.0 + 1e-6


def test_check_f32_accept_reject():
    ref = np.array([[100.0, -3.0]])
    mag = np.array([[200.0, 6.0]])
    K = 256
    bound = 4 * 256 * 2.0 ** -24 * mag + 1e-6
    ok = check_against_oracle(ref + 0.99 * bound, ref, mag, K, "f32")
    assert ok["ok"] and ok["n_bad"] == 0 and ok["max_err_over_bound"] < 1.0
    bad = check_against_oracle(ref + np.array([[0.0, 1.01]]) * bound, ref, mag, K, "f32")
    assert not bad["ok"] and bad["n_bad"] == 1 and bad["first_bad"] == (0, 1)
    neg = check_against_oracle(-ref, ref, mag, K, "f32")       # a sign error must fail
    assert not neg["ok"]


def test_check_bf16_output_allows_exactly_the_final_rounding():
    # ref = 100.3, tiny bound: the only acceptable bf16 outputs are the roundings of
    # values within the bound, i.e. 100.5 (bf16 spacing at 100 is 0.5)
    ref = np.array([100.3])
    mag = np.array([1.0])
    assert check_against_oracle(np.array([100.5]), ref, mag, 1, "bf16")["ok"]
    assert not check_against_oracle(np.array([100.0]), ref, mag, 1, "bf16")["ok"]
    assert not check_against_oracle(np.array([101.0]), ref, mag, 1, "bf16")["ok"]
    # near a rounding boundary both neighbours are acceptable
    ref = np.array([100.25])
    assert check_against_oracle(np.array([100.0]), ref, mag, 1, "bf16")["ok"]
    assert check_against_oracle(np.array([100.5]), ref, mag, 1, "bf16")["ok"]
    assert not check_against_oracle(np.array([99.5]), ref, mag, 1, "bf16")["ok"]


def test_decode_output():
    f = np.array([1.5, -2.25], dtype=np.float32)
    assert (decode_output(f, "f32") == f.astype(np.float64)).all()
    bits = np.array([0x3FC0, 0xC010], dtype=np.uint16)        # 1.5, -2.25 in bf16
    assert (decode_output(bits, "bf16") == np.array([1.5, -2.25])).all()
    hb = np.array([1.5, -2.25], dtype=np.float16).view(np.uint16)
    assert (decode_output(hb, "f16") == np.array([1.5, -2.25])).all()
