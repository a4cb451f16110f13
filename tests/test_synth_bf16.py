"""The seeded input generator's bfloat16 conversions against torch's (CPU): every bf16 input of the
parity tests is produced by synth.f32_to_bf16_bits, so a wrong rounding there would feed both the
oracle and the GPU the same wrong bits and go unnoticed."""
import numpy as np
import torch

from paper_2603_08343_amd import synth


def _torch_bf16_bits(a: np.ndarray) -> np.ndarray:
    return torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def test_rounding_matches_torch_on_random_values():
    rng = np.random.default_rng(0)
    a = np.concatenate([rng.standard_normal(200_000).astype(np.float32),
                        (rng.standard_normal(50_000) * 1e-3).astype(np.float32),
                        (rng.standard_normal(50_000) * 300.0).astype(np.float32)])
    assert np.array_equal(synth.f32_to_bf16_bits(a), _torch_bf16_bits(a))


def test_ties_round_to_even():
    # values exactly half way between two bfloat16 neighbours: low 16 bits = 0x8000
    hi = np.array([0x3F80, 0x3F81, 0x4000, 0x4001, 0xBF80, 0xBF81, 0x0080, 0x7F7E], dtype=np.uint32)
    ties = ((hi << np.uint32(16)) | np.uint32(0x8000)).view(np.float32)
    got = synth.f32_to_bf16_bits(ties)
    want = np.where(hi & 1, hi + 1, hi).astype(np.uint16)          # odd mantissa rounds up, even stays
    assert np.array_equal(got, want)
    assert np.array_equal(got, _torch_bf16_bits(ties))
    # just below / just above the tie
    below = ((hi << np.uint32(16)) | np.uint32(0x7FFF)).view(np.float32)
    above = ((hi << np.uint32(16)) | np.uint32(0x8001)).view(np.float32)
    assert np.array_equal(synth.f32_to_bf16_bits(below), hi.astype(np.uint16))
    assert np.array_equal(synth.f32_to_bf16_bits(above), (hi + 1).astype(np.uint16))


def test_widening_is_exact_and_matches_torch():
    bits = np.arange(0, 0x7F80, 7, dtype=np.uint16)                 # finite, non-negative patterns
    bits = np.concatenate([bits, bits | np.uint16(0x8000)])
    wide = synth.bf16_bits_to_f32(bits)
    want = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(wide.view(np.uint32), want.view(np.uint32))
    assert np.array_equal(synth.f32_to_bf16_bits(wide), bits)       # round trip


def test_workload_inputs_are_bf16_exact():
    inp = synth.make_inputs(5, 64, "bf16", seed=1)
    assert inp.x.dtype == np.uint16 and inp.dy.dtype == np.uint16
    x32 = synth.bf16_bits_to_f32(inp.x)
    assert np.array_equal(_torch_bf16_bits(x32), inp.x)


def test_two_term_split_error_bound_stated_in_the_header():
    """include/wht_affine.h promises that a float32 value entering a matrix-core round as
    hi = RNE_bf16(v), lo = RNE_bf16(v - hi) is carried to a relative error of at most 2^-17.
    Checked here with torch's conversions on dense and random values: v - hi is exact in float32,
    the bound holds, and it is attained to within a factor two (so it is not loose by more)."""
    rng = np.random.default_rng(1)
    v = np.concatenate([np.linspace(1.0, 2.0, 2_000_001, dtype=np.float32),
                        rng.standard_normal(2_000_000).astype(np.float32),
                        (rng.standard_normal(500_000) * 1e-6).astype(np.float32)])
    v = v[v != 0]
    t = torch.from_numpy(v)
    hi = t.to(torch.bfloat16).float()
    rest = t - hi
    assert torch.equal(rest.double(), t.double() - hi.double())    # exact difference
    lo = rest.to(torch.bfloat16).float()
    err = ((t.double() - hi.double() - lo.double()).abs() / t.double().abs()).max().item()
    assert err <= 2.0 ** -17
    assert err > 2.0 ** -18
