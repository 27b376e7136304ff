"""Pins for the oracle's storage-dtype helpers: torch's own bf16 cast is the library
routine they must agree with on fp32-representable inputs; ties are checked by hand."""
import numpy as np
import torch

from oracle import storage


def test_bf16_roundtrip_matches_torch_cast():
    rng = np.random.default_rng(0)
    x32 = np.concatenate([
        rng.standard_normal(20000).astype(np.float32) * 0.02,
        rng.standard_normal(20000).astype(np.float32) * 1e-3,
        np.float32(2.0) ** rng.integers(-30, 30, 2000).astype(np.float32),
        np.array([0.0, -0.0, 1.0, -1.0, 3.0e38, -3.0e38], dtype=np.float32),
    ])
    want = torch.from_numpy(x32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = storage.f64_to_bf16_bits(x32.astype(np.float64))
    assert np.array_equal(got, want)
    back = storage.bf16_bits_to_f64(got)
    assert np.array_equal(back, torch.from_numpy(x32).to(torch.bfloat16).double().numpy())


def test_bf16_ties_to_even_and_single_rounding():
    # 1 + 2^-8 is halfway between 1 and 1 + 2^-7: tie -> even mantissa (1.0)
    assert storage.round_to_storage(np.array([1.0 + 2.0 ** -8]), "bf16")[0] == 1.0
    # 1 + 3*2^-8 is halfway between 1+2^-7 and 1+2^-6: tie -> 1 + 2^-6 (even)
    assert storage.round_to_storage(np.array([1.0 + 3 * 2.0 ** -8]), "bf16")[0] == 1.0 + 2.0 ** -6
    # just above a tie must round up even though fp32 would first round it onto the tie
    x = 1.0 + 2.0 ** -8 + 2.0 ** -40
    assert storage.round_to_storage(np.array([x]), "bf16")[0] == 1.0 + 2.0 ** -7
    assert storage.round_to_storage(np.array([-x]), "bf16")[0] == -(1.0 + 2.0 ** -7)


def test_bf16_ulp():
    assert storage.bf16_ulp(np.array([1.0]))[0] == 2.0 ** -7
    assert storage.bf16_ulp(np.array([0.02]))[0] == 2.0 ** -13
    assert storage.bf16_ulp(np.array([-3.0]))[0] == 2.0 ** -6


def test_f32_storage():
    x = np.array([0.1, 1.0 / 3.0])
    assert np.array_equal(storage.round_to_storage(x, "f32"), x.astype(np.float32).astype(np.float64))
