"""Pins for the oracle's storage-format helpers (bfloat16 widening and rounding)."""
import numpy as np
import torch

from oracle import medusa_oracle as O


def test_widen_bf16_matches_torch():
    bits = np.arange(0, 1 << 16, dtype=np.uint16)
    bits = bits[(bits & 0x7F80) != 0x7F80]                    # finite patterns only
    ours = O.widen(bits)
    lib = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(ours, lib)


def test_round_to_bf16_hand_cases():
    # spacing of bfloat16 in [1, 2) is 2^-7
    x = np.array([1.0, 1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 1 + 2.0 ** -8 + 2.0 ** -40, -(1 + 3 * 2.0 ** -8), 0.0,
                  3.0e38, 3.4e38, 3.0 * 2.0 ** -133 + 2.0 ** -135, 2.0 ** -134])
    want = np.array([1.0, 1.0, 1 + 2.0 ** -6, 1 + 2.0 ** -7, -(1 + 2.0 ** -6), 0.0,
                     226 * 2.0 ** 120, np.inf, 3.0 * 2.0 ** -133, 0.0])
    got = O.round_to_bf16(x)
    assert np.array_equal(got, want)


def test_round_to_bf16_matches_torch_on_float32_inputs():
    # For inputs that are already float32, torch's float32 -> bfloat16 cast is the same rounding.
    rng = np.random.default_rng(5)
    x32 = (rng.standard_normal(200000) * np.exp(rng.uniform(-20, 20, 200000))).astype(np.float32)
    lib = torch.from_numpy(x32).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(O.round_to_bf16(x32.astype(np.float64)), lib)


def test_round_to_bf16_is_direct_not_via_float32():
    # 1 + 2^-8 + 2^-30 is above the tie; float32 would first round it down onto the tie.
    x = np.array([1 + 2.0 ** -8 + 2.0 ** -30])
    assert O.round_to_bf16(x)[0] == 1 + 2.0 ** -7
    via32 = torch.tensor(x.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    assert via32[0] == 1.0


def test_generator_bf16_rounding_matches_torch():
    from workloads import bf16_bits_from_f32, f32_from_bf16_bits
    rng = np.random.default_rng(6)
    x = rng.standard_normal(100000).astype(np.float32)
    bits = bf16_bits_from_f32(x)
    lib = torch.from_numpy(x).to(torch.bfloat16)
    assert np.array_equal(bits.view(np.int16), lib.view(torch.int16).numpy())
    assert np.array_equal(f32_from_bf16_bits(bits), lib.to(torch.float32).numpy())


def test_generator_is_deterministic_and_chunk_independent():
    from workloads import draw_normal
    a = draw_normal(3, 7, (5, 1000), 1.0, "f32")
    b = draw_normal(3, 7, (5, 1000), 1.0, "f32")
    c = draw_normal(3, 8, (5, 1000), 1.0, "f32")
    assert np.array_equal(a, b) and not np.array_equal(a, c)
    big = draw_normal(1, 2, ((1 << 22) + 17,), 0.02, "bf16")     # two chunks
    assert big.dtype == np.uint16 and big.shape == ((1 << 22) + 17,)
    assert abs(float(O.widen(big).std()) - 0.02) < 2e-4
