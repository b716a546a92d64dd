"""Pins for the oracle's attention: torch scaled_dot_product_attention and two closed forms."""
import numpy as np
import torch

from oracle import qvg_oracle as O
from conftest import bf16_bits, bits_to_f32


def _rand_bf16(rng, *shape, scale=1.0):
    return torch.from_numpy((rng.standard_normal(shape) * scale).astype(np.float32)).to(torch.bfloat16)


def test_matches_torch_sdpa(rng):
    Nq, Nk, d = 17, 203, 128
    q, k, v = _rand_bf16(rng, Nq, d), _rand_bf16(rng, Nk, d), _rand_bf16(rng, Nk, d, scale=3.0)
    out, lse = O.attention(bf16_bits(q), bf16_bits(k), bf16_bits(v), want_lse=True)
    want = torch.nn.functional.scaled_dot_product_attention(
        q.double()[None], k.double()[None], v.double()[None])[0].numpy()
    assert np.allclose(out, want, rtol=1e-9, atol=1e-10)
    s = (q.double() @ k.double().T) / np.sqrt(d)
    assert np.allclose(lse, torch.logsumexp(s, dim=1).numpy(), rtol=1e-12)
    # non-default scale
    out2 = O.attention(bf16_bits(q), bf16_bits(k), bf16_bits(v), scale=0.3)
    want2 = torch.nn.functional.scaled_dot_product_attention(
        q.double()[None], k.double()[None], v.double()[None], scale=0.3)[0].numpy()
    assert np.allclose(out2, want2, rtol=1e-9, atol=1e-10)


def test_single_key_returns_its_value(rng):
    q, k, v = _rand_bf16(rng, 5, 128), _rand_bf16(rng, 1, 128), _rand_bf16(rng, 1, 128)
    out = O.attention(bf16_bits(q), bf16_bits(k), bf16_bits(v))
    assert np.array_equal(out, np.repeat(bits_to_f32(bf16_bits(v)).astype(np.float64), 5, 0))


def test_identical_keys_average_the_values(rng):
    q, k1, v = _rand_bf16(rng, 4, 128), _rand_bf16(rng, 1, 128), _rand_bf16(rng, 9, 128)
    k = k1.repeat(9, 1)
    out = O.attention(bf16_bits(q), bf16_bits(k), bf16_bits(v))
    assert np.allclose(out, v.double().mean(0).numpy()[None].repeat(4, 0), rtol=1e-12, atol=1e-13)


def test_batch_heads_are_independent(rng):
    H, Nq, Nk, d = 3, 6, 20, 128
    q, k, v = _rand_bf16(rng, H, Nq, d), _rand_bf16(rng, H, Nk, d), _rand_bf16(rng, H, Nk, d)
    out = O.attention_batch(bf16_bits(q), bf16_bits(k), bf16_bits(v))
    for h in range(H):
        assert np.array_equal(out[h], O.attention(bf16_bits(q[h]), bf16_bits(k[h]), bf16_bits(v[h])))
