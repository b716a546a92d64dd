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


# ---- attention-side integration: merge of two partial results, rotary embedding of decoded keys ----
def test_merge_of_two_key_sets_equals_attention_over_their_union(rng):
    """The identity the merge is defined by (Sec. 3.1: a chunk attends to the cached chunks and
    to itself): softmax over A ∪ B from the two partial results and their log-sum-exps."""
    Nq, Na, Nb, d = 13, 150, 37, 128
    q = _rand_bf16(rng, Nq, d)
    ka, va = _rand_bf16(rng, Na, d), _rand_bf16(rng, Na, d, scale=2.0)
    kb, vb = _rand_bf16(rng, Nb, d, scale=1.5), _rand_bf16(rng, Nb, d)      # B's scores are larger
    oa, la = O.attention(bf16_bits(q), bf16_bits(ka), bf16_bits(va), want_lse=True)
    ob, lb = O.attention(bf16_bits(q), bf16_bits(kb), bf16_bits(vb), want_lse=True)
    o, l = O.attn_merge(oa, la, ob, lb)
    want, lw = O.attention(bf16_bits(q), bf16_bits(torch.cat([ka, kb])), bf16_bits(torch.cat([va, vb])),
                           want_lse=True)
    assert np.allclose(o, want, rtol=1e-11, atol=1e-12) and np.allclose(l, lw, rtol=1e-13)
    # a far smaller second set changes nothing; swapping the operands changes nothing
    o2, l2 = O.attn_merge(oa, la, ob, lb - 800.0)
    assert np.array_equal(o2, oa) and np.array_equal(l2, la)
    o3, l3 = O.attn_merge(ob, lb, oa, la)
    assert np.allclose(o3, o, rtol=1e-14, atol=1e-15) and np.allclose(l3, l, rtol=1e-15)


def _rope_table(rng, N, d, theta=10000.0, positions=None):
    pos = np.arange(N, dtype=np.float64) if positions is None else np.asarray(positions, np.float64)
    freq = theta ** (-np.arange(d // 2, dtype=np.float64) / (d // 2))
    ang = pos[:, None] * freq[None]
    tab = np.stack([np.cos(ang), np.sin(ang)], -1).astype(np.float16)       # [N, d/2, 2]
    return tab.view(np.uint16), tab.astype(np.float64)


def test_rope_matches_complex_multiplication(rng):
    """Interleaved pairs rotated by (cos, sin): torch's complex product on the same binary16 table
    in fp64, to the bf16 rounding of the result; the sign and the pairing are what this pins."""
    N, d = 50, 128
    k = _rand_bf16(rng, N, d, scale=2.0)
    bits, tab = _rope_table(rng, N, d)
    got = bits_to_f32(O.rope_keys(bf16_bits(k), bits)).astype(np.float64)
    z = torch.view_as_complex(k.double().reshape(N, d // 2, 2).contiguous())
    rot = torch.view_as_complex(torch.from_numpy(tab).contiguous())
    want = torch.view_as_real(z * rot).reshape(N, d).numpy()
    assert np.abs(got - want).max() <= 2.0 ** -8 * np.abs(want).max()
    assert (np.abs(got - want) <= 2.0 ** -8 * np.abs(want) + 1e-6).all()
    # position 0 (cos 1, sin 0) leaves the keys bit-identical
    assert np.array_equal(O.rope_keys(bf16_bits(k[:1]), bits[:1]), bf16_bits(k[:1]))
    # a quarter turn in every pair: (x0, x1) -> (-x1, x0), exactly
    quarter = np.zeros((1, d // 2, 2), np.float16); quarter[..., 1] = 1.0
    out = bits_to_f32(O.rope_keys(bf16_bits(k[:1]), quarter.view(np.uint16)))
    kk = k[:1].float().numpy()
    assert np.array_equal(out[0, 0::2], -kk[0, 1::2]) and np.array_equal(out[0, 1::2], kk[0, 0::2])


def test_rope_scores_depend_on_the_position_difference(rng):
    """The property the embedding exists for: <R(p) q, R(p') k> = <R(p - p') q, k>."""
    d = 128
    q, k = _rand_bf16(rng, 1, d), _rand_bf16(rng, 1, d)
    def score(pq, pk):
        bq, _ = _rope_table(rng, 1, d, positions=[pq])
        bk, _ = _rope_table(rng, 1, d, positions=[pk])
        rq = bits_to_f32(O.rope_keys(bf16_bits(q), bq)).astype(np.float64)
        rk = bits_to_f32(O.rope_keys(bf16_bits(k), bk)).astype(np.float64)
        return float((rq * rk).sum())
    base = score(7, 3)
    for shift in (1, 10, 40):
        assert abs(score(7 + shift, 3 + shift) - base) < 0.05 * np.sqrt(d)      # bf16/f16 rounding only
    assert abs(score(7, 3) - score(3, 7)) > 0.05                               # not symmetric
