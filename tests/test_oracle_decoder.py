"""Pins of the oracle's decoder and KV cache: brute force without a cache, and a
whole-sequence forward written with library routines.  CPU only."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import sb_inputs as si
from helpers import tiny_model, params


VARIANTS = {
    "fp32-mha": dict(),
    "bf16-mha": dict(weight_dtype=si.configs.BF16, kv_dtype=si.configs.BF16),
    "fp32-gqa": dict(n_kv_heads=2),
    "bf16-gqa-bigrope": dict(weight_dtype=si.configs.BF16, kv_dtype=si.configs.BF16, n_kv_heads=1,
                             rope_base=500000.0),
}


@pytest.mark.parametrize("variant", list(VARIANTS))
def test_cached_decode_equals_bruteforce_without_cache(variant):
    shape, w, m = tiny_model(n_layers=3, n_exit_heads=0, seed=11, **VARIANTS[variant])
    prompt = si.make_prompt(shape.vocab, 9, 5)
    n_new = 7
    bf, bf_logits = m.greedy_nocache(prompt, n_new, want_logits=True)
    s = m.session()
    out = s.generate(prompt, n_new, params(0, 1))
    assert out.tolist() == bf.tolist()
    # logits that chose the last token: cached path vs recomputed-from-scratch path
    cached = s.verify_logits(0)
    assert np.max(np.abs(cached - bf_logits)) <= 1e-9 * max(1.0, np.max(np.abs(bf_logits)))


def _torch_forward(shape, w, tokens):
    """All positions at once with torch library ops (float64); returns logits [n, V]."""
    def mat(name):
        a = w[name]
        a = si.bf16_to_f32(a) if a.dtype == np.uint16 else a
        return torch.from_numpy(a.astype(np.float64))
    def rnd(x):
        if shape.kv_dtype == si.configs.BF16:
            return x.float().bfloat16().double()
        return x.float().double()
    n = len(tokens)
    hd, Hq, Hkv = shape.head_dim, shape.n_heads, shape.n_kv_heads
    h = mat("embed")[torch.as_tensor(np.asarray(tokens), dtype=torch.long)]
    pos = torch.arange(n, dtype=torch.float64)
    inv = torch.tensor([shape.rope_base ** (-2.0 * i / hd) for i in range(hd // 2)], dtype=torch.float64)
    ang = pos[:, None] * inv[None, :]
    # the rope table is held in float (double -> float), as in the oracle's definition
    rot = torch.polar(torch.ones_like(ang), ang)
    rot = torch.complex(rot.real.float().double(), rot.imag.float().double())
    def rope(x):  # x [n, H, hd], pairs (i, i + hd/2)
        z = torch.complex(x[..., : hd // 2], x[..., hd // 2:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)
    for l in range(shape.n_layers):
        x = F.rms_norm(h, (shape.d_model,), torch.from_numpy(w[f"attn_norm.{l}"]).double(), shape.rms_eps)
        qkv = F.linear(x, mat(f"w_qkv.{l}"))
        q, k, v = torch.split(qkv, [Hq * hd, Hkv * hd, Hkv * hd], dim=-1)
        q = rope(q.view(n, Hq, hd)); k = rnd(rope(k.view(n, Hkv, hd))); v = rnd(v.view(n, Hkv, hd))
        k = k.repeat_interleave(Hq // Hkv, dim=1); v = v.repeat_interleave(Hq // Hkv, dim=1)
        a = F.scaled_dot_product_attention(q.transpose(0, 1), k.transpose(0, 1), v.transpose(0, 1),
                                           is_causal=True)
        h = h + F.linear(a.transpose(0, 1).reshape(n, Hq * hd), mat(f"w_o.{l}"))
        x = F.rms_norm(h, (shape.d_model,), torch.from_numpy(w[f"ffn_norm.{l}"]).double(), shape.rms_eps)
        g, u = F.linear(x, mat(f"w_gate_up.{l}")).chunk(2, dim=-1)
        h = h + F.linear(F.silu(g) * u, mat(f"w_down.{l}"))
    x = F.rms_norm(h, (shape.d_model,), torch.from_numpy(w["final_norm"]).double(), shape.rms_eps)
    return F.linear(x, mat("lm_head")).numpy()


@pytest.mark.parametrize("variant", list(VARIANTS))
def test_teacher_forced_logits_equal_library_forward(variant):
    shape, w, m = tiny_model(n_layers=3, n_exit_heads=0, seed=12, **VARIANTS[variant])
    tokens = si.make_prompt(shape.vocab, 12, 6)
    ref = _torch_forward(shape, w, tokens)
    s = m.session()
    first = s.prefill(tokens[:5])
    assert first == int(np.argmax(ref[4]))
    assert np.max(np.abs(s.verify_logits(0) - ref[4])) < 2e-5
    for i in range(5, 12):
        am, z = s.step(int(tokens[i]))
        # bf16 KV rounding happens on slightly different doubles: allow a few bf16 ulps of K/V
        lim = 2e-5 if shape.kv_dtype == si.configs.FP32 else 5e-3
        assert np.max(np.abs(z - ref[i])) < lim, (i, np.max(np.abs(z - ref[i])))
        if np.sort(ref[i])[-1] - np.sort(ref[i])[-2] > 2 * lim:
            assert am == int(np.argmax(ref[i]))


def test_float_oracle_tracks_double_oracle():
    shape, w, m64 = tiny_model(n_layers=4, n_exit_heads=2, seed=13)
    _, _, m32 = tiny_model(n_layers=4, n_exit_heads=2, seed=13, bits=32)
    prompt = si.make_prompt(shape.vocab, 16, 7)
    s64, s32 = m64.session(), m32.session()
    assert s64.prefill(prompt) == s32.prefill(prompt)
    z64, z32 = s64.verify_logits(0), s32.verify_logits(0)
    assert np.max(np.abs(z64 - z32)) < 1e-4 * np.max(np.abs(z64))


def test_kv_cache_rounding_point():
    shape, w, m = tiny_model(n_layers=2, n_exit_heads=0, seed=14, weight_dtype=si.configs.BF16,
                             kv_dtype=si.configs.BF16)
    s = m.session()
    s.prefill(si.make_prompt(shape.vocab, 4, 8))
    k, v = s.kv_read(1, 3)
    # everything in the cache is exactly representable in bf16
    assert np.array_equal(si.bf16_to_f32(si.round_to_bf16(k)), k)
    assert np.array_equal(si.bf16_to_f32(si.round_to_bf16(v)), v)
    assert np.abs(k).max() > 0 and np.abs(v).max() > 0
