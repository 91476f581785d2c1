"""Pins of the oracle's binary16 input path (the paper serves its models in float16,
Sec. 4.1.1): the element decoder against numpy's float16 for every bit pattern, and the
whole forward against a library routine on float16 inputs.  CPU only.
"""
import math

import numpy as np
import torch

from oracle import decode_elems, input_format, swaa_attn_oracle, swaa_attn_oracle_numpy
from paper_2512_10411_amd.inputs import f16_bits_to_f32, f32_to_f16_bits, make_qkv


def test_every_binary16_pattern_decodes_like_numpy():
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float64)
    with input_format("fp16"):
        got = decode_elems(bits)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], ref[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(ref[~nan]))
    # and the switch is restored: the same patterns read as bfloat16 again
    again = decode_elems(bits[:0x7f80])
    assert np.array_equal(again, (bits[:0x7f80].astype(np.uint32) << 16).view(np.float32).astype(np.float64))


def test_rounding_helper_matches_torch():
    x = np.random.Generator(np.random.Philox(6)).standard_normal(4096, dtype=np.float32)
    x[:6] = [0.0, -0.0, 1.0, 1.00048828125, 65519.0, 6e-8]
    ours = f32_to_f16_bits(x)
    ref = torch.from_numpy(x).to(torch.float16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, ref)
    assert np.array_equal(f16_bits_to_f32(ours), torch.from_numpy(x).to(torch.float16).float().numpy())


def test_float16_inputs_against_sdpa_and_numpy_route():
    B, Hq, Hkv, N, D = 2, 4, 2, 64, 32
    q, k, v = make_qkv(B, Hq, Hkv, N, D, seed=17, fmt="fp16")
    scale = 1 / math.sqrt(D)
    with input_format("fp16"):
        o, lse = swaa_attn_oracle(q, k, v, N, 0, scale)
        o2, l2 = swaa_attn_oracle_numpy(q, k, v, 9, 3, scale)
        o3, l3 = swaa_attn_oracle(q, k, v, 9, 3, scale)
    f = lambda a: torch.from_numpy(a.view(np.float16).astype(np.float64))
    ref = torch.nn.functional.scaled_dot_product_attention(
        f(q), f(k).repeat_interleave(2, 1), f(v).repeat_interleave(2, 1), is_causal=True, scale=scale)
    assert np.abs(o - ref.numpy()).max() < 1e-12
    assert np.abs(o2 - o3).max() < 1e-13 and np.abs(l2 - l3).max() < 1e-13
    # the same bits read as bfloat16 give another answer: the switch matters
    o_bf, _ = swaa_attn_oracle(q, k, v, N, 0, scale)
    assert not np.allclose(o, o_bf)
