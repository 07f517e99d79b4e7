"""Pins of the 8-bit KV cache variant's oracle: the E4M3 decoder against the format's published values and
against an independent library's float8 type; the byte encoder of the input generator against the same
library; the attention with 8-bit caches against the ordinary oracle on the decoded values."""
import numpy as np
import torch

import oracle
import workloads


def test_decoder_against_published_values_and_torch():
    all_codes = np.arange(256, dtype=np.uint8)
    v = oracle.decode_e4m3(all_codes)
    # values the format's definition fixes (bias 7, 3 mantissa bits, no infinities, max 448)
    assert v[0x00] == 0.0 and v[0x80] == 0.0 and np.signbit(v[0x80])
    assert v[0x01] == 2.0 ** -9 and v[0x07] == 7 * 2.0 ** -9 and v[0x08] == 2.0 ** -6
    assert v[0x38] == 1.0 and v[0x3C] == 1.5 and v[0x40] == 2.0 and v[0xC0] == -2.0
    assert v[0x7E] == 448.0 and v[0xFE] == -448.0 and np.isnan(v[0x7F]) and np.isnan(v[0xFF])
    assert (np.diff(v[:0x7F]) > 0).all()
    ref = torch.from_numpy(all_codes.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.array_equal(v, ref, equal_nan=True)


def test_encoder_of_the_input_generator_against_torch():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(20000) * 3, rng.standard_normal(2000) * 1e-2, rng.uniform(-448, 448, 2000),
                        [0.0, -0.0, 448.0, -448.0, 2.0 ** -10, 3 * 2.0 ** -10, 2.0 ** -9, 0.9375, 1.0625]]).astype(np.float32)
    got = workloads.f32_to_e4m3_bits(x)
    ref = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(got, ref)
    assert np.array_equal(workloads.f32_to_e4m3_bits(np.float32([1000.0, -1e9])), np.uint8([0x7E, 0xFE]))  # saturates
    # decoding what was encoded is the nearest representable value
    back = oracle.decode_e4m3(got)
    assert np.all(np.abs(back - x) <= np.maximum(np.abs(x) * 2.0 ** -4, 2.0 ** -10))


def test_kv8_attention_equals_ordinary_attention_on_decoded_caches():
    b = workloads.make_batch(1, rep=2, with_probs=False)
    rng = np.random.default_rng(3)
    k_scale = rng.uniform(0.5, 2.0, b.H_kv).astype(np.float32)
    v_scale = rng.uniform(0.5, 2.0, b.H_kv).astype(np.float32)
    kf = workloads.bf16_bits_to_f32(b.k_cache) if b.k_cache.dtype == np.uint16 else b.k_cache
    vf = workloads.bf16_bits_to_f32(b.v_cache) if b.v_cache.dtype == np.uint16 else b.v_cache
    k8 = workloads.f32_to_e4m3_bits(kf / k_scale.reshape(1, -1, 1, 1))
    v8 = workloads.f32_to_e4m3_bits(vf / v_scale.reshape(1, -1, 1, 1))
    q_bits = b.q if b.q.dtype == np.uint16 else workloads.f32_to_bf16_bits(b.q)
    out, lse = oracle.verify_attention_kv8(q_bits, k8, v8, k_scale, v_scale, b.block_tables, b.ctx_lens, b.cu_q,
                                           H_q=b.H_q, H_kv=b.H_kv, D=b.D, P=b.P, scale=b.scale)
    # power-of-two scales and fp32-exact products: the ordinary fp32 oracle on the dequantised caches must agree
    ks2, vs2 = np.float32([0.5, 2.0] * (b.H_kv // 2) + [1.0] * (b.H_kv % 2)), np.float32([4.0, 0.25] * (b.H_kv // 2) + [1.0] * (b.H_kv % 2))
    out2, lse2 = oracle.verify_attention_kv8(q_bits, k8, v8, ks2, vs2, b.block_tables, b.ctx_lens, b.cu_q,
                                             H_q=b.H_q, H_kv=b.H_kv, D=b.D, P=b.P, scale=b.scale)
    kd = (oracle.decode_e4m3(k8) * ks2.reshape(1, -1, 1, 1)).astype(np.float32)
    vd = (oracle.decode_e4m3(v8) * vs2.reshape(1, -1, 1, 1)).astype(np.float32)
    qf = workloads.bf16_bits_to_f32(q_bits)
    ref, lse_ref = oracle.verify_attention(qf, kd, vd, b.block_tables, b.ctx_lens, b.cu_q, H_q=b.H_q, H_kv=b.H_kv, D=b.D,
                                           P=b.P, dtype="f32", scale=b.scale)
    assert np.array_equal(out2, ref) and np.array_equal(lse2, lse_ref)
    # a value scale multiplies the output, a key scale is a change of the softmax scale
    out3, _ = oracle.verify_attention_kv8(q_bits, k8, v8, ks2, 2 * vs2, b.block_tables, b.ctx_lens, b.cu_q,
                                          H_q=b.H_q, H_kv=b.H_kv, D=b.D, P=b.P, scale=b.scale)
    assert np.allclose(out3, 2 * out2, rtol=1e-14, atol=0)
    assert np.isfinite(out).all() and out.shape == (b.N, b.H_q, b.D)


def test_oracle_encoder_against_torch_and_the_generators_encoder():
    """The oracle's own E4M3 encoder (a search over the codes) against torch's conversion and against the
    input generator's table-based encoder: three independent writings of the same rounding."""
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.standard_normal(5000) * 4, rng.standard_normal(2000) * 2e-2, rng.uniform(-448, 448, 1000),
                        [0.0, -0.0, 448.0, -448.0, 2.0 ** -10, 3 * 2.0 ** -10, 5 * 2.0 ** -10, 2.0 ** -9, 0.9375, 1.0625,
                         17.0, 19.0, 460.0, -1e6]]).astype(np.float32)
    got = oracle.encode_e4m3(x)
    inside = np.abs(x) <= 448
    ref = torch.from_numpy(x[inside]).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(got[inside], ref)
    assert np.array_equal(got, workloads.f32_to_e4m3_bits(x))          # saturation included
    assert oracle.encode_e4m3(np.float32([np.nan]))[0] == 0x7F
    # every finite code is a fixed point
    codes = np.array([c for c in range(256) if c & 0x7F != 0x7F], np.uint8)
    assert np.array_equal(oracle.encode_e4m3(oracle.decode_e4m3(codes).astype(np.float32)), codes)


def test_quantising_append_is_quantise_then_append():
    b = workloads.make_batch(2, rep=4, with_probs=False, ctx_lens=[5, 17, 30], spec_lens=[2, 0, 3])
    rng = np.random.default_rng(2)
    ks, vs = rng.uniform(0.01, 0.1, b.H_kv).astype(np.float32), rng.uniform(0.01, 0.1, b.H_kv).astype(np.float32)
    k_new = workloads.f32_to_bf16_bits(rng.standard_normal((b.N, b.H_kv, b.D)).astype(np.float32))
    v_new = workloads.f32_to_bf16_bits(rng.standard_normal((b.N, b.H_kv, b.D)).astype(np.float32))
    kc0 = rng.integers(0, 127, size=b.k_cache.shape).astype(np.uint8)
    vc0 = rng.integers(0, 127, size=b.k_cache.shape).astype(np.uint8)
    kc, vc = oracle.kv_append_kv8(k_new, v_new, kc0, vc0, ks, vs, b.block_tables, b.ctx_lens, b.cu_q, P=b.P)
    changed = 0
    for i in range(b.B):
        for j in range(int(b.cu_q[i + 1] - b.cu_q[i])):
            t = int(b.ctx_lens[i]) + j
            page, slot, row = b.block_tables[i, t // b.P], t % b.P, int(b.cu_q[i]) + j
            want = workloads.f32_to_e4m3_bits(workloads.bf16_bits_to_f32(k_new[row]) / ks[:, None])
            assert np.array_equal(kc[page, :, slot, :], want)
            changed += 1
    assert changed == b.N and (kc != kc0).sum() <= b.N * b.H_kv * b.D and (kc != kc0).any()
