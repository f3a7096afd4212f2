"""The seeded input generators: shapes, determinism, bf16 rounding (CPU only)."""
import numpy as np
import torch

from paper_2601_15473_amd import workloads as W


def test_bf16_rounding_is_nearest_even():
    r = np.random.default_rng(0)
    a = (r.standard_normal(200000) * np.exp(r.uniform(-20, 20, 200000))).astype(np.float32)
    # exact ties and near-ties
    ties = np.array([0x3F808000, 0x3F818000, 0x3F807FFF, 0x3F808001, 0xBF808000, 0x00000000],
                    dtype=np.uint32).view(np.float32)
    a = np.concatenate([a, ties])
    bits = W.f32_to_bf16_bits(a)
    want = torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(bits, want)
    assert bits[-6] == 0x3F80 and bits[-5] == 0x3F82      # ties go to the even mantissa
    back = W.bf16_bits_to_f32(bits)
    np.testing.assert_array_equal(back, torch.from_numpy(a).to(torch.bfloat16).float().numpy())


def test_generate_shapes_and_determinism():
    w = W.scaled(W.BERT_BASE_FFN_UP, tokens=40)
    t1, t2 = W.generate(w), W.generate(w)
    assert t1.stored["x"].shape == (40, 768) and t1.stored["x"].dtype == np.uint16
    assert t1.stored["S"].shape == (2, 768, 64) and t1.stored["U"].shape == (2, 64, 3072)
    assert t1.stored["b"].shape == (3072,) and t1.stored["dY"].shape == (40, 3072)
    for n in t1.stored:
        np.testing.assert_array_equal(t1.stored[n], t2.stored[n])
        np.testing.assert_array_equal(W.bf16_bits_to_f32(t1.stored[n]), t1.value[n])
    assert "b" not in W.generate(w, with_bias=False).stored
    S_cat, U_cat = t1.S_cat("value"), t1.U_cat("value")
    assert S_cat.shape == (768, 128) and U_cat.shape == (128, 3072)
    np.testing.assert_array_equal(S_cat[:, 64:], t1.value["S"][1])
    np.testing.assert_array_equal(U_cat[64:], t1.value["U"][1])


def test_distributions():
    w = W.scaled(W.TINY, tokens=4096)
    t = W.generate(w)
    assert t.stored["x"].dtype == np.float32
    assert abs(t.value["x"].var() - 1.0) < 0.02
    assert abs(t.value["S"].var() * w.k - 1.0) < 0.05
    assert abs(t.value["U"].var() * w.l * w.k - 1.0) < 0.05
    assert abs(t.value["b"].var() / 0.01 - 1.0) < 0.3
    h = W.generate(W.scaled(W.LLM_MLP, tokens=256, d_out=256))
    xv = h.value["x"].astype(np.float64)
    kurt = np.mean(xv ** 4) / np.mean(xv ** 2) ** 2
    assert kurt > 6.0            # heavy tails (a Gaussian has 3)
    assert 0.5 < xv.var() < 2.0


def test_config_table():
    assert len(W.ALL) == 10
    assert W.LLM_MLP.R == 2048 and W.BERT_BASE_FFN_UP.R == 128
    assert [w.k for w in W.BERT_BASE_PROJ] == [16, 32, 64, 128, 192]
