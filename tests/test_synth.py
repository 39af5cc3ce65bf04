"""The seeded input generators: determinism, slab independence, value ranges and moments."""
import numpy as np
import pytest
import torch

from paper_2505_22758_amd import synth


def test_elements_depend_only_on_seed_name_index():
    a = synth.normal_bf16(5, "t", (1000,), 0.02, "cpu")
    b = synth.normal_bf16(5, "t", (10, 100), 0.02, "cpu")
    assert torch.equal(a, b.view(-1))
    assert not torch.equal(a, synth.normal_bf16(6, "t", (1000,), 0.02, "cpu"))
    assert not torch.equal(a, synth.normal_bf16(5, "u", (1000,), 0.02, "cpu"))
    # chunked generation equals hashing the same indices directly
    old = synth._CHUNK
    try:
        synth._CHUNK = 333
        c = synth.normal_bf16(5, "t", (1000,), 0.02, "cpu")
    finally:
        synth._CHUNK = old
    assert torch.equal(a, c)


def test_moments_and_ranges():
    w = synth.normal_bf16(1, "w", (512, 512), 0.02, "cpu").float()
    assert abs(w.mean().item()) < 2e-4 and w.std().item() == pytest.approx(0.02, rel=0.02)
    g = synth.normal_bf16(1, "g", (4096,), 0.02, "cpu", mean=1.0).float()
    assert g.mean().item() == pytest.approx(1.0, abs=2e-3)
    q = synth.uniform_int(1, "q", (100000,), -127, 127, "cpu", torch.int8)
    assert q.min().item() == -127 and q.max().item() == 127
    assert q.float().std().item() == pytest.approx(73.6, rel=0.02)
    t = synth.make_tokens(synth.TINY, 3, 16, 2)
    assert t.shape == (16, 2) and t.min() >= 0 and t.max() < synth.TINY.vocab


def test_quantised_matrix_layouts():
    S = synth.TINY
    m8 = synth.make_matrix(S, 2, "m", "wq", synth.WDTYPE_INT8, "cpu")
    assert m8["w"].shape == (512, 512) and m8["w"].dtype == torch.int8 and m8["s"].shape == (512,)
    m4 = synth.make_matrix(S, 2, "m", "wq", synth.WDTYPE_INT4, "cpu")
    assert m4["w"].shape == (512, 256) and m4["w"].dtype == torch.uint8
    assert m4["s"].shape == (512, 4) and m4["z"].shape == (512, 4)
    z = m4["z"].float()
    assert torch.equal(z, z.round()) and z.min() >= 0 and z.max() <= 15


def test_byte_model_matches_the_published_roofline_inputs():
    # 8B bf16: parameters read per step (layers + LM head) x 2 bytes, plus norm gains
    S = synth.LLAMA_8B
    params = S.n_layers * S.params_per_layer() + S.vocab * S.d_model
    assert params == 7504658432
    assert synth.weight_bytes_per_step(S, synth.WDTYPE_BF16) == 2 * params + 2 * (2 * S.n_layers + 1) * S.d_model
    assert synth.kv_bytes_per_step(S, 1, 1024) == 32 * 4096 * 1024
