"""CPU-side checks of the boundary: the shared library loads without a GPU, exports every entry
point the header declares, and validates arguments before touching the device."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "flashformer.h")


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ff_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_boundary_named_by_the_benchmark():
    names = _declared_functions()
    for required in ("ff_model_load", "ff_kv_alloc", "ff_decode_step", "ff_decode_step_perop", "ff_debug_dequant"):
        assert required in names


def test_library_exports_every_declared_symbol():
    from paper_2505_22758_amd import binding
    lib = C.CDLL(binding.LIB_PATH)
    for name in _declared_functions():
        assert hasattr(lib, name), f"{name} declared in flashformer.h but not exported"
    assert set(binding.EXPORTS) == set(_declared_functions())


def test_argument_validation_needs_no_device():
    from paper_2505_22758_amd import binding, synth
    cfg = binding.make_config(synth.TINY)
    pb, sb = binding.ff_model_bytes(cfg)
    # packed bytes cover at least every parameter once
    assert pb >= 2 * (synth.TINY.n_layers * synth.TINY.params_per_layer() + 2 * synth.TINY.vocab * synth.TINY.d_model)
    assert sb > 0
    bad = binding.make_config(synth.TINY.replace(head_dim=96))
    with pytest.raises(binding.FFError) as e:
        binding.ff_model_bytes(bad)
    assert e.value.code == binding.FF_ERR_UNSUPPORTED
    bad = binding.make_config(synth.TINY, max_batch=17)
    with pytest.raises(binding.FFError) as e:
        binding.ff_model_bytes(bad)
    assert e.value.code == binding.FF_ERR_ARG
    bad = binding.make_config(synth.TINY, wdtype=binding.FF_W_INT4_G128)   # d_ffn 1376 is not a multiple of 128
    with pytest.raises(binding.FFError) as e:
        binding.ff_model_bytes(bad)
    assert e.value.code == binding.FF_ERR_UNSUPPORTED
    # a normalised input row wider than one staging pass is only supported one sequence at a time
    wide = synth.LLAMA_70B.replace(d_model=16384, n_q_heads=128, n_kv_heads=16)
    binding.ff_model_bytes(binding.make_config(wide, max_batch=1))
    with pytest.raises(binding.FFError) as e:
        binding.ff_model_bytes(binding.make_config(wide, max_batch=2))
    assert e.value.code == binding.FF_ERR_UNSUPPORTED
    # null handles are rejected, not dereferenced
    assert binding._lib.ff_decode_step(None, None, None, None, None, 1, None) == binding.FF_ERR_ARG
    assert binding._lib.ff_kv_bytes(None, 1, 16, None) == binding.FF_ERR_ARG
    assert b"null" in binding._lib.ff_last_error()


def test_quantised_packed_size_follows_the_byte_model():
    from paper_2505_22758_amd import binding, synth
    S = synth.LLAMA_8B
    for wd in (0, 1, 2):
        pb, _ = binding.ff_model_bytes(binding.make_config(S, wdtype=wd))
        per_step = synth.weight_bytes_per_step(S, wd)
        embed = S.vocab * S.d_model * 2
        # packed = weights read per step + the embedding table + alignment padding
        assert per_step + embed <= pb <= per_step + embed + (1 << 20)
