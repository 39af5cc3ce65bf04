"""The allocation-free entry point (ff_decode_step_static: exchange scratch in a static device
array inside the library) against ff_decode_step, through the C ABI, on two calls in a row, the
second with a smaller input."""
import numpy as np
import pytest
import torch

from paper_2505_22758_amd import synth
from tests import helpers

pytestmark = pytest.mark.gpu


def test_static_scratch_step_equals_the_workspace_step_twice_in_a_row():
    from paper_2505_22758_amd import binding
    S, seed = synth.TINY, 0x5ca7
    # first call: batch 4 on a 40-row context; second call: a smaller input (batch 2, other model
    # instance of another weight type, shorter context) on the same static array
    calls = [(synth.WDTYPE_BF16, 4, 40), (synth.WDTYPE_INT8, 2, 9)]
    shapes = {synth.WDTYPE_BF16: S, synth.WDTYPE_INT8: S.replace(d_ffn=1408)}
    models = {}
    for wd, B, T0 in calls:
        models[wd] = helpers.hip_side(shapes[wd], seed, wd, B, T0, max_ctx=T0 + 4, n_caches=2)
    for rep in range(2):   # the pair of calls twice: the second pair starts from the first pair's leftovers
        for wd, B, T0 in calls:
            dec, caches = models[wd]
            shape = shapes[wd]
            tok = synth.make_tokens(shape, seed + rep, 1, B)[0].to("cuda:0")
            pos = torch.full((B,), T0 + rep, dtype=torch.int32, device="cuda:0")
            want = torch.zeros(B, shape.vocab, device="cuda:0")
            got = torch.full_like(want, -3.0)
            binding.ff_decode_step(dec.model, tok, pos, caches[0][0], want, B)
            binding.ff_decode_step_static(dec.model, tok, pos, caches[1][0], got, B)
            binding.ff_status(dec.model)
            # same kernels, same arithmetic, same order: identical bits
            assert torch.equal(got, want), (rep, wd, B, float((got - want).abs().max()))
            assert torch.equal(caches[0][1], caches[1][1]), "appended cache rows differ"
    # a configuration whose exchange scratch exceeds the static array is rejected, not truncated
    big = synth.LLAMA_8B.replace(n_layers=1, vocab=1024)
    dec = binding.Decoder(big, synth.WDTYPE_BF16, max_batch=4)
    dec.load_layer(0, synth.make_layer(big, 1, 0, synth.WDTYPE_BF16, "cuda:0"))
    dec.load_head(synth.make_head(big, 1, synth.WDTYPE_BF16, "cuda:0"))
    dec.alloc_kv(4, 8)
    tok = torch.zeros(4, dtype=torch.int32, device="cuda:0")
    lg = torch.zeros(4, big.vocab, device="cuda:0")
    with pytest.raises(binding.FFError) as e:
        binding.ff_decode_step_static(dec.model, tok, tok, dec.kv, lg, 4)
    assert e.value.code == binding.FF_ERR_NOMEM
    dec.close()
    for dec, _ in models.values():
        dec.close()
