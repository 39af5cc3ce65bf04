"""GPU parity: the HIP decode step (fused whole-model kernel and per-op baseline, both through
the C ABI) against the CPU oracle, element by element, on the same seeded inputs."""
import numpy as np
import pytest
import torch

from paper_2505_22758_amd import synth
from tests import helpers

pytestmark = pytest.mark.gpu


def _run_teacher_forced(shape, seed, wdtype, batch, T0, steps, check_kv=True, gpu_generated=False, quant_lm_head=True):
    from paper_2505_22758_amd import binding
    from oracle import oracle
    T0s = helpers.prefill_lengths(T0, batch)   # one prefill length for all sequences, or one each
    max_ctx = max(T0s) + steps + 3
    if gpu_generated:
        M, okv, dec, caches = helpers.both_sides_gpu_generated(shape, seed, wdtype, batch, T0, max_ctx, n_caches=2, quant_lm_head=quant_lm_head)
    else:
        M, okv = helpers.oracle_side(shape, seed, wdtype, batch, T0, max_ctx, quant_lm_head=quant_lm_head)
        dec, caches = helpers.hip_side(shape, seed, wdtype, batch, T0, max_ctx, n_caches=2, quant_lm_head=quant_lm_head)
    toks = synth.make_tokens(shape, seed, steps, batch)
    logits_f = torch.zeros(batch, shape.vocab, dtype=torch.float32, device="cuda:0")
    logits_p = torch.zeros_like(logits_f)
    worst = {"fused": [0.0, 0.0], "perop": [0.0, 0.0]}
    agree = {"fused": [], "perop": []}
    for s in range(steps):
        pos = np.array([t + s for t in T0s], dtype=np.int32)
        ref = M.decode_step(toks[s].numpy(), pos, okv)
        tok_d = toks[s].to("cuda:0")
        pos_d = torch.from_numpy(pos).to("cuda:0")
        binding.ff_decode_step(dec.model, tok_d, pos_d, caches[0][0], logits_f, batch)
        binding.ff_decode_step_perop(dec.model, tok_d, pos_d, caches[1][0], logits_p, batch)
        binding.ff_status(dec.model)
        for name, lg in (("fused", logits_f), ("perop", logits_p)):
            ma, rl, same = helpers.compare_logits(lg.cpu().numpy(), ref)
            worst[name][0] = max(worst[name][0], ma)
            worst[name][1] = max(worst[name][1], rl)
            agree[name].extend(same.tolist())
    print(f"\n[{shape.name} wd={wdtype} B={batch} T0={T0} steps={steps}] worst (max_abs, rel_l2): {worst}")
    for name in ("fused", "perop"):
        assert worst[name][0] <= helpers.MAX_ABS_TOL, (name, worst)
        assert worst[name][1] <= helpers.REL_L2_TOL, (name, worst)
        assert np.mean(agree[name]) >= helpers.ARGMAX_MIN_AGREE, (name, np.mean(agree[name]))
    if check_kv:
        # rows appended by the kernel: bf16 bits equal to the oracle's except for rare 1-ulp flips
        # (the two sides round values that differ by summation order)
        for ci in range(2):
            mism = tot = 0
            for l in range(shape.n_layers):
                for b in range(batch):
                    k = torch.empty(steps, shape.n_kv_heads, shape.head_dim, dtype=torch.bfloat16, device="cuda:0")
                    v = torch.empty_like(k)
                    binding.ff_kv_read(caches[ci][0], l, b, T0s[b], k, v)
                    for kv_i, t in ((0, k), (1, v)):
                        got = t.cpu().view(torch.int16).numpy().view(np.uint16)
                        want = okv[l, b, kv_i, T0s[b]:T0s[b] + steps]
                        gv, wv = oracle.bf16_bits_to_f64(got), oracle.bf16_bits_to_f64(want)
                        ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(wv), 1e-30))) - 7)
                        # One bf16 step: the two sides round values that differ by summation order, so a
                        # value near a rounding boundary may land on either neighbour.  Once one stored
                        # element has flipped, every later layer sees a slightly different input, and so
                        # do the values it stores; that perturbation is of the size of the step's logit
                        # error, which bounds the extra slack.
                        slack = 1e-4 + 2.0 * max(worst["fused"][0], worst["perop"][0])
                        excess = float(np.max(np.abs(gv - wv) - (ulp + slack)))
                        assert excess <= 0, f"appended cache row off by more than one bf16 step (layer {l}, seq {b}, kv {kv_i}, excess {excess:.3e})"
                        mism += int((got != want).sum())
                        tot += got.size
            # exact bit equality is the rule; after an upstream flip (see above) a sequence's later rows
            # differ in their last bit more often, hence the loose count bound
            assert mism <= max(2, tot * 3 // 10), (mism, tot)
    dec.close()
    return worst


def test_generators_are_bit_identical_on_cpu_and_gpu():
    a = synth.normal_bf16(11, "w", (300, 512), 0.02, "cpu")
    b = synth.normal_bf16(11, "w", (300, 512), 0.02, "cuda:0").cpu()
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    for wd in (synth.WDTYPE_INT8, synth.WDTYPE_INT4):
        ma = synth.make_matrix(synth.TINY, 3, "m", "wq", wd, "cpu")
        mb = synth.make_matrix(synth.TINY, 3, "m", "wq", wd, "cuda:0")
        for key in ma:
            assert torch.equal(ma[key].view(torch.uint8) if ma[key].dtype == torch.int8 else ma[key].view(torch.int16) if ma[key].dtype == torch.float16 else ma[key],
                               (mb[key].cpu().view(torch.uint8) if mb[key].dtype == torch.int8 else mb[key].cpu().view(torch.int16) if mb[key].dtype == torch.float16 else mb[key].cpu()))


def test_tiny_bf16_batch1_teacher_forced_16_steps():
    """The small benchmark configuration: 4 layers, d 512, 8q/2kv heads, ctx 128, 16 steps."""
    _run_teacher_forced(synth.TINY, 0x2505, synth.WDTYPE_BF16, batch=1, T0=128, steps=16)


def test_tiny_bf16_empty_cache_and_ragged_lengths():
    # T0 = 0: first step attends only to itself; lengths that are not multiples of a wave's rows
    _run_teacher_forced(synth.TINY, 7, synth.WDTYPE_BF16, batch=1, T0=0, steps=5)
    _run_teacher_forced(synth.TINY, 8, synth.WDTYPE_BF16, batch=1, T0=77, steps=3)
    _run_teacher_forced(synth.TINY, 9, synth.WDTYPE_BF16, batch=1, T0=1031, steps=2)


def test_tiny_bf16_batches_2_3_4():
    for b in (2, 3, 4):
        _run_teacher_forced(synth.TINY, 20 + b, synth.WDTYPE_BF16, batch=b, T0=40, steps=3)


def test_sequences_of_different_lengths_in_one_batch():
    """Every sequence has its own position (the number of splits follows each sequence's length):
    empty, shorter than one split, ragged and long caches side by side; then the 8B shape."""
    _run_teacher_forced(synth.TINY, 71, synth.WDTYPE_BF16, batch=4, T0=[0, 5, 77, 300], steps=3)
    _run_teacher_forced(synth.TINY, 72, synth.WDTYPE_BF16, batch=7, T0=[1, 0, 130, 64, 63, 65, 9], steps=2)
    _run_teacher_forced(synth.LLAMA_8B, 0x250522766, synth.WDTYPE_BF16, batch=4, T0=[1024, 1000, 7, 2048], steps=1, gpu_generated=True)


def test_tiny_batches_above_one_pass():
    """Batches 5..16: with bf16 weights one pass serves up to eight sequences (5, 7, 8 in one pass,
    16 in two), with int8 weights four (6 = a full and a ragged pass)."""
    for b in (5, 7, 8, 16):
        _run_teacher_forced(synth.TINY, 40 + b, synth.WDTYPE_BF16, batch=b, T0=24, steps=2)
    _run_teacher_forced(synth.TINY.replace(d_ffn=1408), 61, synth.WDTYPE_INT8, batch=6, T0=24, steps=2)


def test_llama8b_bf16_batch1_ctx1024_full_size():
    """The benchmark workload at full size (32 layers, d 4096, vocab 128256, ctx 1024), in the
    launch configuration bench.py times; every logit of three teacher-forced steps is compared."""
    _run_teacher_forced(synth.LLAMA_8B, 0x250522758, synth.WDTYPE_BF16, batch=1, T0=1024, steps=3, gpu_generated=True)


def test_int8_and_int4_dequantised_weights_are_bit_exact():
    """ff_debug_dequant (packed copy, kernel arithmetic) against the oracle's dequantised matrices."""
    from paper_2505_22758_amd import binding
    from oracle import oracle
    S = synth.TINY.replace(n_layers=2, d_ffn=1408)   # int4 groups need K % 128 == 0
    for wd in (synth.WDTYPE_BF16, synth.WDTYPE_INT8, synth.WDTYPE_INT4):
        dec = binding.Decoder(S, wd, max_batch=1)
        layers = [synth.make_layer(S, 31, l, wd, "cuda:0") for l in range(S.n_layers)]
        head = synth.make_head(S, 31, wd, "cuda:0")
        for l, lw in enumerate(layers):
            dec.load_layer(l, lw)
        dec.load_head(head)
        for l in (0, 1):
            for which in synth.LAYER_MATS:
                n, k = synth.mat_shape(S, which)
                out = torch.empty(n, k, dtype=torch.float32, device="cuda:0")
                binding.ff_debug_dequant(dec.model, l, which, out)
                ref = oracle.dequant_matrix({kk: v.cpu() for kk, v in layers[l][which].items()})
                assert np.array_equal(out.cpu().numpy().view(np.uint32), ref.view(np.uint32)), (wd, l, which)
        out = torch.empty(S.vocab, S.d_model, dtype=torch.float32, device="cuda:0")
        binding.ff_debug_dequant(dec.model, 0, "lm_head", out)
        ref = oracle.dequant_matrix({kk: v.cpu() for kk, v in head["lm_head"].items()})
        assert np.array_equal(out.cpu().numpy().view(np.uint32), ref.view(np.uint32)), (wd, "lm_head")
        dec.close()


def test_tiny_shaped_int8_and_int4_steps():
    S = synth.TINY.replace(d_ffn=1408)
    for wd in (synth.WDTYPE_INT8, synth.WDTYPE_INT4):
        _run_teacher_forced(S, 40 + wd, wd, batch=1, T0=70, steps=4)
        _run_teacher_forced(S, 50 + wd, wd, batch=4, T0=33, steps=2)
        _run_teacher_forced(S, 60 + wd, wd, batch=2, T0=21, steps=2)
        _run_teacher_forced(S, 70 + wd, wd, batch=3, T0=45, steps=2)


def test_quantised_layers_with_a_bf16_lm_head():
    """quant_lm_head = 0: the LM head keeps bf16 weights while the layers are int8 / int4, so it
    runs as separate launches behind the fused kernel (final residual sum, norm, projection)."""
    S = synth.TINY.replace(d_ffn=1408)
    _run_teacher_forced(S, 81, synth.WDTYPE_INT8, batch=1, T0=40, steps=3, quant_lm_head=False)
    _run_teacher_forced(S, 82, synth.WDTYPE_INT4, batch=3, T0=25, steps=2, quant_lm_head=False)
    _run_teacher_forced(S, 83, synth.WDTYPE_INT8, batch=6, T0=10, steps=2, quant_lm_head=False)


def test_model_load_in_one_call_and_partial_cache_fills():
    """ff_model_load (create + every layer + head in one call) gives the same model as the
    layer-by-layer calls; a cache filled in two pieces (rows [0, 17) and [17, 30)) equals one
    filled at once: logits bit-identical."""
    from paper_2505_22758_amd import binding
    S, seed, T0 = synth.TINY, 9, 30
    dec, caches = helpers.hip_side(S, seed, synth.WDTYPE_INT8, 1, T0, max_ctx=40)
    cfg = binding.make_config(S, synth.WDTYPE_INT8, 1)
    pb, sb = binding.ff_model_bytes(cfg)
    packed = torch.empty(pb, dtype=torch.uint8, device="cuda:0")
    scratch = torch.empty(sb, dtype=torch.uint8, device="cuda:0")
    layers = [synth.make_layer(S, seed, l, synth.WDTYPE_INT8, "cuda:0") for l in range(S.n_layers)]
    head = synth.make_head(S, seed, synth.WDTYPE_INT8, "cuda:0")
    model = binding.ff_model_load(cfg, layers, head, packed, scratch)
    kvbuf = torch.zeros(binding.ff_kv_bytes(model, 1, 40), dtype=torch.uint8, device="cuda:0")
    kv = binding.ff_kv_alloc(model, 1, 40, kvbuf)
    for l in range(S.n_layers):
        k, v = synth.make_kv_prefill(S, seed, l, 0, T0, "cuda:0")
        binding.ff_kv_fill(kv, l, 0, 0, k[:17].contiguous(), v[:17].contiguous())
        binding.ff_kv_fill(kv, l, 0, 17, k[17:].contiguous(), v[17:].contiguous())
    tok = torch.tensor([7], dtype=torch.int32, device="cuda:0")
    pos = torch.tensor([T0], dtype=torch.int32, device="cuda:0")
    a = torch.zeros(1, S.vocab, device="cuda:0")
    b = torch.zeros(1, S.vocab, device="cuda:0")
    binding.ff_decode_step(dec.model, tok, pos, caches[0][0], a, 1)
    binding.ff_decode_step(model, tok, pos, kv, b, 1)
    torch.cuda.synchronize()
    binding.ff_status(dec.model)
    binding.ff_status(model)
    assert torch.equal(a, b)
    binding.ff_kv_free(kv)
    binding.ff_model_free(model)


def test_timeline_buffer_of_the_documented_size():
    """ff_debug_timeline with a buffer of exactly the size the header states: stamps arrive in order
    (input staged before the projection is done, phase after phase) and nothing is written behind
    the buffer; ff_fused_schedule reports the launch shape the layout depends on."""
    from paper_2505_22758_amd import binding
    S = synth.TINY
    dec, caches = helpers.hip_side(S, 5, synth.WDTYPE_BF16, 2, 30, max_ctx=40)
    barriers, W, threads = binding.ff_fused_schedule(dec.model)
    assert barriers == 0 and W > 0 and threads == 256
    P = 4 * S.n_layers + 1
    n = 12 * P + 72 * W
    guard = 64
    buf = torch.full((n + guard,), -1, dtype=torch.int64, device="cuda:0")
    buf[:n] = 0
    tok = torch.tensor([3, 4], dtype=torch.int32, device="cuda:0")
    pos = torch.tensor([30, 30], dtype=torch.int32, device="cuda:0")
    lg = torch.zeros(2, S.vocab, device="cuda:0")
    binding.ff_debug_timeline(dec.model, buf)
    binding.ff_decode_step(dec.model, tok, pos, caches[0][0], lg, 2)
    torch.cuda.synchronize()
    binding.ff_debug_timeline(dec.model, None)
    binding.ff_status(dec.model)
    h = buf.cpu().numpy()
    assert (h[n:] == -1).all()
    t = h[:12 * P].reshape(P, 12)
    staged, done = t[:, 0], t[:, 1]
    assert (staged > 0).all() and (done > staged).all() and (staged[1:] > done[:-1]).all()
    # stamps off: a further step leaves the buffer alone
    before = buf.clone()
    binding.ff_decode_step(dec.model, tok, pos + 1, caches[0][0], lg, 2)
    torch.cuda.synchronize()
    assert torch.equal(before, buf)


def test_out_of_range_position_is_reported_and_skipped():
    from paper_2505_22758_amd import binding
    S = synth.TINY
    dec, caches = helpers.hip_side(S, 3, synth.WDTYPE_BF16, 1, 4, max_ctx=8)
    tok = torch.tensor([1], dtype=torch.int32, device="cuda:0")
    logits = torch.zeros(1, S.vocab, dtype=torch.float32, device="cuda:0")
    for fn in (binding.ff_decode_step, binding.ff_decode_step_perop):
        pos = torch.tensor([8], dtype=torch.int32, device="cuda:0")     # == max_ctx
        fn(dec.model, tok, pos, caches[0][0], logits, 1)
        with pytest.raises(binding.FFError) as e:
            binding.ff_status(dec.model)
        assert e.value.code == binding.FF_ERR_RANGE
        bad_tok = torch.tensor([S.vocab], dtype=torch.int32, device="cuda:0")
        fn(dec.model, bad_tok, torch.tensor([4], dtype=torch.int32, device="cuda:0"), caches[0][0], logits, 1)
        with pytest.raises(binding.FFError):
            binding.ff_status(dec.model)
    # the model is still usable afterwards
    binding.ff_decode_step(dec.model, tok, torch.tensor([4], dtype=torch.int32, device="cuda:0"), caches[0][0], logits, 1)
    binding.ff_status(dec.model)
    assert torch.isfinite(logits).all()
    dec.close()


def test_llama8b_int8_ctx4096_and_int4_ctx2048_full_size():
    """The quantised benchmark configurations at full size: 8B int8 (batch 1, context 4096) and
    8B int4 group-128 (batch 1 and batch 4, context 2048); every logit compared."""
    _run_teacher_forced(synth.LLAMA_8B, 0x250522760, synth.WDTYPE_INT8, batch=1, T0=4096, steps=2, gpu_generated=True)
    _run_teacher_forced(synth.LLAMA_8B, 0x250522761, synth.WDTYPE_INT4, batch=1, T0=2048, steps=2, gpu_generated=True)
    _run_teacher_forced(synth.LLAMA_8B, 0x250522762, synth.WDTYPE_INT4, batch=4, T0=2048, steps=1, gpu_generated=True)


def test_llama70b_shaped_layers_batch1_ctx2048():
    """Width, head geometry (64 query / 8 kv heads) and vocabulary of the 70B configuration with
    two of its 80 layers (the oracle needs the whole model in host memory and ~2 flop per
    parameter per step): exercises the d_model 8192 / d_ffn 28672 / 8-queries-per-kv-head instances."""
    _run_teacher_forced(synth.LLAMA_70B.replace(n_layers=2), 0x250522763, synth.WDTYPE_BF16, batch=1, T0=2048, steps=2, gpu_generated=True)
    _run_teacher_forced(synth.LLAMA_70B.replace(n_layers=2), 0x250522764, synth.WDTYPE_BF16, batch=2, T0=300, steps=1, gpu_generated=True)


def test_llama70b_shaped_one_layer_batch16():
    """Batch 16 at the 70B width (one layer, short context so that the oracle finishes in seconds)."""
    _run_teacher_forced(synth.LLAMA_70B.replace(n_layers=1), 0x250522765, synth.WDTYPE_BF16, batch=16, T0=64, steps=1, gpu_generated=True)


def test_llama8b_shaped_one_layer_batch8_single_pass():
    """Eight sequences in ONE pass at the 8B width (one layer): the matrix-core projections with two
    sets of four sequences, input rows staged in two groups, the down projection cut into four
    segments along K, sequences of different lengths."""
    _run_teacher_forced(synth.LLAMA_8B.replace(n_layers=1), 0x250522766, synth.WDTYPE_BF16, batch=8, T0=[96, 1, 300, 64, 63, 65, 0, 200], steps=2,
                        gpu_generated=True)


def test_llama8b_shaped_one_layer_quantised_batches():
    """The matrix-core projections for int8 and int4 weights at the 8B width (one layer): the down
    projection's 14336-column input staged in one long pass (batch 2) and in two K segments
    (batch 4), several chunks per row group."""
    S = synth.LLAMA_8B.replace(n_layers=1)
    _run_teacher_forced(S, 0x250522767, synth.WDTYPE_INT8, batch=2, T0=80, steps=1, gpu_generated=True)
    _run_teacher_forced(S, 0x250522768, synth.WDTYPE_INT8, batch=4, T0=70, steps=1, gpu_generated=True)
    _run_teacher_forced(S, 0x250522769, synth.WDTYPE_INT4, batch=2, T0=90, steps=1, gpu_generated=True)


def test_wide_model_staged_in_several_passes():
    """d_model 16384 (one layer, batch 1): the normalised input rows no longer fit one staging pass
    of eight quads per thread, so the embedding, the residual sum and the final norm go through
    the several-pass staging with its separate rescaling step."""
    S = synth.TINY.replace(name="wide", n_layers=1, d_model=16384, n_q_heads=8, n_kv_heads=2, head_dim=128, d_ffn=2048, vocab=1000)
    _run_teacher_forced(S, 0x25052276a, synth.WDTYPE_BF16, batch=1, T0=40, steps=2, gpu_generated=True)


def test_eight_query_heads_per_kv_head_small_model_all_formats():
    """The (head_dim 128, 8 query heads per kv head) kernel family on a small model, in the batch
    classes the 70B-shaped tests do not reach: eight sequences in one pass (bf16), and the int8 and
    int4 matrix-core projections at batch 4 and 3."""
    S = synth.TINY.replace(name="g8", n_layers=2, d_model=1024, n_q_heads=8, n_kv_heads=1, head_dim=128, d_ffn=1536, vocab=1500)
    _run_teacher_forced(S, 0x25052276b, synth.WDTYPE_BF16, batch=8, T0=70, steps=2)
    _run_teacher_forced(S, 0x25052276c, synth.WDTYPE_INT8, batch=4, T0=33, steps=2)
    _run_teacher_forced(S, 0x25052276d, synth.WDTYPE_INT4, batch=3, T0=90, steps=2)
    _run_teacher_forced(S, 0x25052276e, synth.WDTYPE_INT4, batch=1, T0=130, steps=2)


def test_half_a_row_group_per_wave():
    """d_model 2048 at batch 2: the output and down projections have 512 four-row groups for the
    1024 waves of the grid, so every wave multiplies half of a group (split along K) and every
    group is finished through the wave pair's mailbox; bf16 and int4."""
    S = synth.TINY.replace(name="half", n_layers=2, d_model=2048, n_q_heads=16, n_kv_heads=4, head_dim=128, d_ffn=2048, vocab=3000)
    _run_teacher_forced(S, 0x25052276f, synth.WDTYPE_BF16, batch=2, T0=50, steps=2)
    _run_teacher_forced(S, 0x250522770, synth.WDTYPE_INT4, batch=4, T0=20, steps=2)


def test_two_models_interleaved_on_a_side_stream():
    """Two models of different geometry (head_dim 64 vs 128, bf16 vs int8) alive at once and stepped
    alternately on a non-default stream: no state is shared between models, and a model's result does
    not depend on what ran in between (compared with a run of the same model alone)."""
    from paper_2505_22758_amd import binding
    shapes = [(synth.TINY, synth.WDTYPE_BF16, 91), (synth.TINY.replace(head_dim=128, n_q_heads=4, n_kv_heads=1, d_ffn=1408), synth.WDTYPE_INT8, 92)]
    T0, steps = 50, 3

    def setup(shape, wd, seed):
        dec, caches = helpers.hip_side(shape, seed, wd, 1, T0, T0 + steps + 2, n_caches=1)
        toks = synth.make_tokens(shape, seed, steps, 1).to("cuda:0")
        return dec, caches[0][0], caches, toks, torch.zeros(1, shape.vocab, device="cuda:0")

    def run(models, stream):
        outs = [[] for _ in models]
        with torch.cuda.stream(stream):
            for s in range(steps):
                for i, (dec, kv, _, toks, lg) in enumerate(models):
                    pos = torch.tensor([T0 + s], dtype=torch.int32, device="cuda:0")
                    binding.ff_decode_step(dec.model, toks[s], pos, kv, lg, 1)
                    stream.synchronize()
                    binding.ff_status(dec.model)
                    outs[i].append(lg.cpu().clone())
        return outs

    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    both = [setup(*a) for a in shapes]
    together = run(both, side)
    for i, a in enumerate(shapes):
        alone = run([setup(*a)], torch.cuda.current_stream())[0]
        for s in range(steps):
            assert torch.equal(alone[s], together[i][s]), (i, s)
    for m in both:
        m[0].close()


def test_batch_size_changing_from_step_to_step():
    """Steps of different batch sizes on one model and one cache: a sequence that sits out some steps
    (among them exactly as many as make the exchange vectors' 4-bit write counters come round again:
    with 4 layers, 4 steps) must not be served values its exchange rows kept from its last step."""
    from paper_2505_22758_amd import binding
    from oracle import oracle
    shape, seed, T0 = synth.TINY, 0x77, 20
    sizes = [4, 1, 1, 1, 1, 4, 2, 2, 2, 2, 3, 1, 4, 4, 1, 1, 1, 1, 1, 1, 1, 1, 2]
    max_ctx = T0 + len(sizes) + 2
    layers = [synth.make_layer(shape, seed, l, synth.WDTYPE_BF16, "cpu") for l in range(shape.n_layers)]
    M = oracle.OracleModel(shape, layers, synth.make_head(shape, seed, synth.WDTYPE_BF16, "cpu"))
    okv = []
    for b in range(4):
        kv = M.new_kv(1, max_ctx)
        for l in range(shape.n_layers):
            k, v = synth.make_kv_prefill(shape, seed, l, b, T0, "cpu")
            kv[l, 0, 0, :T0], kv[l, 0, 1, :T0] = oracle._np(k), oracle._np(v)
        okv.append(kv)
    dec, caches = helpers.hip_side(shape, seed, synth.WDTYPE_BF16, 4, T0, max_ctx, n_caches=1)
    toks = synth.make_tokens(shape, seed, len(sizes), 4)
    pos = [T0] * 4
    logits = torch.zeros(4, shape.vocab, dtype=torch.float32, device="cuda:0")
    for s, b in enumerate(sizes):
        tok_d = toks[s, :b].contiguous().to("cuda:0")
        pos_d = torch.tensor(pos[:b], dtype=torch.int32, device="cuda:0")
        binding.ff_decode_step(dec.model, tok_d, pos_d, caches[0][0], logits, b)
        binding.ff_status(dec.model)
        got = logits[:b].cpu().numpy()
        for r in range(b):
            ref = M.decode_step(toks[s, r:r + 1].numpy(), np.array([pos[r]], dtype=np.int32), okv[r])
            ma, rl, same = helpers.compare_logits(got[r:r + 1], ref)
            assert ma <= helpers.MAX_ABS_TOL and rl <= helpers.REL_L2_TOL and same.all(), (s, b, r, ma, rl)
            pos[r] += 1
    dec.close()
