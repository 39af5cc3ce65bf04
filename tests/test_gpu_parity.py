"""GPU parity: the HIP decode step (fused whole-model kernel and per-op baseline, both through
the C ABI) against the CPU oracle, element by element, on the same seeded inputs."""
import numpy as np
import pytest
import torch

from paper_2505_22758_amd import synth
from tests import helpers

pytestmark = pytest.mark.gpu


def _progress(capsys, msg):
    """A line on the real stdout (pytest captures the test's own): long tests say that they are alive."""
    if capsys is None:
        print(msg, flush=True)
    else:
        with capsys.disabled():
            print(msg, flush=True)


def _step_stats(stats, name, s, got, ref):
    """Per-sequence error figures of one step: max-abs, relative L2, arg-max agreement, and for a
    disagreeing arg-max the oracle's gap between its two largest logits."""
    got = got.astype(np.float64)
    for b in range(got.shape[0]):
        d = got[b] - ref[b]
        ma, rl = float(np.max(np.abs(d))), float(np.linalg.norm(d) / np.linalg.norm(ref[b]))
        same = int(got[b].argmax()) == int(ref[b].argmax())
        st = stats[name].setdefault(b, {"max_abs": 0.0, "rel_l2": 0.0, "agree": []})
        st["max_abs"], st["rel_l2"] = max(st["max_abs"], ma), max(st["rel_l2"], rl)
        st["agree"].append(same)
        if not same:
            top2 = np.partition(ref[b], -2)[-2:]
            print(f"  arg-max differs ({name}, step {s}, sequence {b}): oracle top-1/top-2 gap {abs(top2[1] - top2[0]):.3e}, max_abs {ma:.3e}")


def _check_stats(stats, tag):
    worst = {}
    for name, per_seq in stats.items():
        agree = [a for st in per_seq.values() for a in st["agree"]]
        worst[name] = (max(st["max_abs"] for st in per_seq.values()), max(st["rel_l2"] for st in per_seq.values()))
        print(f"[{tag}] {name}: " + " | ".join(f"seq {b}: max_abs {st['max_abs']:.2e} rel_l2 {st['rel_l2']:.2e}" for b, st in sorted(per_seq.items()))
              + f" | arg-max equal on {sum(agree)}/{len(agree)} decisions")
        assert worst[name][0] <= helpers.MAX_ABS_TOL, (name, worst)
        assert worst[name][1] <= helpers.REL_L2_TOL, (name, worst)
        assert np.mean(agree) >= helpers.ARGMAX_MIN_AGREE, (name, np.mean(agree), len(agree))
    return worst


def _check_appended_rows(got_bits, want_bits):
    """Rows appended by the kernels against the oracle's bf16 bits: (differing words, words, largest
    distance beyond one bf16 step of the oracle's value)."""
    gv, wv = oracle_bits_to_f64(got_bits), oracle_bits_to_f64(want_bits)
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(wv), 1e-30))) - 7)
    return int((got_bits != want_bits).sum()), got_bits.size, float(np.max(np.abs(gv - wv) - ulp))


def _check_appended_cache(read_rows, okv_rows, n_layers, batch, seq_stats, tag):
    """read_rows(l, b) -> (k bits, v bits) of the kernel's appended rows; okv_rows(l, b, kv) -> the
    oracle's.  Both sides round a projection output to bf16 whose unrounded values differ by the
    summation order and -- once an earlier stored element has landed on the other neighbour -- by
    that flip's propagated effect, which also shows in the sequence's logits.  Per sequence, with
    e = its largest logit error and r = its largest relative L2 logit error over the run:
      every element within one bf16 step + KV_ABS_SLACK + KV_SLACK_PER_LOGIT_ERR * e;
      fraction of differing words <= KV_RATE_FLOOR + KV_RATE_PER_REL_ERR * r
    (a word flips when the unrounded difference, of relative size about r, straddles a rounding
    boundary: probability about r / 2^-8).  The constants are a few times the measured figures."""
    rates, excesses = [], []
    for b in range(batch):
        mism = tot = 0
        exc = -1.0
        for l in range(n_layers):
            k, v = read_rows(l, b)
            for kv_i, got in ((0, k), (1, v)):
                m_, t_, e_ = _check_appended_rows(got, okv_rows(l, b, kv_i))
                mism, tot, exc = mism + m_, tot + t_, max(exc, e_)
        rates.append(mism / max(tot, 1))
        excesses.append(exc)
    print(f"[{tag}] appended cache rows per sequence: differing words " + " ".join(f"{r:.2e}" for r in rates)
          + " | rate / rel_l2 " + " ".join(f"{r / max(seq_stats[b]['rel_l2'], 1e-12):.0f}" for b, r in enumerate(rates))
          + " | beyond one bf16 step / logit max_abs " + " ".join(f"{max(e, 0) / max(seq_stats[b]['max_abs'], 1e-12):.2f}" for b, e in enumerate(excesses)))
    for b in range(batch):
        assert excesses[b] <= helpers.KV_ABS_SLACK + helpers.KV_SLACK_PER_LOGIT_ERR * seq_stats[b]["max_abs"], (tag, b, excesses[b], seq_stats[b])
        assert rates[b] <= helpers.KV_RATE_FLOOR + helpers.KV_RATE_PER_REL_ERR * seq_stats[b]["rel_l2"], (tag, b, rates[b], seq_stats[b])


def oracle_bits_to_f64(a):
    from oracle import oracle
    return oracle.bf16_bits_to_f64(a)


def _run_teacher_forced(shape, seed, wdtype, batch, T0, steps, check_kv=True, gpu_generated=False, quant_lm_head=True, perop_steps=None,
                        capsys=None, attention_by_length=True):
    """Teacher-forced decoding on both sides; every logit of every step is compared.  perop_steps
    limits how many steps the per-operation path runs as well (it shares no kernels' schedule with
    the fused one; long runs check it on their first steps only)."""
    from paper_2505_22758_amd import binding
    T0s = helpers.prefill_lengths(T0, batch)   # one prefill length for all sequences, or one each
    max_ctx = max(T0s) + steps + 3
    perop_steps = steps if perop_steps is None else perop_steps
    if gpu_generated:
        M, okv, dec, caches = helpers.both_sides_gpu_generated(shape, seed, wdtype, batch, T0, max_ctx, n_caches=2, quant_lm_head=quant_lm_head)
    else:
        M, okv = helpers.oracle_side(shape, seed, wdtype, batch, T0, max_ctx, quant_lm_head=quant_lm_head)
        dec, caches = helpers.hip_side(shape, seed, wdtype, batch, T0, max_ctx, n_caches=2, quant_lm_head=quant_lm_head)
    if not attention_by_length:
        binding.ff_debug_set_attention_balance(dec.model, False)
    toks = synth.make_tokens(shape, seed, steps, batch)
    logits_f = torch.zeros(batch, shape.vocab, dtype=torch.float32, device="cuda:0")
    logits_p = torch.zeros_like(logits_f)
    stats = {"fused": {}, "perop": {}}
    tag = f"{shape.name} L={shape.n_layers} wd={wdtype} B={batch} T0={T0} steps={steps}"
    for s in range(steps):
        pos = np.array([t + s for t in T0s], dtype=np.int32)
        ref = M.decode_step(toks[s].numpy(), pos, okv)
        tok_d = toks[s].to("cuda:0")
        pos_d = torch.from_numpy(pos).to("cuda:0")
        binding.ff_decode_step(dec.model, tok_d, pos_d, caches[0][0], logits_f, batch)
        if s < perop_steps:
            binding.ff_decode_step_perop(dec.model, tok_d, pos_d, caches[1][0], logits_p, batch)
        binding.ff_status(dec.model)
        _step_stats(stats, "fused", s, logits_f.cpu().numpy(), ref)
        if s < perop_steps:
            _step_stats(stats, "perop", s, logits_p.cpu().numpy(), ref)
        if steps > 8 and s % 8 == 7:
            _progress(capsys, f"  [{tag}] step {s + 1}/{steps}")
    print()
    worst = _check_stats(stats, tag)
    if check_kv:
        for ci, n_rows, name in ((0, steps, "fused"), (1, perop_steps, "perop")):
            def read_rows(l, b):
                k = torch.empty(n_rows, shape.n_kv_heads, shape.head_dim, dtype=torch.bfloat16, device="cuda:0")
                v = torch.empty_like(k)
                binding.ff_kv_read(caches[ci][0], l, b, T0s[b], k, v)
                return [t.cpu().view(torch.int16).numpy().view(np.uint16) for t in (k, v)]
            _check_appended_cache(read_rows, lambda l, b, kv_i: okv[l, b, kv_i, T0s[b]:T0s[b] + n_rows], shape.n_layers, batch,
                                  stats[name], f"{tag} {name}")
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


def test_attention_work_list_follows_the_lengths():
    """One long sequence among short ones: the step's attention work list gives it most of the grid
    (16 slices where equal shares allow 8, resp. 2 in the wide pass); both forms of the list against
    the oracle, on a model with 8 kv heads (32 / 96 head groups on 256 workgroups)."""
    S = synth.TINY.replace(name="kv8", n_layers=2, n_q_heads=32, n_kv_heads=8)
    for by_length in (True, False):
        _run_teacher_forced(S, 0x2505227a0, synth.WDTYPE_BF16, batch=4, T0=[2100, 3, 40, 0], steps=2, perop_steps=1, attention_by_length=by_length)
        _run_teacher_forced(S, 0x2505227a1, synth.WDTYPE_BF16, batch=12, T0=[5, 1800] + [6 * i for i in range(10)], steps=2, perop_steps=1,
                            attention_by_length=by_length)


def test_tiny_batches_above_one_pass():
    """Batches 5..16: with bf16 weights one wide pass each (a single K segment at this width, workgroups
    that own one row group or none), with int8 weights passes of four (6 = a full and a ragged pass)."""
    for b in (5, 7, 8, 16):
        _run_teacher_forced(synth.TINY, 40 + b, synth.WDTYPE_BF16, batch=b, T0=24, steps=2)
    _run_teacher_forced(synth.TINY.replace(d_ffn=1408), 61, synth.WDTYPE_INT8, batch=6, T0=24, steps=2)


def test_llama8b_bf16_batch1_ctx1024_full_size(capsys):
    """The benchmark workload at full size (32 layers, d 4096, vocab 128256, ctx 1024), in the
    launch configuration bench.py times; every logit of the configured 64 teacher-forced steps is
    compared (the per-operation path on the first four), and the arg-max rate is a rate over 64
    decisions.  The 2-bit write counters of the exchange vectors come round 512 times."""
    _run_teacher_forced(synth.LLAMA_8B, 0x250522758, synth.WDTYPE_BF16, batch=1, T0=1024, steps=64, gpu_generated=True, perop_steps=4,
                        capsys=capsys)


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


def test_llama8b_int8_ctx4096_and_int4_ctx2048_full_size(capsys):
    """The quantised benchmark configurations at full size: 8B int8 (batch 1, context 4096) and
    8B int4 group-128 (batch 1 and batch 4, context 2048); every logit of 16 steps (batch 4: 4 steps
    = 16 arg-max decisions) compared, the per-operation path on the first two."""
    _run_teacher_forced(synth.LLAMA_8B, 0x250522760, synth.WDTYPE_INT8, batch=1, T0=4096, steps=16, gpu_generated=True, perop_steps=2, capsys=capsys)
    _run_teacher_forced(synth.LLAMA_8B, 0x250522761, synth.WDTYPE_INT4, batch=1, T0=2048, steps=16, gpu_generated=True, perop_steps=2, capsys=capsys)
    _run_teacher_forced(synth.LLAMA_8B, 0x250522762, synth.WDTYPE_INT4, batch=4, T0=2048, steps=4, gpu_generated=True, perop_steps=1, capsys=capsys)


def test_llama70b_shaped_layers_batch1_ctx2048():
    """Width, head geometry (64 query / 8 kv heads) and vocabulary of the 70B configuration with
    two of its 80 layers (the oracle needs the whole model in host memory and ~2 flop per
    parameter per step): exercises the d_model 8192 / d_ffn 28672 / 8-queries-per-kv-head instances."""
    _run_teacher_forced(synth.LLAMA_70B.replace(n_layers=2), 0x250522763, synth.WDTYPE_BF16, batch=1, T0=2048, steps=2, gpu_generated=True)
    _run_teacher_forced(synth.LLAMA_70B.replace(n_layers=2), 0x250522764, synth.WDTYPE_BF16, batch=2, T0=300, steps=1, gpu_generated=True)


def test_llama70b_shaped_one_layer_batch16():
    """Batch 16 at the 70B width (one layer, short context so that the oracle finishes in seconds)."""
    _run_teacher_forced(synth.LLAMA_70B.replace(n_layers=1), 0x250522765, synth.WDTYPE_BF16, batch=16, T0=64, steps=1, gpu_generated=True)


def test_llama70b_shaped_one_layer_int4_and_int8():
    """The quantised formats at the 70B width (one layer; eight query heads per KV head, 8192-column
    rows = 64 int4 groups per row, gate/up rows in the interleaved order), batch 1 and a batch of 3."""
    S = synth.LLAMA_70B.replace(n_layers=1)
    _run_teacher_forced(S, 0x250522767, synth.WDTYPE_INT4, batch=1, T0=300, steps=2, gpu_generated=True)
    _run_teacher_forced(S, 0x250522768, synth.WDTYPE_INT4, batch=3, T0=[64, 0, 130], steps=1, gpu_generated=True)
    _run_teacher_forced(S, 0x250522769, synth.WDTYPE_INT8, batch=1, T0=100, steps=1, gpu_generated=True)


def test_llama8b_shaped_one_layer_batch8_single_pass():
    """Eight sequences in ONE (wide) pass at the 8B width (one layer): one or two tiles of 16 rows per
    workgroup (seven for gate/up), inputs copied in two K segments (seven for the down projection),
    sequences of different lengths."""
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
    classes the 70B-shaped tests do not reach: eight sequences in one wide pass (bf16), and the int8
    and int4 matrix-core projections at batch 4 and 3."""
    S = synth.TINY.replace(name="g8", n_layers=2, d_model=1024, n_q_heads=8, n_kv_heads=1, head_dim=128, d_ffn=1536, vocab=1500)
    _run_teacher_forced(S, 0x25052276b, synth.WDTYPE_BF16, batch=8, T0=70, steps=2)
    # (wide pass, ragged: its attention takes the scores of 16 rows at a time from the matrix cores)
    _run_teacher_forced(S, 0x25052276f, synth.WDTYPE_BF16, batch=6, T0=[0, 1, 15, 17, 333, 640], steps=2)
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


def _run_changing_batches(nseq, sizes, wdtype=synth.WDTYPE_BF16):
    from paper_2505_22758_amd import binding
    from oracle import oracle
    shape, seed, T0 = synth.TINY, 0x77, 20
    max_ctx = T0 + len(sizes) + 2
    layers = [synth.make_layer(shape, seed, l, wdtype, "cpu") for l in range(shape.n_layers)]
    M = oracle.OracleModel(shape, layers, synth.make_head(shape, seed, wdtype, "cpu"))
    okv = []
    for b in range(nseq):
        kv = M.new_kv(1, max_ctx)
        for l in range(shape.n_layers):
            k, v = synth.make_kv_prefill(shape, seed, l, b, T0, "cpu")
            kv[l, 0, 0, :T0], kv[l, 0, 1, :T0] = oracle._np(k), oracle._np(v)
        okv.append(kv)
    dec, caches = helpers.hip_side(shape, seed, wdtype, nseq, T0, max_ctx, n_caches=1)
    toks = synth.make_tokens(shape, seed, len(sizes), nseq)
    pos = [T0] * nseq
    logits = torch.zeros(nseq, shape.vocab, dtype=torch.float32, device="cuda:0")
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


def test_batch_size_changing_from_step_to_step():
    """Steps of different batch sizes on one model and one cache: a sequence that sits out some steps
    (the exchange vectors' 2-bit write counters come round every step of this 4-layer model, so any
    number of skipped steps leaves the counter bits a reader would accept) must not be served values
    its exchange rows kept from its last step."""
    _run_changing_batches(4, [4, 1, 1, 1, 1, 4, 2, 2, 2, 2, 3, 1, 4, 4, 1, 1, 1, 1, 1, 1, 1, 1, 2])


def test_wide_and_row_partitioned_steps_alternate_on_one_model():
    """A model created for 16 sequences stepped with batches on both sides of the wide pass's
    threshold: wide steps leave the compact exchange rows of the other paths untouched (those are
    re-initialised before the next small batch), small steps leave the wide pass's epochs alone."""
    _run_changing_batches(16, [6, 1, 16, 4, 9, 2, 5, 5, 1, 1, 12, 3, 16])
    # int8: the wide pass from four sequences on
    _run_changing_batches(16, [5, 1, 4, 3, 16, 2, 4, 1, 9, 3], wdtype=synth.WDTYPE_INT8)


def _run_sequences_stopping_early(nseq, stops, steps, wdtype=synth.WDTYPE_BF16, quant_lm_head=True, perop=False):
    """Teacher-forced steps of one batch in which sequence b takes part only in steps < stops[b]
    (token FF_TOKEN_SKIP afterwards, with a position the kernels must ignore).  Active sequences are
    compared with the oracle stepped one sequence at a time; a stopped sequence's cache planes and
    logits row must stay bit for bit what they were."""
    from paper_2505_22758_amd import binding
    from oracle import oracle
    shape, seed, T0 = (synth.TINY if wdtype == synth.WDTYPE_BF16 else synth.TINY.replace(d_ffn=1408)), 0x51, 9
    max_ctx = T0 + steps + 1
    layers = [synth.make_layer(shape, seed, l, wdtype, "cpu") for l in range(shape.n_layers)]
    M = oracle.OracleModel(shape, layers, synth.make_head(shape, seed, wdtype, "cpu", quant_lm_head))
    okv = []
    for b in range(nseq):
        kv = M.new_kv(1, max_ctx)
        for l in range(shape.n_layers):
            k, v = synth.make_kv_prefill(shape, seed, l, b, T0, "cpu")
            kv[l, 0, 0, :T0], kv[l, 0, 1, :T0] = oracle._np(k), oracle._np(v)
        okv.append(kv)
    dec, caches = helpers.hip_side(shape, seed, wdtype, nseq, T0, max_ctx, n_caches=2, quant_lm_head=quant_lm_head)
    step_fn = binding.ff_decode_step_perop if perop else binding.ff_decode_step
    n_cache_words = shape.n_layers * nseq * shape.n_kv_heads * 2 * max_ctx * shape.head_dim
    planes = [c[1][:2 * n_cache_words].view(torch.int16).view(shape.n_layers, nseq, -1) for c in caches]   # [layer][sequence][rows of all heads]
    toks = synth.make_tokens(shape, seed, steps, nseq)
    pos = [T0] * nseq
    sentinel = 7.25
    logits = torch.full((nseq, shape.vocab), sentinel, dtype=torch.float32, device="cuda:0")
    # One sequence sitting out does not change the others' results by a bit: the same first step on
    # the second cache with everybody taking part.
    if stops[0] > 0 and min(stops) == 0:
        full = torch.zeros_like(logits)
        step_fn(dec.model, toks[0].contiguous().to("cuda:0"), torch.tensor(pos, dtype=torch.int32, device="cuda:0"), caches[1][0], full, nseq)
        binding.ff_status(dec.model)
    else:
        full = None
    for s in range(steps):
        active = [s < stops[b] for b in range(nseq)]
        tok = toks[s].clone()
        p = torch.tensor(pos, dtype=torch.int32)
        for b in range(nseq):
            if not active[b]:
                tok[b] = binding.FF_TOKEN_SKIP
                p[b] = (-7, 10 ** 6, max_ctx)[(s + b) % 3]   # ignored for a sequence that sits the step out
        frozen = [planes[0][:, b].clone() for b in range(nseq)]
        step_fn(dec.model, tok.contiguous().to("cuda:0"), p.to("cuda:0"), caches[0][0], logits, nseq)
        binding.ff_status(dec.model)
        got = logits.cpu().numpy()
        for b in range(nseq):
            if active[b]:
                ref = M.decode_step(toks[s, b:b + 1].numpy(), np.array([pos[b]], dtype=np.int32), okv[b])
                ma, rl, same = helpers.compare_logits(got[b:b + 1], ref)
                assert ma <= helpers.MAX_ABS_TOL and rl <= helpers.REL_L2_TOL and same.all(), (s, b, ma, rl)
                if s == 0 and full is not None:
                    assert torch.equal(logits[b], full[b]), ("another sequence sitting out changed this one's logits", b)
                pos[b] += 1
                logits[b] = sentinel
            else:
                assert (got[b] == sentinel).all(), ("logits written for a sequence that sat the step out", s, b)
                assert torch.equal(frozen[b], planes[0][:, b]), ("cache touched for a sequence that sat the step out", s, b)
    dec.close()


def test_sequences_that_stop_early_in_a_batch():
    """Early stop inside a batch (beyond the lock-step batches of the paper's Section 5.2): on the
    row-partitioned pass of up to four sequences, the wide pass, consecutive passes with the LM head
    as separate launches, the quantised formats and the per-operation path; also a step in which
    nobody takes part."""
    _run_sequences_stopping_early(4, [6, 0, 3, 6], 6)
    _run_sequences_stopping_early(2, [2, 3], 4)                                   # last step: nobody
    _run_sequences_stopping_early(1, [1], 2)
    _run_sequences_stopping_early(7, [5, 0, 5, 2, 5, 1, 3], 5)                     # one wide pass
    _run_sequences_stopping_early(16, [3] * 5 + [0] + [1] * 9 + [3], 3)
    _run_sequences_stopping_early(6, [4, 0, 2, 4, 1, 4], 4, wdtype=synth.WDTYPE_INT8, quant_lm_head=False)   # passes of four and two, bf16 LM head
    _run_sequences_stopping_early(6, [4, 0, 2, 4, 1, 4], 4, wdtype=synth.WDTYPE_INT8)                        # int8 wide pass
    _run_sequences_stopping_early(3, [3, 0, 1], 3, wdtype=synth.WDTYPE_INT4)
    _run_sequences_stopping_early(5, [3, 0, 1, 3, 2], 3, perop=True)


def test_llama70b_full_depth_batch1_and_batch16_ctx2048(capsys):
    """The 80-layer 70B configuration at full size (139 GB of packed weights): batch 1 for four
    teacher-forced steps and batch 16 for one, context 2048, every logit against the oracle run
    layer-major (see helpers.layer_major_both_sides); appended cache rows of every layer compared."""
    from paper_2505_22758_amd import binding
    shape, seed = synth.LLAMA_70B, 0x250522771
    runs = [{"batch": 1, "T0": 2048, "steps": 4}, {"batch": 16, "T0": 2048, "steps": 1}]
    dec = helpers.layer_major_both_sides(shape, seed, synth.WDTYPE_BF16, runs, lambda m: _progress(capsys, m))
    for r in runs:
        B, S, T0 = r["batch"], r["steps"], r["T0"]
        logits = torch.zeros(B, shape.vocab, dtype=torch.float32, device="cuda:0")
        stats = {"fused": {}}
        for s in range(S):
            pos_d = torch.full((B,), T0 + s, dtype=torch.int32, device="cuda:0")
            binding.ff_decode_step(dec.model, r["toks"][s].to("cuda:0"), pos_d, r["kv"], logits, B)
            binding.ff_status(dec.model)
            _step_stats(stats, "fused", s, logits.cpu().numpy(), r["ref"][s])
        print()
        _check_stats(stats, f"llama3-70b L=80 B={B} T0={T0} steps={S}")
        def read_rows(l, b):
            k = torch.empty(S, shape.n_kv_heads, shape.head_dim, dtype=torch.bfloat16, device="cuda:0")
            v = torch.empty_like(k)
            binding.ff_kv_read(r["kv"], l, b, T0, k, v)
            return [t.cpu().view(torch.int16).numpy().view(np.uint16) for t in (k, v)]
        _check_appended_cache(read_rows, lambda l, b, kv_i: r["okv_new"][l, b, kv_i], shape.n_layers, B, stats["fused"], f"llama3-70b B={B}")
        _progress(capsys, f"  70B batch-{B} run compared")
        binding.ff_kv_free(r["kv"])
    dec.close()


def test_hot_path_dequantisation_is_bit_exact_on_unit_vectors():
    """ff_debug_gemv runs the decode kernels' own projection code (vector-ALU GEMV: path 0,
    matrix-core GEMV: path 1) on unit vectors e_k: output row n is then the single product the
    kernel forms for weight (n, k) -- q * s for int8, s * (code - z) for int4, in either path's
    arrangement of the arithmetic -- and must equal the oracle's dequantised matrix bit for bit.
    Every column of every matrix of a small model, sampled columns at the 8B width."""
    from paper_2505_22758_amd import binding
    from oracle import oracle
    cases = [(synth.TINY.replace(n_layers=1, d_ffn=1408), None), (synth.LLAMA_8B.replace(n_layers=1, vocab=2048), 24)]
    for S, n_cols in cases:
        for wd in (synth.WDTYPE_BF16, synth.WDTYPE_INT8, synth.WDTYPE_INT4):
            dec = binding.Decoder(S, wd, max_batch=4)
            lw = synth.make_layer(S, 33, 0, wd, "cuda:0")
            head = synth.make_head(S, 33, wd, "cuda:0")
            dec.load_layer(0, lw)
            dec.load_head(head)
            mats = [(w, lw[w]) for w in synth.LAYER_MATS] + [("lm_head", head["lm_head"])]
            for which, m in mats:
                ref = oracle.dequant_matrix({kk: v.cpu() for kk, v in m.items()})   # fp32 [N, K]
                n, k = ref.shape
                rng = np.random.default_rng(n * 31 + k)
                cols = np.arange(k) if n_cols is None else np.unique(np.concatenate([[0, 1, 127, 128, k - 1], rng.integers(0, k, n_cols)]))
                for path, bsz in ((0, 1), (0, 4), (1, 2), (1, 4)):
                    if path == 1 and k * 4 * bsz > 128 * 1024:
                        continue   # the matrix-core path stages one K segment here
                    out = torch.empty(bsz, n, dtype=torch.float32, device="cuda:0")
                    for c0 in range(0, len(cols), bsz):
                        cc = cols[c0:c0 + bsz]
                        cc = np.concatenate([cc, np.repeat(cc[-1:], bsz - len(cc))])
                        x = torch.zeros(bsz, k, dtype=torch.float32, device="cuda:0")
                        x[torch.arange(bsz), torch.from_numpy(cc).to("cuda:0")] = 1.0
                        binding.ff_debug_gemv(dec.model, 0, which, x, out, path)
                        got = out.cpu().numpy()
                        for i, c in enumerate(cc):
                            assert np.array_equal(got[i].view(np.uint32), ref[:, c].view(np.uint32)), (S.name, wd, which, path, bsz, int(c))
            dec.close()


def test_bad_position_in_a_later_pass_skips_the_whole_step():
    """Batch 6 with int8 weights runs as a pass of four and a pass of two.  A position == max_ctx in
    the SECOND pass must skip the first pass too: no row is appended, the logits buffer is left
    alone, ff_status reports FF_ERR_RANGE, and the next good step matches a model that never saw
    the bad one."""
    from paper_2505_22758_amd import binding
    S, seed, T0, B = synth.TINY.replace(d_ffn=1408), 95, 6, 6
    for fn in (binding.ff_decode_step, binding.ff_decode_step_perop):
        dec, caches = helpers.hip_side(S, seed, synth.WDTYPE_INT8, B, T0, max_ctx=8, n_caches=2)
        tok = torch.arange(1, B + 1, dtype=torch.int32, device="cuda:0")
        good = torch.full((B,), T0, dtype=torch.int32, device="cuda:0")
        bad = good.clone()
        bad[5] = 8
        sentinel = torch.full((B, S.vocab), 7.5, dtype=torch.float32, device="cuda:0")
        logits = sentinel.clone()
        before = caches[0][1].clone()
        fn(dec.model, tok, bad, caches[0][0], logits, B)
        with pytest.raises(binding.FFError) as e:
            binding.ff_status(dec.model)
        assert e.value.code == binding.FF_ERR_RANGE
        if fn is binding.ff_decode_step:   # (the per-operation path leaves undefined logits behind)
            assert torch.equal(logits, sentinel), "a pass of a skipped step wrote logits"
        assert torch.equal(before, caches[0][1]), "a pass of a skipped step appended cache rows"
        fn(dec.model, tok, good, caches[0][0], logits, B)
        binding.ff_status(dec.model)
        clean = torch.zeros_like(logits)
        fn(dec.model, tok, good, caches[1][0], clean, B)   # same model, untouched cache
        binding.ff_status(dec.model)
        assert torch.equal(logits, clean)
        dec.close()


def test_fused_step_replayed_from_a_hip_graph():
    """ff_decode_step carries no host-side per-step state, so a captured step can be replayed: tokens
    and positions live in fixed device tensors that are updated between replays (with the program's
    own eager work and synchronisations in between), and every replay must equal the eager result
    of the same step on a second cache; batch 1, batch 3 (with the row re-initialisation launch) and
    batch 6 (wide pass: embedding launch + fused kernel, epochs derived from the device-side counter)."""
    from paper_2505_22758_amd import binding
    S, seed, T0, steps = synth.TINY, 97, 30, 6
    for B in (1, 3, 6):
        dec, caches = helpers.hip_side(S, seed, synth.WDTYPE_BF16, B, T0, max_ctx=T0 + steps + 2, n_caches=2)
        toks = synth.make_tokens(S, seed, steps, B).to("cuda:0")
        tok_s = toks[0].clone()
        pos_s = torch.full((B,), T0, dtype=torch.int32, device="cuda:0")
        lg_graph = torch.zeros(B, S.vocab, device="cuda:0")
        lg_eager = torch.zeros_like(lg_graph)
        # eager step 0 on both caches first (warm-up outside the capture)
        binding.ff_decode_step(dec.model, tok_s, pos_s, caches[0][0], lg_graph, B)
        binding.ff_decode_step(dec.model, tok_s, pos_s, caches[1][0], lg_eager, B)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        with torch.cuda.graph(g, stream=side):
            binding.ff_decode_step(dec.model, tok_s, pos_s, caches[0][0], lg_graph, B, stream=side)
        torch.cuda.synchronize()
        for s in range(1, steps):
            tok_s.copy_(toks[s])
            pos_s.fill_(T0 + s)
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            binding.ff_decode_step(dec.model, toks[s], torch.full((B,), T0 + s, dtype=torch.int32, device="cuda:0"), caches[1][0], lg_eager, B)
            torch.cuda.synchronize()
            binding.ff_status(dec.model)
            assert torch.equal(lg_graph, lg_eager), (B, s)
        dec.close()


def test_wide_pass_with_int8_weights():
    """The wide pass with int8 per-channel weights (five or more sequences, int8 LM head): the codes are
    converted to bf16 in registers (exact) and multiplied on the same 16x16x32 tiles, one ring stage of 512
    columns per tile and K segment, row scales on the finished sums.  A small model with an odd and an even
    number of tiles per workgroup (16 and 11 sequences, ragged lengths), the model whose output and down
    projections are split along K, and one layer at the 8B width."""
    S = synth.TINY.replace(name="wide8", n_layers=2, d_model=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, d_ffn=6144, vocab=3000)
    _run_teacher_forced(S, 0x2505227b0, synth.WDTYPE_INT8, batch=16, T0=[40, 0, 1, 130, 64, 63, 65, 9, 300, 17, 128, 5, 77, 256, 2, 33], steps=2)
    _run_teacher_forced(S, 0x2505227b1, synth.WDTYPE_INT8, batch=11, T0=[7, 70, 0, 129, 31, 64, 200, 1, 90, 12, 55], steps=2)
    _run_teacher_forced(KSPLIT, 0x2505227b2, synth.WDTYPE_INT8, batch=9, T0=[3, 70, 0, 129, 31, 64, 200, 1, 90], steps=2)
    _run_teacher_forced(synth.LLAMA_8B.replace(n_layers=1), 0x2505227b3, synth.WDTYPE_INT8, batch=8, T0=[96, 1, 300, 64, 63, 65, 0, 200], steps=2,
                        gpu_generated=True)


def test_wide_pass_with_int4_weights():
    """The wide pass with int4 group-128 weights (input widths multiples of 512, int4 LM head): codes as bf16
    128 + n on the 16x16x32 tiles, one ring stage per pair of tiles, group sums of the inputs from a ones operand,
    scales and zeros fetched across lanes into the accumulator layout.  A small model with odd and even numbers
    of tile pairs (16 and 11 sequences, ragged lengths), the model whose output and down projections are split
    along K, and one layer at the 8B width."""
    S = synth.TINY.replace(name="wide4", n_layers=2, d_model=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, d_ffn=6144, vocab=3000)
    _run_teacher_forced(S, 0x2505227c0, synth.WDTYPE_INT4, batch=16, T0=[40, 0, 1, 130, 64, 63, 65, 9, 300, 17, 128, 5, 77, 256, 2, 33], steps=2)
    _run_teacher_forced(S, 0x2505227c1, synth.WDTYPE_INT4, batch=11, T0=[7, 70, 0, 129, 31, 64, 200, 1, 90, 12, 55], steps=2)
    _run_teacher_forced(KSPLIT, 0x2505227c2, synth.WDTYPE_INT4, batch=9, T0=[3, 70, 0, 129, 31, 64, 200, 1, 90], steps=2)
    _run_teacher_forced(synth.LLAMA_8B.replace(n_layers=1), 0x2505227c3, synth.WDTYPE_INT4, batch=8, T0=[96, 1, 300, 64, 63, 65, 0, 200], steps=2,
                        gpu_generated=True)


KSPLIT = synth.TINY.replace(name="ksplit", n_layers=2, d_model=1024, n_q_heads=64, n_kv_heads=8, head_dim=128, d_ffn=8192, vocab=2000)


def test_wide_pass_output_and_down_projection_split_along_k():
    """Wide pass on a model whose output and down projections have four K segments each (8192 input
    columns): the workgroups of a pair multiply the rows of both over half of the segments and hand each
    other the partial sums of the partner's rows.  Eight query heads per KV head, ragged lengths (the
    matrix-core attention form), a full pass of 16 and a pass of 7, two layers."""
    _run_teacher_forced(KSPLIT, 0x2505227a0, synth.WDTYPE_BF16, batch=16, T0=[40, 0, 1, 130, 64, 63, 65, 9, 300, 17, 128, 5, 77, 256, 2, 33], steps=2)
    _run_teacher_forced(KSPLIT, 0x2505227a1, synth.WDTYPE_BF16, batch=7, T0=[7, 70, 0, 129, 31, 64, 200], steps=2)


def test_a_silent_workgroup_ends_in_a_timeout_not_a_hang():
    """ff_debug_mute_workgroup makes one workgroup leave without publishing: every workgroup that
    needs its output gives up after its own bounded wait, the launch ends normally and ff_status
    reports FF_ERR_TIMEOUT.  A model created again on the same buffers then works."""
    import time
    from paper_2505_22758_amd import binding
    seed, T0 = 99, 20
    # 6: wide pass (waits on epochs instead of per-word counters); KSPLIT: the muted workgroup's partner waits for its partial sums
    for S, B in ((synth.TINY, 1), (synth.TINY, 2), (synth.TINY, 6), (KSPLIT, 6)):
        dec, caches = helpers.hip_side(S, seed, synth.WDTYPE_BF16, B, T0, max_ctx=T0 + 4)
        tok = torch.arange(3, 3 + B, dtype=torch.int32, device="cuda:0")
        pos = torch.full((B,), T0, dtype=torch.int32, device="cuda:0")
        lg = torch.zeros(B, S.vocab, device="cuda:0")
        want = torch.zeros_like(lg)
        binding.ff_decode_step_perop(dec.model, tok, pos, caches[0][0], want, B)
        binding.ff_status(dec.model)
        binding.ff_debug_mute_workgroup(dec.model, 5)
        t0 = time.perf_counter()
        binding.ff_decode_step(dec.model, tok, pos, caches[0][0], lg, B)
        with pytest.raises(binding.FFError) as e:
            binding.ff_status(dec.model)
        assert e.value.code == binding.FF_ERR_TIMEOUT
        print(f"\ntime-out path at batch {B}: {time.perf_counter() - t0:.2f} s")
        binding.ff_debug_mute_workgroup(dec.model, -1)
        # a fresh model (and cache handle) over the same device buffers; the cache rows are still there
        binding.ff_kv_free(caches[0][0])
        binding.ff_model_free(dec.model)
        dec.model = binding.ff_model_create(dec.cfg, dec.packed, dec.scratch)
        for l in range(S.n_layers):
            dec.load_layer(l, synth.make_layer(S, seed, l, synth.WDTYPE_BF16, "cuda:0"))
        dec.load_head(synth.make_head(S, seed, synth.WDTYPE_BF16, "cuda:0"))
        kv = binding.ff_kv_alloc(dec.model, B, T0 + 4, caches[0][1])
        binding.ff_decode_step(dec.model, tok, pos, kv, lg, B)
        binding.ff_status(dec.model)
        assert float((lg - want).abs().max()) < 1e-3
        binding.ff_kv_free(kv)
        dec.close()


def test_synthetic_loaders_match_the_python_generators_bit_for_bit():
    """ff_model_load_synthetic / ff_kv_fill_synthetic (device-side generator) against the canonical
    tensors of synth.py loaded through ff_model_load / ff_kv_fill: every dequantised matrix, the cache
    buffers and the logits of a decode step (embedding, gains) must be identical.  The seed has more
    than 32 bits (the key uses its low word on both sides)."""
    from paper_2505_22758_amd import binding
    S, seed, T0, B = synth.TINY.replace(n_layers=2, d_ffn=1408), 0x250522758, 33, 2
    for wd, qlm in ((synth.WDTYPE_BF16, True), (synth.WDTYPE_INT8, True), (synth.WDTYPE_INT8, False), (synth.WDTYPE_INT4, True)):
        cfg = binding.make_config(S, wd, B, qlm)
        pb, sb = binding.ff_model_bytes(cfg)
        packed = torch.zeros(pb, dtype=torch.uint8, device="cuda:0")
        scratch = torch.zeros(sb, dtype=torch.uint8, device="cuda:0")
        layers = [synth.make_layer(S, seed, l, wd, "cuda:0") for l in range(S.n_layers)]
        head = synth.make_head(S, seed, wd, "cuda:0", qlm)
        ma = binding.ff_model_load(cfg, layers, head, packed, scratch)
        dec = binding.Decoder.synthetic(S, seed, wd, B, qlm)
        mb = dec.model
        for l in range(S.n_layers):
            for which in synth.LAYER_MATS:
                n, k = synth.mat_shape(S, which)
                a = torch.empty(n, k, dtype=torch.float32, device="cuda:0")
                b = torch.empty_like(a)
                binding.ff_debug_dequant(ma, l, which, a)
                binding.ff_debug_dequant(mb, l, which, b)
                assert torch.equal(a, b), (wd, l, which)
        a = torch.empty(S.vocab, S.d_model, dtype=torch.float32, device="cuda:0")
        b = torch.empty_like(a)
        binding.ff_debug_dequant(ma, 0, "lm_head", a)
        binding.ff_debug_dequant(mb, 0, "lm_head", b)
        assert torch.equal(a, b), (wd, "lm_head")
        bufs, kvs = [], []
        for m in (ma, mb):
            buf = torch.zeros(binding.ff_kv_bytes(m, B, T0 + 4), dtype=torch.uint8, device="cuda:0")
            bufs.append(buf)
            kvs.append(binding.ff_kv_alloc(m, B, T0 + 4, buf))
        for l in range(S.n_layers):
            for sq in range(B):
                k, v = synth.make_kv_prefill(S, seed, l, sq, T0, "cuda:0")
                binding.ff_kv_fill(kvs[0], l, sq, 0, k, v)
        binding.ff_kv_fill_synthetic(kvs[1], seed, T0)
        torch.cuda.synchronize()
        assert torch.equal(bufs[0], bufs[1]), (wd, "kv prefill")
        tok = torch.tensor([5, 4000], dtype=torch.int32, device="cuda:0")
        pos = torch.full((B,), T0, dtype=torch.int32, device="cuda:0")
        la, lb = torch.zeros(B, S.vocab, device="cuda:0"), torch.zeros(B, S.vocab, device="cuda:0")
        binding.ff_decode_step(ma, tok, pos, kvs[0], la, B)
        binding.ff_decode_step(mb, tok, pos, kvs[1], lb, B)
        binding.ff_status(ma)
        binding.ff_status(mb)
        assert torch.equal(la, lb) and bool(torch.isfinite(la).all()), (wd, "logits")
        for kv in kvs:
            binding.ff_kv_free(kv)
        binding.ff_model_free(ma)
        dec.close()


def test_stacked_linear_layers_all_modes_against_the_oracle():
    """ff_debug_stack_linear (the ablation kernel of the paper's stacked-linear study) against the
    oracle's matrix-vector product applied layer after layer: one launch per layer, fused, and fused
    with cross-layer overlap give the same vector within the exchange format's rounding."""
    from paper_2505_22758_amd import binding
    from oracle import oracle
    for d, L in ((2048, 3), (4096, 2), (6144, 5)):
        w = synth.normal_bf16(5, f"stack{d}", (L, d, d), 0.02, "cuda:0")
        x = synth.normal_bf16(5, "stack.x", (d,), 1.0, "cuda:0").float()
        ref = x.cpu().numpy().astype(np.float64)
        for l in range(L):
            ref = oracle.matvec({"w": w[l].cpu()}, ref)
        scratch = torch.zeros(2 * ((4 * d + 255) // 256 * 256) + 256, dtype=torch.uint8, device="cuda:0")
        for mode in (0, 1, 2):
            y = torch.full((d,), 7.0, device="cuda:0")
            for _ in range(2):   # twice: the second call starts from the first one's exchange words
                binding.ff_debug_stack_linear(w, x, y, mode, scratch)
            torch.cuda.synchronize()
            assert int(scratch[-256:].view(torch.int32)[0]) == 0
            err = np.max(np.abs(y.cpu().numpy().astype(np.float64) - ref)) / np.max(np.abs(ref))
            print(f"stacked linear d={d} L={L} mode {mode}: max error / max |y| = {err:.2e}")
            assert err < 2e-6 * L, (d, L, mode, err)


def test_overlap_switch_changes_timing_not_results():
    """ff_debug_set_overlap(False) (tiles requested after the input has arrived) gives bit-identical logits."""
    from paper_2505_22758_amd import binding
    S, seed, T0 = synth.TINY, 101, 40
    dec, caches = helpers.hip_side(S, seed, synth.WDTYPE_BF16, 1, T0, max_ctx=T0 + 4, n_caches=2)
    tok = torch.tensor([9], dtype=torch.int32, device="cuda:0")
    pos = torch.tensor([T0], dtype=torch.int32, device="cuda:0")
    a, b = torch.zeros(1, S.vocab, device="cuda:0"), torch.zeros(1, S.vocab, device="cuda:0")
    binding.ff_decode_step(dec.model, tok, pos, caches[0][0], a, 1)
    binding.ff_debug_set_overlap(dec.model, False)
    binding.ff_decode_step(dec.model, tok, pos, caches[1][0], b, 1)
    binding.ff_debug_set_overlap(dec.model, True)
    binding.ff_status(dec.model)
    assert torch.equal(a, b)
    dec.close()


def test_glu_as_one_stream_small_model_all_formats(monkeypatch):
    """Single-sequence steps of a small model whose FFN is a whole number of gate/up pairs per wave
    (d_ffn 8192 over 1024 waves), so gate/up + down run as one stream with the down projection's input
    staged chunk by chunk (four chunks with bf16 weights, two with int8 / int4); the same models at
    batch 2 and 3 use the interleaved gate/up row order with the ordinary phase sequence."""
    S = synth.TINY.replace(name="glu", n_layers=3, d_model=2048, n_q_heads=16, n_kv_heads=4, head_dim=128, d_ffn=8192, vocab=3000)
    monkeypatch.setenv("FF_GLU_PIPE", "all")   # int8 weights take the one-stream form only on request (read when a model is created)
    for wd in (synth.WDTYPE_BF16, synth.WDTYPE_INT8, synth.WDTYPE_INT4):
        _run_teacher_forced(S, 0x250522780 + wd, wd, batch=1, T0=37, steps=3)
    _run_teacher_forced(S, 0x250522784, synth.WDTYPE_BF16, batch=2, T0=20, steps=2)
    _run_teacher_forced(S, 0x250522785, synth.WDTYPE_INT4, batch=3, T0=20, steps=2)


def test_wide_pass_of_up_to_16_sequences_small_model():
    """More than four sequences (bf16 weights) run as ONE wide pass: projections on 16x16x32 matrix-core
    tiles, inputs copied one K segment of 2048 columns at a time (d_model 4096 = 2 segments, d_ffn 6144
    = 3) from images written by the workgroups that own the values, the RMSNorm factor applied to the
    projection outputs, the LM head in row blocks: a full pass of 16 and a ragged one of 11, sequences
    of different lengths, two layers so that the residual rows are carried from layer to layer."""
    S = synth.TINY.replace(name="wide", n_layers=2, d_model=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, d_ffn=6144, vocab=3000)
    _run_teacher_forced(S, 0x250522790, synth.WDTYPE_BF16, batch=16, T0=[40, 0, 1, 130, 64, 63, 65, 9, 300, 17, 128, 5, 77, 256, 2, 33], steps=2)
    _run_teacher_forced(S, 0x250522791, synth.WDTYPE_BF16, batch=11, T0=[7, 70, 0, 129, 31, 64, 200, 1, 90, 12, 55], steps=2)
