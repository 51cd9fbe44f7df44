"""Batch > 1 (sb_new_batch / sb_batch_decode): the rounds of several sequences side by side,
sharing every weight sweep.  The oracle of a batch is the oracle of each sequence on its own:
every sequence's output must be what the library gives for it alone -- bit for bit, since a row's
value never depends on the rows beside it -- and that single-sequence output is scored by the
CPU oracle as everywhere else."""
import numpy as np
import pytest

import oracle as orc
import sb_inputs as si
from helpers import tiny_model, gpu_model, gpu_params, linear_T, teacher_forced_check
from oracle import Oracle

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sb():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2604_12247_amd as sb
    return sb


B16 = si.configs.BF16
KW = dict(weight_dtype=B16, kv_dtype=B16, d_ffn=768)


def _prompts(vocab, n, seed0):
    return [si.make_prompt(vocab, 7 + 5 * i, seed0 + i) for i in range(n)]


@pytest.mark.parametrize("B,w_max,gqa", [(2, 4, False), (4, 2, False), (3, 2, True), (8, 1, False)])
def test_batch_output_equals_each_sequence_alone_and_the_oracle(sb, B, w_max, gqa):
    kw = dict(KW, n_kv_heads=2, rope_base=500000.0) if gqa else KW
    shape, w, om = tiny_model(n_layers=6, n_exit_heads=3, seed=31, max_seq=160, **kw)
    gm = gpu_model(shape, w, 160)
    prompts = _prompts(shape.vocab, B, 900)
    n_new = 33
    # different forced schedules per sequence (exit layers, depth bounds, injected wrong drafts)
    P = []
    for b in range(B):
        fe = si.forced_exit_schedule(40 + b, 300, 0, 3)
        fd = np.where(np.random.default_rng(b).random(300) < 0.3, 5 + b, -1).astype(np.int32)
        P.append(gpu_params(3, w_max, 0.5, forced_exit=fe, forced_draft=fd))
    alone, stats_alone = [], []
    for b in range(B):
        out, st = gm.session().generate(prompts[b], n_new, P[b])
        alone.append(out); stats_alone.append(st)
    sess = [gm.session() for _ in range(B)]
    firsts = [s.prefill(p) for s, p in zip(sess, prompts)]
    bt = sb.Batch(sess)
    outs = bt.decode(n_new - 1, P)
    for b in range(B):
        assert [firsts[b]] + outs[b].tolist() == alone[b].tolist(), b
        st = sess[b].stats()
        for k in ("rounds", "drafts", "emitted", "draft_steps", "head_evals"):
            assert st[k] == stats_alone[b][k], (b, k)
        assert st["accept_hist"] == stats_alone[b]["accept_hist"] and st["exit_hist"] == stats_alone[b]["exit_hist"]
    # the point of the batch: far fewer weight sweeps than the sequences need one by one
    decode_sweeps_alone = sum(st["layer_sweeps"] for st in stats_alone) - sum(
        shape.n_layers * -(-len(p) // sb.SB_MAX_W) for p in prompts)
    sweeps_batch = sess[0].stats()["layer_sweeps"] - shape.n_layers * -(-len(prompts[0]) // sb.SB_MAX_W)
    assert sweeps_batch < 0.75 * decode_sweeps_alone
    # the sessions go on alone afterwards, from the state the batch left
    more, _ = sess[1].decode(5, gpu_params(0, 1))
    ref, _ = gm.session().generate(prompts[1], n_new + 5, gpu_params(0, 1))
    assert more.tolist() == ref[n_new:].tolist()
    # the single-sequence output is the oracle's up to near-ties
    flagged, _ = teacher_forced_check(om, prompts[0], alone[0])
    assert flagged <= 2


def test_batch_with_computed_exits_and_sampling(sb):
    """Computed exits (the device decides per sequence) on the easy-token fixture, one sequence
    sampled and one greedy in the same batch: each equals its own single-sequence run."""
    shape = si.tiny_shape(n_layers=12, n_exit_heads=8, **KW)
    w = si.easy_token_weights(shape, si.make_weights(shape, 77), decay=0.5, head_scale=20.0)
    gm = gpu_model(shape, w, 256)
    prompts = _prompts(shape.vocab, 2, 950)
    T = sb.temperature_schedule(0.2, 8, 8)
    U = np.random.default_rng(9).random(2 * 256).astype(np.float32)
    P = [sb.Params(8, 4, T, 0.3), sb.Params(8, 4, T, 0.5, sample_temperature=0.8, top_p=0.9, sample_u=U)]
    alone = [gm.session().generate(prompts[b], 40, P[b]) for b in range(2)]
    sess = [gm.session() for _ in range(2)]
    firsts = [s.prefill(p) for s, p in zip(sess, prompts)]
    outs = sb.Batch(sess).decode(39, P)
    for b in range(2):
        assert [firsts[b]] + outs[b].tolist() == alone[b][0].tolist()
        assert sess[b].stats()["drafts"] == alone[b][1]["drafts"] > 0
        assert sess[b].stats()["exit_hist"] == alone[b][1]["exit_hist"]
    # eos of one sequence ends it while the other goes on
    eos = int(alone[0][0][7])
    P2 = [sb.Params(8, 4, T, 0.3, eos_id=eos), P[1]]
    sess = [gm.session() for _ in range(2)]
    firsts = [s.prefill(p) for s, p in zip(sess, prompts)]
    outs = sb.Batch(sess).decode(39, P2)
    full0 = [firsts[0]] + outs[0].tolist()
    assert full0 == alone[0][0][: alone[0][0].tolist().index(eos) + 1].tolist()
    assert [firsts[1]] + outs[1].tolist() == alone[1][0].tolist()


def test_batch_of_sampled_sequences_at_a_large_vocabulary(sb):
    """Two sampled sequences (different temperatures and uniforms) over a vocabulary above 32768, where the
    acceptance kernel keeps part of each row's soft-max weights in the workspace: every sequence has a region of
    its own there, so each output equals the sequence's single run, token for token."""
    shape = si.tiny_shape(n_layers=5, n_exit_heads=3, vocab=32768 + 1040, **KW)
    w = si.make_weights(shape, 93)
    gm = gpu_model(shape, w, 128)
    prompts = _prompts(shape.vocab, 2, 990)
    T = linear_T(3)
    g = np.random.default_rng(17)
    P = [sb.Params(3, 4, T, 0.0, sample_temperature=t, top_p=tp, sample_u=g.random(2 * 128).astype(np.float32))
         for t, tp in ((1.0, 0.9), (0.6, 0.7))]
    alone = [gm.session().generate(prompts[b], 24, P[b]) for b in range(2)]
    sess = [gm.session() for _ in range(2)]
    firsts = [s.prefill(p) for s, p in zip(sess, prompts)]
    outs = sb.Batch(sess).decode(23, P)
    for b in range(2):
        assert [firsts[b]] + outs[b].tolist() == alone[b][0].tolist()
        assert sess[b].stats()["rounds"] == alone[b][1]["rounds"]
    assert alone[0][0].tolist() != alone[1][0].tolist()


def test_failed_launch_in_a_batch_abandons_the_open_rounds_of_all_sequences(sb):
    """A projection launch that fails inside a batched round (forced from the host, nothing faults on
    the GPU): sb_batch_decode returns a device error, every sequence keeps its committed tokens and
    cache, and decoding on -- together or alone -- gives what an undisturbed run gives."""
    shape, w, om = tiny_model(n_layers=6, n_exit_heads=3, seed=33, max_seq=160, **KW)
    gm = gpu_model(shape, w, 160)
    prompts = _prompts(shape.vocab, 2, 970)
    P = [gpu_params(3, 4, 0.5, forced_exit=si.forced_exit_schedule(50 + b, 300, 0, 3)) for b in range(2)]
    ref = [gm.session().generate(prompts[b], 31, P[b])[0].tolist() for b in range(2)]
    sess = [gm.session() for _ in range(2)]
    firsts = [s.prefill(p) for s, p in zip(sess, prompts)]
    bt = sb.Batch(sess)
    got = [o.tolist() for o in bt.decode(8, P)]
    c0 = [s.committed_len() for s in sess]
    for nth in (3, 40):                       # in a draft super-step, in the verification
        sess[0].debug_fail_launch(nth)        # (the shared sweeps are launched through the first session)
        with pytest.raises(sb.SbError) as e:
            bt.decode(20, P)
        assert e.value.code == sb.EDEVICE
        assert [s.committed_len() for s in sess] == c0 and all(s.open_rows() == 0 for s in sess)
    sess[0].debug_fail_launch(0)
    more = [o.tolist() for o in bt.decode(12, P)]
    rest1, _ = sess[1].decode(10, P[1])
    for b in range(2):
        assert [firsts[b]] + got[b] + more[b] == ref[b][:21], b
    assert ref[1][21:31] == rest1.tolist()


def test_batch_argument_errors(sb):
    shape, w, om = tiny_model(n_layers=4, n_exit_heads=2, seed=3, max_seq=96, **KW)
    gm = gpu_model(shape, w, 96)
    s1, s2 = gm.session(), gm.session()
    with pytest.raises(sb.SbError) as e:
        sb.Batch([s1])
    assert e.value.code == sb.EINVAL
    with pytest.raises(sb.SbError) as e:
        sb.Batch([s1, s1])
    assert e.value.code == sb.EINVAL
    bt = sb.Batch([s1, s2])
    p = gpu_params(2, 4, 0.5)
    with pytest.raises(sb.SbError) as e:
        bt.decode(4, [p, p])                      # not prefilled
    assert e.value.code == sb.ESTATE
    s1.prefill(si.make_prompt(shape.vocab, 6, 1)); s2.prefill(si.make_prompt(shape.vocab, 9, 2))
    with pytest.raises(sb.SbError) as e:
        bt.decode(4, [gpu_params(2, 5, 0.5), p])  # w_max beyond the 4 rows a sequence has in a batch of 2
    assert e.value.code == sb.EINVAL
    with pytest.raises(sb.SbError) as e:
        bt.decode(90, [p, p])
    assert e.value.code == sb.ECAPACITY
    # fp32 weights (vector-ALU projections) have no batch path
    shape32, w32, _ = tiny_model(n_layers=4, n_exit_heads=2, seed=3, max_seq=96)
    g32 = gpu_model(shape32, w32, 96)
    with pytest.raises(sb.SbError) as e:
        sb.Batch([g32.session(), g32.session()])
    assert e.value.code == sb.EINVAL
