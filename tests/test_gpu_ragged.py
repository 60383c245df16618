"""GPU parity of the ragged entry points (left-padded prompts of different lengths, end-token
stop) against the oracle (the unrounded definition), which runs every sequence alone on its own tokens."""
import numpy as np
import pytest

from oracle import opt_oracle as O
from paper_2308_01320_amd import binding, synth
from tests import util

pytestmark = pytest.mark.gpu

F32_TOL, BF16_TOL, MARGIN = 1e-4, 2e-2, 1e-2


def _f64(w, tied):
    return util.weights_f64(w)


def _ragged_batch(d, lens, S, seed, junk=True):
    """Left-padded [B,S] ids, the per-sequence token arrays, and the lengths."""
    rng = np.random.default_rng(seed)
    B = len(lens)
    # what stands in the padding must not matter: fill it with valid but arbitrary ids
    ids = rng.integers(0, d.vocab, (B, S)).astype(np.int32) if junk else np.zeros((B, S), np.int32)
    prompts = []
    for b, n in enumerate(lens):
        p = rng.integers(0, d.vocab, n).astype(np.int32)
        ids[b, S - n:] = p
        prompts.append(p)
    return ids, prompts, np.asarray(lens, np.int32)


def _teacher_forced(eng, ids, lens, forced, G, samp):
    import torch
    eng.he_reset()
    got = []
    i, lp, lg = eng.he_prefill_ragged(torch.from_numpy(ids).cuda(), torch.from_numpy(lens).cuda(), samp, want_logits=True)
    for n in range(G):
        got.append((i.cpu().numpy(), lp.cpu().numpy(), lg.cpu().numpy()))
        if n + 1 < G:
            i, lp, lg = eng.he_decode_step(torch.from_numpy(np.ascontiguousarray(forced[:, n])).cuda(), samp, want_logits=True)
    torch.cuda.synchronize()
    return got


def _check_teacher_forced(d, lens, S, G, tied, tol, impl=0, mode="gumbel", seed=3):
    w = synth.make_weights(d, seed=seed, tied=tied)
    ids, prompts, ln = _ragged_batch(d, lens, S, seed + 1)
    want = O.generate_ragged(_f64(w, tied), prompts, G, d.n_heads, mode=mode, temperature=0.9, seed=7, eps=d.ln_eps,
                             pos_offset=d.pos_offset)
    eng = util.make_engine(d, w, max_batch=len(lens), max_seq_len=S + G, impl=impl)
    got = _teacher_forced(eng, ids, ln, want["ids"], G, binding.sampling(mode, 0.9, 7))
    eng.he_destroy()
    worst, sure, match = 0.0, 0, 0
    for n in range(G):
        gi, glp, glg = got[n]
        for b in range(len(lens)):
            err = float(np.abs(glg[b] - want["logits"][b][n]).max())
            worst = max(worst, err)
            assert err <= tol, (b, n, err)
            if want["margins"][b, n] > MARGIN:
                sure += 1
                assert gi[b] == want["ids"][b, n], (b, n)
            else:  # a thin margin: one of the oracle's two best
                assert gi[b] in (want["ids"][b, n], want["second"][b, n]), (b, n)
            if gi[b] == want["ids"][b, n]:
                match += 1
                assert abs(glp[b] - want["logprobs"][b, n]) <= tol
    assert sure > 0.5 * G * len(lens)
    return worst


@pytest.mark.parametrize("lens,S,G", [
    ([5, 1, 9, 3], 9, 4),          # a sequence of one token, one that fills its row
    ([1, 2, 3, 4, 5, 6], 6, 3),    # fewer than 8 prompt rows: attention row by row
    ([40, 7, 33, 1, 40], 40, 3),   # prompt attention on the matrix cores, a sequence of one token among them
])
def test_f32_ragged_teacher_forced(lens, S, G):
    d = synth.ModelDims("x", 2, 128, 4, 256, 500, 128, len(lens), S, G, "f32", "gumbel")
    print("f32 ragged err", _check_teacher_forced(d, lens, S, G, True, F32_TOL))


@pytest.mark.parametrize("impl", [0, 1])
@pytest.mark.parametrize("H,nh,lens,S,G", [
    (256, 4, [37, 5, 20, 1], 37, 4),                 # head_dim 64; prompt pass of 36 rows on the matrix cores
    (256, 2, [70, 64, 3, 33, 70, 1, 12], 70, 3),     # head_dim 128; rows past one 64-row stretch
    (128, 2, [9, 2, 5], 10, 3),                      # 9 prompt rows: the short-prompt attention kernel; all rows padded
    (128, 1, [3, 1, 2], 4, 4),                       # 3 prompt rows: attention row by row
    (128, 2, [1 + (7 * i) % 12 for i in range(40)], 12, 3),  # 40 sequences: the decode step for more than 32 rows
])
def test_bf16_ragged_teacher_forced(impl, H, nh, lens, S, G):
    d = synth.ModelDims("x", 2, H, nh, 2 * H, 1000, 128, len(lens), S, G, "bf16", "gumbel")
    print("bf16 ragged err", impl, _check_teacher_forced(d, lens, S, G, impl == 0, BF16_TOL, impl=impl))


def _compare_generation(got_ids, got_lp, got_lens, want, tol, eos, pad):
    """Free-running: a sequence is compared up to its first step whose oracle margin is too thin to
    fix the token; what the engine itself reports must be consistent throughout."""
    B, G = got_ids.shape
    compared = 0
    for b in range(B):
        hits = np.nonzero(got_ids[b] == eos)[0] if eos >= 0 else []
        n_own = int(hits[0]) + 1 if len(hits) else G
        assert got_lens[b] == n_own, (b, got_lens[b], n_own)
        assert (got_ids[b, n_own:] == pad).all() and (got_lp[b, n_own:] == 0).all()
        assert (got_lp[b, :n_own] <= 0).all()
        for n in range(int(want["lens"][b])):
            if want["margins"][b, n] <= MARGIN:  # a thin margin: either of the oracle's two best, and the rows part ways
                assert got_ids[b, n] in (want["ids"][b, n], want["second"][b, n]), (b, n)
                break
            assert got_ids[b, n] == want["ids"][b, n], (b, n)
            assert abs(got_lp[b, n] - want["logprobs"][b, n]) <= tol, (b, n)
            compared += 1
        else:
            assert got_lens[b] == want["lens"][b]
    return compared


@pytest.mark.parametrize("dtype,tol", [("f32", F32_TOL), ("bf16", BF16_TOL)])
@pytest.mark.parametrize("mode", ["greedy", "gumbel"])
def test_generate_ragged_with_end_token(dtype, tol, mode):
    import torch
    lens, S, G = [12, 3, 40, 1, 25, 40], 40, 12
    d = synth.ModelDims("x", 2, 128, 2, 256, 60, 128, len(lens), S, G, dtype, mode)
    w = synth.make_weights(d, seed=11, tied=True)
    ids, prompts, ln = _ragged_batch(d, lens, S, 12)
    w64 = _f64(w, True)
    free = O.generate_ragged(w64, prompts, G, d.n_heads, mode=mode, seed=5, eps=d.ln_eps)
    eos = int(free["ids"][2, 3])  # sequence 2 ends after four tokens, others wherever they meet this token
    want = O.generate_ragged(w64, prompts, G, d.n_heads, mode=mode, seed=5, eos_id=eos, pad_id=1, eps=d.ln_eps)
    assert want["lens"][2] <= 4
    eng = util.make_engine(d, w, max_batch=len(lens), max_seq_len=S + G)
    gi, glp, gl = eng.he_generate_ragged(torch.from_numpy(ids).cuda(), torch.from_numpy(ln).cuda(), G,
                                         binding.sampling(mode, 1.0, 5), eos, 1)
    torch.cuda.synchronize()
    n = _compare_generation(gi.cpu().numpy(), glp.cpu().numpy(), gl.cpu().numpy(), want, tol, eos, 1)
    print("compared", n, "tokens; lens", gl.cpu().numpy(), want["lens"])
    assert n >= 20
    eng.he_destroy()


@pytest.mark.parametrize("H,nh,fp8", [(128, 2, 0), (256, 2, 0), (128, 2, 1)])
def test_generate_ragged_drops_rows_of_ended_sequences(H, nh, fp8):
    """96 sequences, most of which end early (a vocabulary of 40 and near-uniform sampling: one in forty tokens is
    the end token): the step starts on the matrix-core GEMMs of the wide path, and as the rows of ended sequences
    are dropped at the read-backs it moves to two activation slices, one slice, half a slice.  Every sequence is
    compared with the oracle's run of it alone; results must not depend on which row a sequence rides in."""
    import torch
    B, S, G, V = 96, 12, 72, 40
    rng = np.random.default_rng(31)
    lens = [int(x) for x in rng.integers(1, S + 1, B)]
    d = synth.ModelDims("x", 2, H, nh, 2 * H, V, 128, B, S, G, "bf16", "gumbel")
    w = synth.make_weights(d, seed=17, tied=True)
    ids, prompts, ln = _ragged_batch(d, lens, S, 18)
    eos, pad = 7, 1
    wq = w
    if fp8:
        wq = {k: v for k, v in w.items()}
        wq["layers"] = [{n: (O.quantize_e4m3_rows(a)[0] if n in ("wqkv", "wo", "w1", "w2") else a) for n, a in lw.items()}
                        for lw in w["layers"]]
    want = O.generate_ragged(_f64(wq, True), prompts, G, d.n_heads, mode="gumbel", seed=5, eos_id=eos, pad_id=pad,
                             eps=d.ln_eps)
    ended_early = int((want["lens"] < G - 8).sum())
    print("oracle: sequences that end more than 8 steps before the cap:", ended_early, flush=True)
    assert ended_early > B // 2
    stream = torch.cuda.Stream()
    eng = binding.Engine(binding.make_config(d, max_batch=B, max_seq_len=S + G, stream=stream.cuda_stream, weights_fp8=fp8),
                         binding.upload_weights(w, d.dtype))
    samp = binding.sampling("gumbel", 1.0, 5)
    with torch.cuda.stream(stream):
        gi, glp, gl = eng.he_generate_ragged(torch.from_numpy(ids).cuda(), torch.from_numpy(ln).cuda(), G, samp, eos, pad)
        torch.cuda.synchronize()
        rows = eng.he_last_step_rows()
        n = _compare_generation(gi.cpu().numpy(), glp.cpu().numpy(), gl.cpu().numpy(), want, BF16_TOL, eos, pad)
        print("compared", n, "tokens; rows of the last step", rows, flush=True)
        assert n >= 10 * B
        assert rows <= 64, rows  # rows were dropped: the last steps ran on the weight-streaming GEMMs
        assert eng.he_arrival_counters_nonzero() == 0
        # a second run is bit-identical, and the engine goes on as before: one row per sequence again
        gi2, glp2, gl2 = eng.he_generate_ragged(torch.from_numpy(ids).cuda(), torch.from_numpy(ln).cuda(), G, samp, eos, pad)
        torch.cuda.synchronize()
        assert torch.equal(gi, gi2) and torch.equal(glp, glp2) and torch.equal(gl, gl2)
        a_ids, a_lp, a_len = eng.he_generate_ragged(torch.from_numpy(ids).cuda(), torch.from_numpy(ln).cuda(), 6, samp, -1, pad)
        torch.cuda.synchronize()
        assert eng.he_last_step_rows() == B and (a_len == 6).all()
        # without an end token nothing is dropped, and the first tokens are those of the run above wherever that
        # run had not met its end token yet
        g, a, own = gi.cpu().numpy(), a_ids.cpu().numpy(), gl.cpu().numpy()
        for q in range(B):
            k = min(6, int(own[q]))
            assert (a[q, :k] == g[q, :k]).all(), q
    eng.he_destroy()


def test_ragged_with_equal_lengths_is_plain_generation_and_stops_early():
    import torch
    B, S, G = 5, 12, 40
    d = synth.ModelDims("x", 2, 128, 2, 256, 80, 128, B, S, G, "bf16", "greedy")
    w = synth.make_weights(d, seed=13, tied=True)
    stream = torch.cuda.Stream()
    eng = binding.Engine(binding.make_config(d, max_batch=8, max_seq_len=S + G, stream=stream.cuda_stream),
                         binding.upload_weights(w, d.dtype))
    row = synth.make_prompts(d, seed=14, batch=1, prompt_len=S)
    p = torch.from_numpy(np.repeat(row, B, axis=0)).cuda()  # five copies of one prompt
    ln = torch.full((B,), S, dtype=torch.int32, device="cuda")
    s = binding.sampling("greedy", 1.0, 0)
    with torch.cuda.stream(stream):
        g0, lp0 = eng.he_generate(p, G, s)
        g1, lp1, l1 = eng.he_generate_ragged(p, ln, G, s, -1, 0)
        torch.cuda.synchronize()
        # same kernels, the per-sequence numbers just happen to be equal
        assert torch.equal(g0, g1) and torch.equal(lp0, lp1) and (l1 == G).all()
        # identical rows produce identical answers: make their fourth token the end token, so every
        # sequence has ended long before the first read-back of the running count (step 16)
        eos = int(g0[0, 3])
        first = int((g0[0] == eos).nonzero()[0])
        g2, lp2, l2 = eng.he_generate_ragged(p, ln, G, s, eos, 7)
        torch.cuda.synchronize()
        assert (l2 == first + 1).all()
        assert torch.equal(g2[:, :first + 1], g0[:, :first + 1]) and torch.equal(lp2[:, :first + 1], lp0[:, :first + 1])
        assert (g2[:, first + 1:] == 7).all() and (lp2[:, first + 1:] == 0).all()
        assert eng.cache_len() < S + G - 1  # the remaining steps were skipped
        # and the engine goes on as before
        g3, lp3 = eng.he_generate(p, G, s)
        torch.cuda.synchronize()
        assert torch.equal(g0, g3) and torch.equal(lp0, lp3)
    eng.he_destroy()


def test_ragged_argument_errors():
    import torch
    d = synth.ModelDims("x", 1, 128, 2, 128, 300, 64, 2, 8, 4, "bf16", "greedy")
    eng = util.make_engine(d, synth.make_weights(d, seed=1), max_batch=2, max_seq_len=16)
    L = binding.lib()
    import ctypes as C
    ids = torch.zeros(2, 8, dtype=torch.int32, device="cuda")
    ln = torch.tensor([3, 8], dtype=torch.int32, device="cuda")
    o_i = torch.empty(2, 4, dtype=torch.int32, device="cuda")
    o_p = torch.empty(2, 4, dtype=torch.float32, device="cuda")
    o_l = torch.empty(2, dtype=torch.int32, device="cuda")
    s = binding.sampling("greedy", 1.0, 0)
    call = lambda lens, eos, pad, lens_out: L.he_generate_ragged(eng.handle, ids.data_ptr(), lens, 2, 8, 4, C.byref(s), eos, pad,
                                                                 o_i.data_ptr(), o_p.data_ptr(), lens_out)
    assert call(None, -1, 0, o_l.data_ptr()) == binding.HE_ERR_INVALID_ARG
    assert call(ln.data_ptr(), -1, 0, None) == binding.HE_ERR_INVALID_ARG
    assert call(ln.data_ptr(), -1, 300, o_l.data_ptr()) == binding.HE_ERR_INVALID_ARG
    assert call(ln.data_ptr(), 300, 0, o_l.data_ptr()) == binding.HE_ERR_INVALID_ARG
    assert call(ln.data_ptr(), 5, 0, o_l.data_ptr()) == binding.HE_OK
    assert L.he_prefill_ragged(eng.handle, ids.data_ptr(), None, 2, 8, C.byref(s), o_i.data_ptr(), o_p.data_ptr(), None) == \
        binding.HE_ERR_INVALID_ARG
    # lengths outside 1..S are clamped, not trusted
    bad = torch.tensor([0, 99], dtype=torch.int32, device="cuda")
    assert L.he_generate_ragged(eng.handle, ids.data_ptr(), bad.data_ptr(), 2, 8, 4, C.byref(s), -1, 0, o_i.data_ptr(),
                                o_p.data_ptr(), o_l.data_ptr()) == binding.HE_OK
    torch.cuda.synchronize()
    assert bool(torch.isfinite(o_p).all())
    eng.he_destroy()


def test_ragged_headline_layer_shape_sampled_sequences():
    """OPT-13B layer shape, batch 32, left-padded prompts of up to 256 tokens, two layers; the oracle
    follows three of the sequences, each alone on its own tokens, teacher-forced on the engine's ids."""
    import torch
    base = synth.CONFIGS["opt-13b"]
    G = 3
    d = base.sliced(n_layers=2, gen_len=G, max_positions=512)
    w = synth.make_weights(d, seed=5)
    rng = np.random.default_rng(21)
    lens = rng.integers(1, 257, 32)
    lens[0], lens[17], lens[31] = 256, 1, 100
    ids, prompts, ln = _ragged_batch(d, list(lens), 256, 22)
    samp = binding.sampling("gumbel", 1.0, 42)
    eng = util.make_engine(d, w, max_batch=32, max_seq_len=512)
    got, i = [], None
    i, lp, lg = eng.he_prefill_ragged(torch.from_numpy(ids).cuda(), torch.from_numpy(ln).cuda(), samp, want_logits=True)
    for n in range(G):
        got.append((i.cpu().numpy(), lp.cpu().numpy(), lg.cpu().numpy()))
        if n + 1 < G:
            i, lp, lg = eng.he_decode_step(i, samp, want_logits=True)
    torch.cuda.synchronize()
    eng.he_destroy()
    w64 = _f64(w, True)
    for b in (0, 17, 31):
        dec = O.CachedDecoder(w64, d.n_heads, d.ln_eps, d.pos_offset)
        z = dec.prefill(prompts[b].reshape(1, -1))
        for n in range(G):
            err = float(np.abs(got[n][2][b] - z[0]).max())
            print("sequence", b, "len", lens[b], "step", n, "err", err, flush=True)
            assert err <= BF16_TOL
            score = z[0] + O.gumbel_noise(42, b, n, d.vocab)
            order = np.argsort(score)
            if score[order[-1]] - score[order[-2]] > MARGIN:
                assert got[n][0][b] == order[-1]
            else:
                assert got[n][0][b] in (order[-1], order[-2])
            assert abs(got[n][1][b] - O.log_softmax(z)[0, got[n][0][b]]) <= BF16_TOL
            if n + 1 < G:
                z = dec.step(got[n][0][b:b + 1])
