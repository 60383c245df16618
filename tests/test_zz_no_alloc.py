"""he_decode_step_static (the decode step with its scratch in a static device array, for callers
that cannot allocate) against he_decode_step: same engine state, same inputs, outputs bit for bit
-- the two run the same kernels on the same launch plan, only the scratch lives elsewhere.  Two
calls in a row, the second on a smaller batch, so that what the first left in the shared array
(partial sums, statistics, counters, LM-head partials of more rows) is there when the second runs."""
import numpy as np
import pytest

from paper_2308_01320_amd import binding, synth
from tests import util

pytestmark = pytest.mark.gpu


def _steps(eng, prompts, feeds, samp, static):
    import torch
    eng.he_reset()
    p = torch.from_numpy(prompts).cuda()
    out = [eng.he_prefill(p, samp, want_logits=True)]
    for f in feeds:
        step = eng.he_decode_step_static if static else eng.he_decode_step
        out.append(step(torch.from_numpy(f).cuda(), samp, want_logits=True))
    torch.cuda.synchronize()
    return [tuple(t.cpu().numpy() for t in o) for o in out]


def test_static_scratch_decode_step_matches_the_allocating_one():
    # layer shape wide enough for the out-projection and FC2 to be cut along k (their partial sums
    # then cross workgroups through the scratch), a vocabulary of many LM-head tiles with a ragged tail
    d = synth.ModelDims("static-scratch", 2, 1024, 16, 4096, 5000, 64, 32, 9, 4, "bf16", "gumbel")
    w = synth.make_weights(d, seed=11)
    eng = util.make_engine(d, w, max_batch=32, max_seq_len=16)
    samp = binding.sampling("gumbel", 1.0, 7)
    rng = np.random.default_rng(12)
    for B in (32, 5):  # the second call is the smaller one
        prompts = synth.make_prompts(d, seed=13 + B, batch=B)
        feeds = [rng.integers(0, d.vocab, size=B, dtype=np.int32) for _ in range(3)]
        want = _steps(eng, prompts, feeds, samp, static=False)
        got = _steps(eng, prompts, feeds, samp, static=True)
        for n, (g, w_) in enumerate(zip(got, want)):
            assert np.array_equal(g[0], w_[0]), (B, n, "ids")
            assert np.array_equal(g[1], w_[1]), (B, n, "logprobs")
            assert np.array_equal(g[2], w_[2]), (B, n, "logits")
    # and the static steps of the smaller batch against the oracle, teacher-forced on the same ids, to the bf16 bar
    from oracle import opt_oracle as O
    forced = np.stack(feeds + [feeds[0]], axis=1)
    ref = O.generate(w, prompts, 4, d.n_heads, mode="gumbel", temperature=1.0, seed=7, forced_ids=forced)
    for n in range(4):
        assert np.abs(got[n][2] - ref["logits"][n]).max() <= 2e-2, n
        sure = ref["margins"][:, n] > 1e-2
        assert np.array_equal(got[n][0][sure], ref["ids"][sure, n]), n
    eng.he_destroy()


def test_static_scratch_limits_are_errors():
    import torch
    d = synth.CONFIGS["tiny"]
    eng = util.make_engine(d, synth.make_weights(d, seed=0))  # f32 path
    samp = binding.sampling("greedy")
    eng.he_prefill(torch.from_numpy(synth.make_prompts(d)).cuda(), samp)
    with pytest.raises(binding.HeError) as ei:
        eng.he_decode_step_static(torch.zeros(d.batch, dtype=torch.int32, device="cuda"), samp)
    assert ei.value.status == binding.HE_ERR_STATE
    eng.he_destroy()
