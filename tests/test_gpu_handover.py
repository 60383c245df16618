"""GPU checks of the hand-over between training and generation: low-rank adapters folded into the
stored weights on refresh, and the KV arena given back and taken again."""
import numpy as np
import pytest

from oracle import opt_oracle as O
from paper_2308_01320_amd import binding, synth
from tests import util

pytestmark = pytest.mark.gpu

MATS = ("wqkv", "wo", "w1", "w2")


def _adapters(d, w, rank, seed, skip=()):
    """bf16-valued factors A [rank,in], B [out,rank] for every layer matrix not in `skip`."""
    rng = np.random.default_rng(seed)
    out = []
    for lw in w["layers"]:
        ad = {}
        for m in MATS:
            if m in skip:
                continue
            o, i = lw[m].shape
            ad[m] = (synth.round_to_bf16(rng.normal(0, 0.05, (rank, i))), synth.round_to_bf16(rng.normal(0, 0.05, (o, rank))))
        out.append(ad)
    return out


def _merged(w, adapters, scale):
    out = dict(w)
    out["layers"] = []
    for lw, ad in zip(w["layers"], adapters):
        nl = dict(lw)
        for m, (a, b) in ad.items():
            nl[m] = O.merge_lora(lw[m], a, b, scale).astype(np.float32)
        out["layers"].append(nl)
    return out


@pytest.mark.parametrize("rows,cols,rank,scale", [(96, 64, 1, 1.0), (70, 128, 4, 0.75), (1536, 512, 16, 0.75), (1024, 1024, 8, 0.3), (64, 48, 64, -0.3)])
def test_merged_matrix_bit_exact_against_oracle(rows, cols, rank, scale):
    """The folded matrix is a rounding decision: it is compared bit for bit with the oracle's merge,
    through the plain tiling of the oracle's result."""
    import torch
    rng = np.random.default_rng(rows + rank)
    bf = synth.round_to_bf16
    W, A, B = bf(rng.normal(0, 0.05, (rows, cols))), bf(rng.normal(0, 0.05, (rank, cols))), bf(rng.normal(0, 0.05, (rows, rank)))
    dev = lambda x: torch.from_numpy(np.ascontiguousarray(x, np.float32)).cuda().to(torch.bfloat16).contiguous()
    got = binding.he_tile_matrix_lora(dev(W), dev(A), dev(B), scale)
    want = binding.he_tile_matrix(dev(O.merge_lora(W, A, B, scale)))
    torch.cuda.synchronize()
    diff = int((got != want).sum())
    assert diff == 0, f"{diff} bytes differ"
    # and against the plain definition -- the float64 sum rounded once to bf16: the float32 sum can only fall on
    # the other side of a rounding boundary, so at most one bf16 step apart, and on few elements
    exact = binding.he_tile_matrix(dev(O.merge_lora(W, A, B, scale, exact=True)))
    torch.cuda.synchronize()
    g, e = got.view(torch.float16).double(), exact.view(torch.float16).double()
    off = g != e
    assert float(off.double().mean()) < 0.01
    assert bool(((g - e).abs() <= e.abs() * 2.0 ** -7 + 1e-30).all())


@pytest.mark.parametrize("rank,skip", [(4, ()), (16, ("wo", "w1"))])
def test_lora_refresh_equals_an_engine_built_on_merged_weights(rank, skip):
    import torch
    d = synth.ModelDims("x", 2, 256, 4, 512, 1000, 128, 5, 37, 6, "bf16", "gumbel")
    w = synth.make_weights(d, seed=3, tied=True)
    ads = _adapters(d, w, rank, 4, skip)
    scale = 0.75
    p = torch.from_numpy(synth.make_prompts(d, seed=5)).cuda()
    s = binding.sampling("gumbel", 1.0, 9)
    eng = util.make_engine(d, w)
    base_ids, base_lp = eng.he_generate(p, d.gen_len, s)
    to_dev = lambda x: torch.from_numpy(np.ascontiguousarray(x, np.float32)).cuda().to(torch.bfloat16).contiguous()
    dev_ads = [{m: (to_dev(a), to_dev(b)) for m, (a, b) in ad.items()} for ad in ads]
    eng.he_refresh_weights_lora(dev_ads, rank, scale)
    ids1, lp1 = eng.he_generate(p, d.gen_len, s)
    # the oracle's merge (float32 in the stated order, rounded to bf16) fed to a fresh engine as plain weights
    wm = _merged(w, ads, scale)
    eng2 = util.make_engine(d, wm)
    ids2, lp2 = eng2.he_generate(p, d.gen_len, s)
    torch.cuda.synchronize()
    assert torch.equal(ids1, ids2) and torch.equal(lp1, lp2)  # bit for bit: the merged matrices are identical
    assert not torch.equal(lp1, base_lp)                        # and the adapters do change the model
    # teacher-forced against the oracle on the merged weights
    want = util.oracle_run(d, wm, synth.make_prompts(d, seed=5), d.gen_len, "gumbel", 1.0, 9)
    got = util.engine_teacher_forced(eng, synth.make_prompts(d, seed=5), want["ids"], d.gen_len, s)
    rep = util.compare(got, want, 2e-2, 1e-2)
    print(rep)
    # a plain refresh undoes the merge: the caller's matrices were never written
    eng.he_refresh_weights()
    ids3, lp3 = eng.he_generate(p, d.gen_len, s)
    torch.cuda.synchronize()
    assert torch.equal(ids3, base_ids) and torch.equal(lp3, base_lp)
    eng.he_destroy()
    eng2.he_destroy()


def test_lora_argument_errors():
    import torch
    d = synth.ModelDims("x", 1, 128, 2, 128, 300, 64, 2, 8, 4, "bf16", "greedy")
    w = synth.make_weights(d, seed=1)
    eng = util.make_engine(d, w)
    L = binding.lib()
    arr = (binding.he_lora_layer * 1)()
    assert L.he_refresh_weights_lora(eng.handle, None, 4, 1.0) == binding.HE_ERR_INVALID_ARG
    assert L.he_refresh_weights_lora(eng.handle, arr, 0, 1.0) == binding.HE_ERR_INVALID_ARG
    a = torch.zeros(4, 128, dtype=torch.bfloat16, device="cuda")
    arr[0].wo.a = a.data_ptr()  # one factor only
    assert L.he_refresh_weights_lora(eng.handle, arr, 4, 1.0) == binding.HE_ERR_INVALID_ARG
    assert L.he_refresh_weights_lora(eng.handle, (binding.he_lora_layer * 1)(), 4, 1.0) == binding.HE_OK  # no adapters at all
    eng.he_destroy()
    f32 = synth.ModelDims("x", 1, 64, 2, 64, 100, 64, 2, 4, 2, "f32", "greedy")
    e2 = util.make_engine(f32, synth.make_weights(f32, seed=1))
    assert L.he_refresh_weights_lora(e2.handle, (binding.he_lora_layer * 1)(), 4, 1.0) == binding.HE_ERR_STATE
    e2.he_destroy()


def test_arena_release_and_acquire():
    import torch
    d = synth.ModelDims("x", 2, 128, 2, 256, 300, 128, 3, 9, 6, "bf16", "gumbel")
    w = synth.make_weights(d, seed=2)
    stream = torch.cuda.Stream()
    eng = binding.Engine(binding.make_config(d, stream=stream.cuda_stream), binding.upload_weights(w, d.dtype))
    p = torch.from_numpy(synth.make_prompts(d, seed=3)).cuda()
    s = binding.sampling("gumbel", 1.0, 4)
    with torch.cuda.stream(stream):
        ids0, lp0 = eng.he_generate(p, d.gen_len, s)
        sc0 = eng.he_score(torch.cat([p, ids0], 1).contiguous())
        torch.cuda.synchronize()
        free_before = torch.cuda.mem_get_info()[0]
        eng.he_release_arena()
        eng.he_release_arena()  # idempotent
        assert torch.cuda.mem_get_info()[0] >= free_before  # the arena is small here; at least nothing was taken
        L = binding.lib()
        import ctypes as C
        o_i = torch.empty(3, 6, dtype=torch.int32, device="cuda")
        o_p = torch.empty(3, 6, dtype=torch.float32, device="cuda")
        assert L.he_generate(eng.handle, p.data_ptr(), 3, 9, 6, C.byref(s), o_i.data_ptr(), o_p.data_ptr()) == binding.HE_ERR_STATE
        assert L.he_prefill(eng.handle, p.data_ptr(), 3, 9, C.byref(s), o_i.data_ptr(), o_p.data_ptr(), None) == binding.HE_ERR_STATE
        assert L.he_score(eng.handle, p.data_ptr(), 3, 9, o_p.data_ptr()) == binding.HE_ERR_STATE
        assert L.he_decode_step(eng.handle, o_i.data_ptr(), C.byref(s), o_i.data_ptr(), o_p.data_ptr(), None) == binding.HE_ERR_STATE
        eng.he_acquire_arena()
        eng.he_acquire_arena()
        ids1, lp1 = eng.he_generate(p, d.gen_len, s)  # the decode step is captured again on the new arena
        sc1 = eng.he_score(torch.cat([p, ids1], 1).contiguous())
        torch.cuda.synchronize()
        assert torch.equal(ids0, ids1) and torch.equal(lp0, lp1) and torch.equal(sc0, sc1)
    eng.he_destroy()
