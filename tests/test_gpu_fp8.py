"""GPU checks of 8-bit weight storage (he_config.weights_fp8): the quantisation bit for bit against the
oracle's, and the engine against the oracle run on the dequantised weights."""
import numpy as np
import pytest

from oracle import opt_oracle as O
from paper_2308_01320_amd import binding, synth
from tests import util

pytestmark = pytest.mark.gpu

BF16_TOL, MARGIN = 2e-2, 1e-2
MATS = ("wqkv", "wo", "w1", "w2")


def _dequantised(w):
    """The model the engine computes with: layer matrices replaced by their E4M3-quantised values."""
    out = dict(w)
    out["layers"] = []
    for lw in w["layers"]:
        nl = dict(lw)
        for m in MATS:
            nl[m] = O.quantize_e4m3_rows(lw[m])[0].astype(np.float32)
        out["layers"].append(nl)
    return out


@pytest.mark.parametrize("rows,cols,scale", [(48, 64, 0.02), (100, 256, 5.0), (512, 1024, 0.02), (33, 8, 1e-6)])
def test_row_quantisation_bit_exact_against_oracle(rows, cols, scale):
    import torch
    rng = np.random.default_rng(rows + cols)
    W = synth.round_to_bf16(rng.normal(0, scale, (rows, cols)))
    W[1] = 0.0
    W[2] *= 1024.0  # a power of two: the values stay bf16
    if cols >= 64:
        W[3, :] = 0.0
        W[3, 5] = 448.0 * 2.0 ** -3  # a row whose largest value sits exactly at the top of the range
    dev = torch.from_numpy(np.ascontiguousarray(W, np.float32)).cuda().to(torch.bfloat16).contiguous()
    codes, exps, scales = binding.he_fp8_quantize_rows(dev)
    torch.cuda.synchronize()
    _, want_codes, want_e = O.quantize_e4m3_rows(W)
    np.testing.assert_array_equal(exps.cpu().numpy(), want_e)
    np.testing.assert_array_equal(scales.cpu().numpy().astype(np.float64), 2.0 ** want_e.astype(np.float64))
    got = codes.cpu().numpy()
    # the sign bit of a zero is not part of the value
    zero = (want_codes & 0x7F) == 0
    assert np.array_equal(got[~zero], want_codes[~zero]) and np.all((got[zero] & 0x7F) == 0)


@pytest.mark.parametrize("L,H,nh,F,V,B,S,G", [
    (2, 256, 4, 512, 1000, 3, 37, 5),     # prompt rows through the dequantised scratch layer, decode on the codes
    (2, 256, 2, 576, 1111, 5, 70, 4),     # head_dim 128, ffn not a multiple of 128
    (1, 128, 2, 128, 300, 1, 1, 4),       # decode-shaped passes only
    (1, 192, 3, 320, 513, 40, 3, 3),      # more than 32 sequences: every GEMM on the scratch layer
])
def test_fp8_weights_against_oracle_on_dequantised_model(L, H, nh, F, V, B, S, G):
    d = synth.ModelDims("x", L, H, nh, F, V, 128, B, S, G, "bf16", "gumbel")
    w = synth.make_weights(d, seed=3, tied=True)
    wq = _dequantised(w)
    prompts = synth.make_prompts(d, seed=4)
    want = util.oracle_run(d, wq, prompts, G, "gumbel", 0.9, 7)
    eng = binding.Engine(binding.make_config(d, weights_fp8=1), binding.upload_weights(w, d.dtype))
    got = util.engine_teacher_forced(eng, prompts, want["ids"], G, binding.sampling("gumbel", 0.9, 7))
    rep = util.compare(got, want, BF16_TOL, MARGIN)
    print(rep)
    assert eng.he_arrival_counters_nonzero() == 0  # the k-split launches left their counters ready for the next
    # against the unquantised model the logits differ by far more than the tolerance: the codes are in use
    plain = util.oracle_run(d, w, prompts, G, "gumbel", 0.9, 7)
    assert float(np.abs(plain["logits"] - want["logits"]).max()) > 10 * rep["logit_err"]
    # scoring goes through the scratch layer as well
    import torch
    seq = np.concatenate([prompts, want["ids"]], axis=1)
    sc = eng.he_score(torch.from_numpy(seq).cuda()).cpu().numpy()
    ref = O.score(util_f64(wq), seq, d.n_heads, eps=d.ln_eps, pos_offset=d.pos_offset)
    assert float(np.abs(sc - ref).max()) <= BF16_TOL
    eng.he_destroy()


def util_f64(w):
    out = {k: (v.astype(np.float64) if k != "layers" else [{n: a.astype(np.float64) for n, a in lw.items()} for lw in v])
           for k, v in w.items()}
    out["lm_head"] = out["tok_emb"]
    return out


def test_fp8_real_layer_shape_and_memory():
    """OPT-13B layer shape, batch 32: the launch shapes of the benchmark's 8-bit variant."""
    base = synth.CONFIGS["opt-13b"]
    d = base.sliced(n_layers=1, batch=32, prompt_len=9, gen_len=3, max_positions=256)
    w = synth.make_weights(d, seed=42)
    wq = _dequantised(w)
    prompts = synth.make_prompts(d, seed=43)
    want = util.oracle_run(d, wq, prompts, 3, "gumbel", 1.0, 42)
    L = binding.lib()
    import ctypes as C
    # memory, on the full 40-layer configuration (a size query, nothing is allocated): 8-bit codes take half the
    # bytes of the bf16 copies of the layer matrices, minus one layer of bf16 scratch and the row scales
    full8, full16 = binding.make_config(base, weights_fp8=1), binding.make_config(base)
    b8, b16 = L.he_workspace_bytes(C.byref(full8)), L.he_workspace_bytes(C.byref(full16))
    layer16 = 2 * (4 * base.hidden * base.hidden + 2 * base.hidden * base.ffn)
    saved = b16 - b8
    print("engine bytes bf16", b16, "8-bit", b8, "saved", saved, flush=True)
    assert 0.9 * (base.n_layers * layer16 // 2 - layer16) <= saved <= base.n_layers * layer16 // 2
    cfg8 = binding.make_config(d, weights_fp8=1)
    eng = binding.Engine(cfg8, binding.upload_weights(w, d.dtype))
    got = util.engine_teacher_forced(eng, prompts, want["ids"], 3, binding.sampling("gumbel", 1.0, 42))
    rep = util.compare(got, want, BF16_TOL, MARGIN)
    print(rep)
    assert eng.he_arrival_counters_nonzero() == 0
    eng.he_destroy()


def test_fp8_config_errors():
    d = synth.ModelDims("x", 1, 128, 2, 128, 300, 64, 2, 8, 4, "f32", "greedy")
    with pytest.raises(binding.HeError):
        binding.Engine(binding.make_config(d, weights_fp8=1), binding.upload_weights(synth.make_weights(d, seed=1), "f32"))
    d = synth.ModelDims("x", 1, 128, 2, 128, 300, 64, 2, 8, 4, "bf16", "greedy")
    eng = binding.Engine(binding.make_config(d, weights_fp8=1), binding.upload_weights(synth.make_weights(d, seed=1), "bf16"))
    arr = (binding.he_lora_layer * 1)()
    assert binding.lib().he_refresh_weights_lora(eng.handle, arr, 4, 1.0) == binding.HE_ERR_STATE
    eng.he_refresh_weights()  # re-quantises
    eng.he_destroy()
