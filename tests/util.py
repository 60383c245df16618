"""Shared helpers of the GPU parity tests: run the engine teacher-forced on the
oracle's token ids so that every step is comparable, then compare per step."""
import numpy as np

from oracle import opt_oracle as O
from paper_2308_01320_amd import binding, synth


def oracle_run(d, w, prompts, G, mode, temperature=1.0, seed=0, kv_dtype="f64"):
    """The oracle's definition on the configuration's weights (already bf16-representable for dtype
    bf16): float64 arithmetic, keys and values unrounded.  kv_dtype="f16" is the diagnostic run that
    rounds the cache to half as the tuned bf16 path stores it."""
    return O.generate(w, prompts, G, d.n_heads, mode=mode, temperature=temperature, seed=seed,
                      eps=d.ln_eps, pos_offset=d.pos_offset, kv_dtype=kv_dtype)


def weights_f64(w):
    """The same weight dict as float64 arrays (a tied head stays tied): the oracle's matmuls then run in float64."""
    out = {k: (v.astype(np.float64) if k != "layers" else [{n: a.astype(np.float64) for n, a in lw.items()} for lw in v])
           for k, v in w.items()}
    if w["lm_head"] is w["tok_emb"]:
        out["lm_head"] = out["tok_emb"]
    return out


def engine_teacher_forced(eng, prompts_np, forced_ids, G, samp):
    """Returns dict(ids [B,G], logprobs [B,G], logits [G,B,V]) from he_prefill + he_decode_step."""
    import torch
    dev = eng.device
    p = torch.from_numpy(prompts_np).to(dev)
    eng.he_reset()
    ids, lps, lgs = [], [], []
    i, lp, lg = eng.he_prefill(p, samp, want_logits=True)
    for n in range(G):
        ids.append(i), lps.append(lp), lgs.append(lg)
        if n + 1 < G:
            feed = torch.from_numpy(np.ascontiguousarray(forced_ids[:, n])).to(dev)
            i, lp, lg = eng.he_decode_step(feed, samp, want_logits=True)
    torch.cuda.synchronize()
    return {"ids": torch.stack(ids, 1).cpu().numpy(), "logprobs": torch.stack(lps, 1).cpu().numpy(),
            "logits": torch.stack(lgs, 0).cpu().numpy()}


def compare(got, want, logit_tol, id_margin):
    """Logits / log-probs within logit_tol (max-abs).  Token ids: equal to the oracle's wherever the
    oracle's top-2 margin of the arg-maxed score exceeds id_margin; at the remaining (thin-margin) steps
    the engine's id must be one of the oracle's two best."""
    err = float(np.abs(got["logits"] - want["logits"]).max())
    assert err <= logit_tol, f"logits max-abs error {err} > {logit_tol}"
    sure = want["margins"] > id_margin
    same = got["ids"] == want["ids"]
    bad = ~same & sure
    assert not bad.any(), f"{int(bad.sum())} token ids differ at margin > {id_margin}"
    runner_up = got["ids"] == want["second"]
    assert (same | runner_up).all(), "a thin-margin token id is neither of the oracle's two best"
    lp_err = float(np.abs(got["logprobs"] - want["logprobs"])[same].max()) if same.any() else 0.0
    assert lp_err <= logit_tol, f"logprob max-abs error {lp_err} > {logit_tol}"
    return {"logit_err": err, "logprob_err": lp_err, "sure_frac": float(sure.mean()),
            "id_match": float(same.mean())}


def make_engine(d, w_np, max_batch=None, max_seq_len=None, impl=0):
    w_dev = binding.upload_weights(w_np, d.dtype)
    cfg = binding.make_config(d, max_batch=max_batch, max_seq_len=max_seq_len, impl=impl)
    return binding.Engine(cfg, w_dev)
