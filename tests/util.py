"""Shared helpers of the GPU parity tests: run the engine teacher-forced on the
oracle's token ids so that every step is comparable, then compare per step."""
import numpy as np

from oracle import opt_oracle as O
from paper_2308_01320_amd import binding, synth


def oracle_run(d, w, prompts, G, mode, temperature=1.0, seed=0, kv_dtype=None):
    """The oracle on the configuration's own storage formats: weights as given (already
    bf16-representable for dtype bf16) and a bf16 KV cache for dtype bf16."""
    if kv_dtype is None:
        kv_dtype = "bf16" if d.dtype == "bf16" else "f64"
    return O.generate(w, prompts, G, d.n_heads, mode=mode, temperature=temperature, seed=seed,
                      eps=d.ln_eps, pos_offset=d.pos_offset, kv_dtype=kv_dtype)


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
    """Logits / log-probs within logit_tol (max-abs); ids equal wherever the oracle's
    top-2 margin of the arg-maxed score exceeds id_margin, else either of the
    oracle's two best is accepted (checked through the logit tolerance)."""
    err = float(np.abs(got["logits"] - want["logits"]).max())
    assert err <= logit_tol, f"logits max-abs error {err} > {logit_tol}"
    sure = want["margins"] > id_margin
    bad = (got["ids"] != want["ids"]) & sure
    assert not bad.any(), f"{int(bad.sum())} token ids differ at margin > {id_margin}"
    same = got["ids"] == want["ids"]
    lp_err = float(np.abs(got["logprobs"] - want["logprobs"])[same].max()) if same.any() else 0.0
    assert lp_err <= logit_tol, f"logprob max-abs error {lp_err} > {logit_tol}"
    return {"logit_err": err, "logprob_err": lp_err, "sure_frac": float(sure.mean()),
            "id_match": float(same.mean())}


def make_engine(d, w_np, max_batch=None, max_seq_len=None, impl=0):
    w_dev = binding.upload_weights(w_np, d.dtype)
    cfg = binding.make_config(d, max_batch=max_batch, max_seq_len=max_seq_len, impl=impl)
    return binding.Engine(cfg, w_dev)
