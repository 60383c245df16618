"""CPU oracle for the actor's experience-generation phase (TEST INFRASTRUCTURE).

This file is the slow, plain definition of what the HIP engine must compute.
Only tests, the smoke check and the benchmark's `cpu_baseline` leg may import
it; the product never does.  It shares no code with the HIP path.

What the paper fixes (Section 4; Section 5.3 (I)): the actor model is run in
inference mode, first over the whole prompt, then once per generated token
with the keys/values of earlier positions kept in a cache; exactly `G` tokens
are produced after an `S`-token prompt.  The paper names the model family
(OPT, Section 2 and Tables 1-3) but prints none of its equations, so the
decoder below is the published OPT architecture as the benchmark definition
constrains it: pre-LayerNorm, learned absolute positions, multi-head causal
self-attention with biases, ReLU feed-forward, a final LayerNorm and an LM
head that may be tied to the token embedding.

All arithmetic is float64 (numpy); `@` (BLAS matmul) is the only library
primitive.  A KV-cached decode reaches, up to rounding order, exactly the
result of the cache-free forward, so `forward_full` IS the definition and
`CachedDecoder` is checked against it in the tests.

Pins (tests/test_oracle_*.py): cached == cache-free; softmax rows sum to 1;
causal exactness; closed forms for degenerate weights; every primitive against
torch's float64 CPU routine; whole model against an independently written
OPT implementation (transformers, random init); Philox known-answer vectors;
Gumbel-max token frequencies against softmax; bfloat16 and half rounding against
torch's conversions; the scoring pass against that same independent
implementation's cross-entropy, a uniform-logits closed form, normalisation
over every possible next token, and the log-probabilities `generate` reports.  The bf16 tolerance (2e-2) is fixed by the benchmark
definition, not by the paper: parity unpinned for that number only.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64

# --------------------------------------------------------------------------
# primitives
# --------------------------------------------------------------------------


def layer_norm(u, gamma, beta, eps):
    """(u - mean) / sqrt(biased variance + eps) * gamma + beta over the last axis."""
    u = np.asarray(u, F64)
    mu = u.mean(axis=-1, keepdims=True)
    var = ((u - mu) ** 2).mean(axis=-1, keepdims=True)
    return (u - mu) / np.sqrt(var + eps) * np.asarray(gamma, F64) + np.asarray(beta, F64)


def linear(x, W, b=None):
    """y = x W^T + b with W stored [out, in]."""
    y = np.asarray(x, F64) @ np.asarray(W, F64).T
    if b is not None:
        y = y + np.asarray(b, F64)
    return y


def softmax_masked(s, allowed):
    """Row softmax over the allowed entries only; the others get probability 0."""
    s = np.where(allowed, s, -np.inf)
    m = s.max(axis=-1, keepdims=True)
    e = np.exp(s - m)  # exp(-inf) == 0 exactly
    return e / e.sum(axis=-1, keepdims=True)


def attention(q, k, v, q_pos):
    """One head.  q [Tq,d] (already scaled) sits at absolute positions q_pos[i];
    k, v [Tk,d] sit at positions 0..Tk-1.  Query i sees keys j <= q_pos[i]."""
    s = q @ k.T
    allowed = np.arange(k.shape[0])[None, :] <= np.asarray(q_pos)[:, None]
    p = softmax_masked(s, allowed)
    return p @ v, p


def round_bf16(x):
    """Nearest bfloat16 (8 significant bits, ties to even) of float64 values, returned
    as float64: the format the bf16 configuration's weights are given in (used where
    a weight is formed here: LoRA merge, 8-bit dequantisation checks).  (Values are
    assumed to lie in bfloat16's normal range.)"""
    u = np.ascontiguousarray(x, F64).view(np.uint64)
    drop = np.uint64(45)  # 52 fraction bits -> 7
    half = ((u >> drop) & np.uint64(1)) + np.uint64((1 << 44) - 1)
    r = (u + half) & ~np.uint64((1 << 45) - 1)
    return r.view(F64)


def round_f16(x):
    """Nearest IEEE half (11 significant bits, subnormals below 2^-14, ties to even) of
    float64 values, returned as float64; magnitudes above 65504 + 16 become infinite.
    DIAGNOSTIC ONLY: lets a test separate what an implementation's half-precision KV
    cache costs from everything else (kv_dtype="f16" below).  The definition the
    parity tests hold an implementation to keeps keys and values unrounded."""
    with np.errstate(over="ignore"):  # beyond the format's range: infinity, as the format says
        return np.asarray(x, F64).astype(np.float16).astype(F64)


def merge_lora(W, A, B, scale, exact=False):
    """Weights with a low-rank adapter folded in, as stored for generation:
    bf16(W + scale * B A), W [out,in], A [rank,in], B [out,rank] (Section 4: the
    actor is trained with LoRA and generates with the inference kernels, which
    see one dense matrix per linear layer).

    The sum decides a bf16 rounding, so it is taken in the precision the engine
    takes it in, float32, in this order: t = sum over j = 0..rank-1 of B[:,j] A[j,:]
    (each product exact for bf16 inputs, added one by one), then W + scale * t, each
    operation rounded to float32; the result is rounded to nearest-even bf16.
    exact=True: the plain definition instead, W + scale * (B @ A) in float64 rounded
    once to bf16 (the two differ by one bf16 step where the float32 sum falls on the
    other side of a rounding boundary).
    Returns float64 holding the bf16 values."""
    if exact:
        return round_bf16(np.asarray(W, F64) + float(scale) * (np.asarray(B, F64) @ np.asarray(A, F64)))
    W32, A32, B32 = (np.asarray(x, np.float32) for x in (W, A, B))
    t = np.zeros_like(W32)
    for j in range(A32.shape[0]):
        t = t + B32[:, j:j + 1] * A32[j:j + 1, :]
    return round_bf16((W32 + np.float32(scale) * t).astype(F64))


def e4m3_round(x):
    """Nearest OCP FP8 E4M3 value (the published 8-bit format: 1 sign, 4 exponent bits with bias 7,
    3 mantissa bits, subnormals, largest finite value 448, no infinities), ties to even, for
    |x| <= 448.  Returns (values float64, codes uint8)."""
    x = np.asarray(x, F64)
    a = np.abs(x)
    # exponent of the binade, clamped to the smallest normal one (below it the spacing stays 2^-9)
    e = np.floor(np.log2(np.maximum(a, 2.0 ** -20)))
    e = np.clip(e, -6, 8)
    step = 2.0 ** (e - 3)
    q = np.rint(a / step)  # numpy rounds half to even
    val = q * step         # q == 16 carries into the next binade by itself
    assert np.all(val <= 448.0)
    # encode
    ee = np.floor(np.log2(np.maximum(val, 2.0 ** -20)))
    normal = val >= 2.0 ** -6
    ee = np.where(normal, ee, -6)
    man = np.where(normal, val / 2.0 ** ee * 8 - 8, val / 2.0 ** -9)
    code = (np.where(normal, ee + 7, 0).astype(np.int64) << 3) | man.astype(np.int64)
    code = code | (np.signbit(x).astype(np.int64) << 7)
    return np.where(np.signbit(x), -val, val), code.astype(np.uint8)


def quantize_e4m3_rows(W):
    """Weights as stored for 8-bit streaming: row n of W [out,in] becomes q[n,:] * 2^e[n] with q
    in OCP FP8 E4M3 and e[n] the smallest integer for which the row's largest magnitude fits,
    max|W[n,:]| * 2^-e[n] <= 448 (e = 0 for an all-zero row); q = nearest E4M3 value of W * 2^-e,
    ties to even.  Scaling by a power of two is exact, so the only rounding is the one to E4M3,
    and the dequantised weights q * 2^e are bf16 values again (four significant bits).
    (An extension in the direction of Section 5.3 (I): generation is bound by the bytes read per
    token; the paper itself streams 16-bit weights.)
    Returns (dequantised weights float64 [out,in], codes uint8 [out,in], e int32 [out])."""
    W = np.asarray(W, F64)
    amax = np.abs(W).max(axis=1)
    f, x = np.frexp(amax)  # amax = f * 2^x, f in [0.5, 1); 448 = 0.875 * 2^9
    e = np.where(amax == 0, 0, np.where(f <= 0.875, x - 9, x - 8)).astype(np.int32)
    vals, codes = e4m3_round(W * 2.0 ** (-e[:, None].astype(F64)))
    return vals * 2.0 ** e[:, None].astype(F64), codes, e


def log_softmax(z):
    m = z.max(axis=-1, keepdims=True)
    return z - (m + np.log(np.exp(z - m).sum(axis=-1, keepdims=True)))


# --------------------------------------------------------------------------
# the decoder
# --------------------------------------------------------------------------


def _layer(x, lw, n_heads, eps, k_past, v_past, pos0, kv_dtype="f64"):
    """One pre-LN decoder layer over x [B,M,H] whose rows sit at positions
    pos0..pos0+M-1; k_past/v_past [B,pos0,H] are earlier positions (or None).
    kv_dtype "f64" is the definition.  "f16" is a diagnostic: keys and values are
    rounded to IEEE half when stored and every query (the row's own included) reads
    them back from there.  Returns (x_out, k_all, v_all)."""
    B, M, H = x.shape
    d = H // n_heads
    a = layer_norm(x, lw["ln1_g"], lw["ln1_b"], eps)
    qkv = linear(a, lw["wqkv"], lw["bqkv"])
    q = qkv[..., 0:H] * d ** -0.5
    k = qkv[..., H:2 * H]
    v = qkv[..., 2 * H:3 * H]
    if kv_dtype == "f16":
        k, v = round_f16(k), round_f16(v)
    elif kv_dtype != "f64":
        raise ValueError(kv_dtype)
    if k_past is not None:
        k = np.concatenate([k_past, k], axis=1)
        v = np.concatenate([v_past, v], axis=1)
    q_pos = pos0 + np.arange(M)
    o = np.empty((B, M, H), F64)
    for b in range(B):
        for h in range(n_heads):
            sl = slice(h * d, (h + 1) * d)
            o[b, :, sl], _ = attention(q[b, :, sl], k[b, :, sl], v[b, :, sl], q_pos)
    x = x + linear(o, lw["wo"], lw["bo"])
    a2 = layer_norm(x, lw["ln2_g"], lw["ln2_b"], eps)
    hdn = np.maximum(linear(a2, lw["w1"], lw["b1"]), 0.0)
    x = x + linear(hdn, lw["w2"], lw["b2"])
    return x, k, v


def embed(w, ids, pos0, pos_offset):
    ids = np.asarray(ids)
    M = ids.shape[1]
    tok = np.asarray(w["tok_emb"], F64)[ids]
    pos = np.asarray(w["pos_emb"], F64)[pos_offset + pos0 + np.arange(M)]
    return tok + pos[None, :, :]


def lm_logits(w, x, eps):
    xf = layer_norm(x, w["lnf_g"], w["lnf_b"], eps)
    return linear(xf, w["lm_head"])


def forward_full(w, ids, n_heads, eps=1e-5, pos_offset=0, kv_dtype="f64"):
    """Cache-free forward over ids [B,T]: logits [B,T,V] at every position."""
    x = embed(w, ids, 0, pos_offset)
    for lw in w["layers"]:
        x, _, _ = _layer(x, lw, n_heads, eps, None, None, 0, kv_dtype)
    return lm_logits(w, x, eps)


def score(w, ids, n_heads, eps=1e-5, pos_offset=0, kv_dtype="f64"):
    """Log-probability the model gives each token of ids [B,T] after its prefix:
    out[b,t] = log_softmax(logits[b,t,:])[ids[b,t+1]], t = 0..T-2 -> [B,T-1].

    This is the pass that follows generation in the inference phase of an RLHF
    iteration (Section 4: that phase produces the inputs of the training phase;
    Section 5.3 (I) counts it with the generation phase): the prompt-plus-answer
    sequence goes once through the model and the log-probabilities of the tokens
    that are actually there are read off.  No cache, no sampling: the cache-free
    forward, log-softmax, gather."""
    ids = np.asarray(ids)
    lp = log_softmax(forward_full(w, ids, n_heads, eps, pos_offset, kv_dtype))
    return np.take_along_axis(lp[:, :-1, :], ids[:, 1:, None].astype(np.int64), axis=2)[:, :, 0]


class CachedDecoder:
    """Prefill + one-token steps with per-layer K/V kept for earlier positions."""

    def __init__(self, w, n_heads, eps=1e-5, pos_offset=0, kv_dtype="f64"):
        self.w, self.n_heads, self.eps, self.pos_offset = w, n_heads, eps, pos_offset
        self.kv_dtype = kv_dtype
        self.k = [None] * len(w["layers"])
        self.v = [None] * len(w["layers"])
        self.length = 0

    def _run(self, ids, all_positions):
        x = embed(self.w, ids, self.length, self.pos_offset)
        for i, lw in enumerate(self.w["layers"]):
            x, self.k[i], self.v[i] = _layer(x, lw, self.n_heads, self.eps, self.k[i], self.v[i], self.length,
                                             self.kv_dtype)
        self.length += np.asarray(ids).shape[1]
        if not all_positions:
            x = x[:, -1:, :]
        return lm_logits(self.w, x, self.eps)

    def prefill(self, ids, all_positions=False):
        """ids [B,S] -> logits of the last position [B,V] (or all [B,S,V])."""
        assert self.length == 0
        z = self._run(ids, all_positions)
        return z if all_positions else z[:, 0, :]

    def step(self, ids):
        """ids [B] (one new token per sequence) -> logits [B,V]."""
        return self._run(np.asarray(ids).reshape(-1, 1), False)[:, 0, :]


# --------------------------------------------------------------------------
# counter-based RNG and sampling
# --------------------------------------------------------------------------

_PHILOX_M0 = np.uint64(0xD2511F53)
_PHILOX_M1 = np.uint64(0xCD9E8D57)
_PHILOX_W0 = 0x9E3779B9
_PHILOX_W1 = 0xBB67AE85
_MASK32 = np.uint64(0xFFFFFFFF)


def philox4x32_10(c0, c1, c2, c3, k0, k1):
    """Philox-4x32 with 10 rounds (Salmon et al., SC'11).  Counter words c0..c3
    and key words k0,k1 are uint32 (arrays broadcast); returns 4 uint32 arrays."""
    c0, c1, c2, c3 = (np.asarray(c, np.uint64) & _MASK32 for c in (c0, c1, c2, c3))
    k0 = int(k0) & 0xFFFFFFFF
    k1 = int(k1) & 0xFFFFFFFF
    for r in range(10):
        p0 = _PHILOX_M0 * c0  # 32x32 -> 64 bit products, exact in uint64
        p1 = _PHILOX_M1 * c2
        hi0, lo0 = p0 >> np.uint64(32), p0 & _MASK32
        hi1, lo1 = p1 >> np.uint64(32), p1 & _MASK32
        c0, c1, c2, c3 = (hi1 ^ c1 ^ np.uint64(k0)), lo1, (hi0 ^ c3 ^ np.uint64(k1)), lo0
        k0 = (k0 + _PHILOX_W0) & 0xFFFFFFFF
        k1 = (k1 + _PHILOX_W1) & 0xFFFFFFFF
    return tuple(c.astype(np.uint32) for c in (c0, c1, c2, c3))


def random_u32(seed, b, n, v):
    """The engine's random word for (sequence b, generation step n, vocab id v):
    word 0 of Philox4x32-10 with counter (v, n, b, 0) and key (seed lo, seed hi)."""
    seed = int(seed) & 0xFFFFFFFFFFFFFFFF
    return philox4x32_10(v, n, b, 0, seed & 0xFFFFFFFF, seed >> 32)[0]


def uniform_open(x_u32):
    """u = ((x >> 9) + 1/2) * 2^-23, strictly inside (0,1), exact in fp32."""
    return ((np.asarray(x_u32, np.uint32) >> np.uint32(9)).astype(F64) + 0.5) * 2.0 ** -23


def gumbel_noise(seed, b, n, V):
    """g_v = -log(-log(u_v)) for v = 0..V-1."""
    u = uniform_open(random_u32(seed, b, n, np.arange(V, dtype=np.uint32)))
    return -np.log(-np.log(u))


def sample(z, mode, temperature, seed, n, rows=None):
    """z [B,V] logits of generation step n; row i is sequence rows[i] of the
    batch (default i) -- the noise is keyed by that number.  Returns (tok int32 [B],
    logprob [B], margin [B], second int32 [B]): greedy takes argmax z; 'gumbel' takes
    argmax(z/temperature + g).  Ties go to the lowest index.  logprob is the
    untempered log-softmax of z at tok; margin is the gap between the best and
    second-best arg-maxed score (ids are only unique where it is large) and second
    the id of that second-best score (-1 when the vocabulary has one entry)."""
    z = np.asarray(z, F64)
    B, V = z.shape
    lp = log_softmax(z)
    tok = np.empty(B, np.int32)
    second = np.full(B, -1, np.int32)
    margin = np.empty(B, F64)
    for b in range(B):
        if mode == "greedy":
            score = z[b]
        elif mode == "gumbel":
            score = z[b] / temperature + gumbel_noise(seed, b if rows is None else rows[b], n, V)
        else:
            raise ValueError(mode)
        t = int(np.argmax(score))  # first maximum = lowest index
        tok[b] = t
        if V > 1:
            rest = score.copy()
            rest[t] = -np.inf
            second[b] = int(np.argmax(rest))
            margin[b] = score[t] - rest[second[b]]
        else:
            margin[b] = np.inf
    return tok, lp[np.arange(B), tok], margin, second


def generate(w, prompt_ids, G, n_heads, mode="greedy", temperature=1.0, seed=0,
             eps=1e-5, pos_offset=0, forced_ids=None, kv_dtype="f64"):
    """Prefill the prompt [B,S], then G-1 cached steps: exactly G tokens, no
    stop token.  Token 0 comes from the prompt's last position.  If forced_ids
    [B,G] is given, those ids are fed forward instead of the sampled ones
    (teacher forcing) while the sampled ids are still reported.

    Returns dict(ids [B,G], logprobs [B,G], margins [B,G], second [B,G] (the runner-up
    ids), logits [G,B,V])."""
    prompt_ids = np.asarray(prompt_ids)
    B = prompt_ids.shape[0]
    dec = CachedDecoder(w, n_heads, eps, pos_offset, kv_dtype)
    ids = np.empty((B, G), np.int32)
    sec = np.empty((B, G), np.int32)
    lps = np.empty((B, G), F64)
    mar = np.empty((B, G), F64)
    logits = []
    z = dec.prefill(prompt_ids)
    for n in range(G):
        logits.append(z)
        ids[:, n], lps[:, n], mar[:, n], sec[:, n] = sample(z, mode, temperature, seed, n)
        if n + 1 < G:
            feed = ids[:, n] if forced_ids is None else np.asarray(forced_ids)[:, n]
            z = dec.step(feed)
    return {"ids": ids, "logprobs": lps, "margins": mar, "second": sec, "logits": np.stack(logits)}


def generate_ragged(w, prompts, G, n_heads, mode="greedy", temperature=1.0, seed=0, eos_id=-1, pad_id=0,
                    eps=1e-5, pos_offset=0, forced_ids=None, kv_dtype="f64"):
    """Prompts of different lengths and answers that may end early.

    The benchmark setting pads or cuts every prompt to one length and lets every
    answer run to the cap (Section 5.3 (I): 256 and 256 tokens); real prompts are
    shorter than the cap and sit right-aligned behind padding, and an answer is
    over once the end-of-sequence token has been produced.  Padding is not part of
    a sequence: what the model computes for sequence b is, by definition, what it
    computes for that sequence's own tokens alone, at positions 0, 1, 2, ...  So
    each sequence is run by itself here, on its unpadded prompt; only its row
    number b enters, through the sampling noise.

    prompts: list of B one-dimensional id arrays (length >= 1).  After the step
    that samples eos_id (eos_id < 0: never) a sequence produces nothing more: its
    remaining ids are pad_id and their log-probabilities 0.  forced_ids [B,G]
    feeds those ids forward instead of the sampled ones (the stop still follows
    the fed id).

    Returns dict(ids [B,G], logprobs [B,G], margins [B,G] (inf where nothing was
    sampled), second [B,G] (runner-up ids, -1 where nothing was sampled), lens [B] =
    tokens produced including the end token, logits = list over b of [lens[b], V])."""
    B = len(prompts)
    ids = np.full((B, G), pad_id, np.int32)
    sec = np.full((B, G), -1, np.int32)
    lps = np.zeros((B, G), F64)
    mar = np.full((B, G), np.inf, F64)
    lens = np.zeros(B, np.int32)
    logits = []
    for b, prompt in enumerate(prompts):
        dec = CachedDecoder(w, n_heads, eps, pos_offset, kv_dtype)
        z = dec.prefill(np.asarray(prompt).reshape(1, -1))
        zs = []
        for n in range(G):
            zs.append(z[0])
            tok, lp, m, s2 = sample(z, mode, temperature, seed, n, rows=[b])
            ids[b, n], lps[b, n], mar[b, n], sec[b, n] = tok[0], lp[0], m[0], s2[0]
            lens[b] = n + 1
            feed = tok[0] if forced_ids is None else int(np.asarray(forced_ids)[b, n])
            if feed == eos_id or n + 1 == G:
                break
            z = dec.step(np.array([feed]))
        logits.append(np.stack(zs))
    return {"ids": ids, "logprobs": lps, "margins": mar, "second": sec, "lens": lens, "logits": logits}
