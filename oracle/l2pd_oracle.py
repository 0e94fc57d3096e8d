"""CPU oracle for the Learn2PD decoding loop (arXiv 2509.25188).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
decoding path computes.  Only the test-suite, the smoke check and the
CPU-baseline leg of the benchmark may import it; the product path never does,
and this file imports nothing from the product.

What it states, in the paper's order and notation:

* the mask predictor M(X) -> logits.  The paper treats the dLLM as a black box
  (Sec. 3.1.1, "mask predictor p_theta"; Alg. 2, "conf, pre = M(X)"); the
  architecture here is the LLaDA-style family of the workloads: pre-norm
  transformer, RMSNorm, rotary position embedding, bidirectional (unmasked)
  softmax attention, SwiGLU FFN, untied LM head, no biases;
* greedy estimate  pre_j = argmax_v p_theta(v | X)        (Eq. 3);
* confidence       conf_j = p_theta(pre_j | X)            (Eq. 4);
* the filter       p = sigmoid(f_theta(conf)), f_theta a two-layer MLP on the
  block's confidence vector (Sec. 3.2; Sec. 4.1: 2,112 parameters at block 32);
  the single- and four-layer filters of Table 3 are read as the same MLP with
  no, resp. three, hidden layers (ReLU between layers; the paper gives no widths);
* the inference loop: blocks left to right, `while M != {}` per block, unmask j
  when p_j > tau (Alg. 2);
* End-of-Text Prediction: after a block's loop ends, stop if an end-of-text
  token is in the response (Alg. 3, Appendix A; Fig. 4 caption);
* step-granular End-of-Text Prediction (Sec. 3.3, the text, as opposed to the
  block-granular Alg. 3): after every step, once the response holds an
  end-of-text token, everything after its first occurrence is discarded and
  the next step runs on the shortened sequence;
* the Extremely Greedy Parallel rollout that labels training data (Sec. 3.1.3,
  Alg. 1 without its update line), the binary cross-entropy of Eq. 6 with its
  gradient for a filter of any depth, and AdamW (Sec. 4.1 names the optimiser,
  learning rate 1e-3 and 5,000 epochs; the update rule is the published one);
* the prefix KV cache variant (Sec. 4.3 names the technique only): K/V of the
  prompt and finished blocks come from a forward over that prefix alone and
  are refreshed once per block; a step recomputes only the active block;
* the dual KV cache variant (Sec. 4.3 and Table 2 name it and cite the work it
  comes from; the mechanism restated here is that work's): at each block start a
  full bidirectional forward over the whole current sequence stores every
  position's K/V per layer; a step recomputes only the active block, whose fresh
  K/V stand in for the stored ones at its positions, and attends to the stored
  K/V of everything before AND after the block, which stay as they were at the
  block start.

Readings of points the paper leaves open (each also listed in the design notes):
mask id excluded from the vocabulary distribution; ties -> lowest index;
already-committed block positions feed the filter the constant 1.0; the masked
position with the highest confidence is always unmasked (progress guarantee);
the end-of-text search covers the response region only; after an early stop
the undecoded tail keeps the mask id.  Step-granular EoTP: positions of the
active block after the first end-of-text leave the mask set undecoded; the
filter still takes block_len inputs and discarded positions enter as 1.0 like
committed ones; the block's loop ends when no masked position is left up to the
end-of-text; discarded positions come back as mask id, decoded_len counts the
response up to and including the end-of-text.  EGP / training: every one of
the block's positions is a training entry, committed ones as (1.0, label 1);
when no masked position's prediction equals the reference, the most confident
masked position takes the REFERENCE token with label 0 (Alg. 1 would not
terminate); one epoch is one full-batch AdamW step over all collected rows;
AdamW defaults beta = (0.9, 0.999), eps = 1e-8, weight decay 0.01.

Parity pins: every function below is pinned by tests/test_oracle_*.py against
brute-force loops, closed forms and invariants, except the whole trajectory on
a random-init model, for which the paper prints no worked example:
PARITY UNPINNED for `generate` beyond its invariants and special cases.

Precision: `dtype` is numpy float32 (default) or float64.  Weights given as
uint16 arrays are bf16 bit patterns and are widened exactly.  For bf16 models
("bf16 weights, fp32 accumulate") the model can also be evaluated with every
matrix-product INPUT rounded to bf16 (`gemm_input="bf16"`: normalised
activations, rotated q and k, v, softmax probabilities, attention output,
SwiGLU output), accumulation, residual stream, norms and softmax staying in
`dtype`.  That is the arithmetic a bf16 matrix unit performs; comparing against
both modes separates implementation error from the error of the number format.
"""
from __future__ import annotations

import numpy as np


# --------------------------------------------------------------------------- helpers
def widen(w, dtype):
    """Exact widening of a stored weight (float array, or uint16 bf16 bit patterns) to `dtype`."""
    w = np.asarray(w)
    if w.dtype == np.uint16:
        return (w.astype(np.uint32) << 16).view(np.float32).astype(dtype, copy=False)
    return w.astype(dtype, copy=False)


def round_bf16(x):
    """Round to the nearest bf16 value (ties to even), result kept in x's dtype."""
    a = np.ascontiguousarray(x, dtype=np.float32)
    u = a.view(np.uint32)
    r = ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)).view(np.float32)
    return r.astype(np.asarray(x).dtype, copy=False)


def rmsnorm(x, g, eps):
    """y = x / sqrt(mean(x^2) + eps) * g, along the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + x.dtype.type(eps)) * g


def rope(x, pos, base):
    """Rotary embedding, rotate-half pairing.

    x: [T, H, Dh]; pos: [T] absolute positions.  Feature pair (i, i + Dh/2)
    is rotated by the angle pos * base^(-2i/Dh).
    """
    dh = x.shape[-1]
    half = dh // 2
    i = np.arange(half, dtype=np.float64)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * base ** (-2.0 * i / dh)   # [T, half]
    cos = np.cos(ang).astype(x.dtype)[:, None, :]
    sin = np.sin(ang).astype(x.dtype)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * cos - x2 * sin, x2 * cos + x1 * sin], axis=-1)


def softmax(z, axis=-1):
    z = z - np.max(z, axis=axis, keepdims=True)
    e = np.exp(z)
    return e / np.sum(e, axis=axis, keepdims=True)


def attention(q, k, v, rin=None):
    """Bidirectional attention.  q: [Tq, H, Dh]; k, v: [Tk, H, Dh] -> [Tq, H, Dh].

    Every query sees every key: there is no causal mask (the dLLM refines the
    whole sequence at once, Sec. 1).  `rin`, if given, rounds the probabilities
    before they enter the product with v.
    """
    dh = q.shape[-1]
    qh, kh, vh = (np.transpose(a, (1, 0, 2)) for a in (q, k, v))                  # per head: [H, T, Dh]
    s = np.matmul(qh, np.transpose(kh, (0, 2, 1))) / q.dtype.type(np.sqrt(dh))    # scores [H, Tq, Tk]
    p = softmax(s, axis=-1)
    if rin is not None:
        p = rin(p)
    return np.transpose(np.matmul(p, vh), (1, 0, 2))                              # [Tq, H, Dh]


def silu(x):
    return x / (1.0 + np.exp(-x))


def sigmoid(x):
    with np.errstate(over="ignore"):        # exp(-x) may overflow to inf for very negative x: the result is then 0, as it should be
        return 1.0 / (1.0 + np.exp(-x))


# --------------------------------------------------------------------------- mask predictor M(X)
class Model:
    """The mask predictor.  `shape` needs n_layers, d_model, n_heads, head_dim, rope_base, rms_eps;
    `weights` maps tensor names to arrays ([out, in] row-major matrices)."""

    def __init__(self, shape, weights, dtype=np.float32, gemm_input="fp32"):
        self.s = shape
        self.w = weights
        self.dtype = np.dtype(dtype)
        assert gemm_input in ("fp32", "bf16")
        self.rin = round_bf16 if gemm_input == "bf16" else (lambda x: x)
        self.p_rin = round_bf16 if gemm_input == "bf16" else None

    def W(self, name):
        return widen(self.w[name], self.dtype)

    def embed(self, tokens):
        tok = np.asarray(tokens, dtype=np.int64)
        e = self.w["tok_emb"]
        return widen(np.asarray(e)[tok], self.dtype)

    def qkv(self, l, h, pos):
        """Layer l's rotated queries/keys and values for hidden rows h at positions pos."""
        s, p = self.s, f"layers.{l}."
        a = self.rin(rmsnorm(h, self.W(p + "attn_norm_g"), s.rms_eps))
        t = a.shape[0]
        q = (a @ self.W(p + "wq").T).reshape(t, s.n_heads, s.head_dim)
        k = (a @ self.W(p + "wk").T).reshape(t, s.n_heads, s.head_dim)
        v = (a @ self.W(p + "wv").T).reshape(t, s.n_heads, s.head_dim)
        return self.rin(rope(q, pos, s.rope_base)), self.rin(rope(k, pos, s.rope_base)), self.rin(v)

    def finish_layer(self, l, h, o):
        """Attention output projection + residual, then the SwiGLU FFN + residual."""
        p = f"layers.{l}."
        h = h + self.rin(o.reshape(h.shape[0], -1)) @ self.W(p + "wo").T
        f = self.rin(rmsnorm(h, self.W(p + "ffn_norm_g"), self.s.rms_eps))
        act = self.rin(silu(f @ self.W(p + "w_gate").T) * (f @ self.W(p + "w_up").T))
        return h + act @ self.W(p + "w_down").T

    def head(self, h_rows):
        return self.rin(rmsnorm(h_rows, self.W("final_norm_g"), self.s.rms_eps)) @ self.W("lm_head").T

    def forward(self, tokens, row_begin=0, row_count=None):
        """logits[row_count, V] of one sequence `tokens` [T]; full bidirectional forward."""
        t = len(tokens)
        if row_count is None:
            row_count = t - row_begin
        pos = np.arange(t)
        h = self.embed(tokens)
        for l in range(self.s.n_layers):
            q, k, v = self.qkv(l, h, pos)
            h = self.finish_layer(l, h, attention(q, k, v, self.p_rin))
        return self.head(h[row_begin:row_begin + row_count])

    # ---- prefix KV cache (Sec. 4.3) ----
    def prefix_kv(self, tokens_prefix):
        """Per-layer (K, V) of a forward over the prefix alone (nothing after it is visible)."""
        c = len(tokens_prefix)
        pos = np.arange(c)
        h = self.embed(tokens_prefix)
        cache = []
        for l in range(self.s.n_layers):
            q, k, v = self.qkv(l, h, pos)
            cache.append((k, v))
            if l + 1 < self.s.n_layers:
                h = self.finish_layer(l, h, attention(q, k, v, self.p_rin))
        return cache

    def forward_block_cached(self, cache, block_tokens, c):
        """logits[s, V] for the active block at positions c..c+s-1: its queries attend to the
        cached prefix keys/values plus the block's own, and to nothing after the block."""
        n = len(block_tokens)
        pos = np.arange(c, c + n)
        h = self.embed(block_tokens)
        for l in range(self.s.n_layers):
            q, k, v = self.qkv(l, h, pos)
            kc, vc = cache[l]
            o = attention(q, np.concatenate([kc, k], axis=0), np.concatenate([vc, v], axis=0), self.p_rin)
            h = self.finish_layer(l, h, o)
        return self.head(h)


    # ---- dual KV cache (Sec. 4.3, Table 2) ----
    def full_kv(self, tokens):
        """Per-layer (K, V) of every position, from a full bidirectional forward over `tokens`."""
        t = len(tokens)
        pos = np.arange(t)
        h = self.embed(tokens)
        cache = []
        for l in range(self.s.n_layers):
            q, k, v = self.qkv(l, h, pos)
            cache.append((k, v))
            if l + 1 < self.s.n_layers:
                h = self.finish_layer(l, h, attention(q, k, v, self.p_rin))
        return cache

    def forward_block_dual(self, cache, block_tokens, c):
        """logits[s, V] for the active block at positions c..c+s-1: its queries attend to every
        position of the sequence; keys/values of the block's own positions are recomputed from
        `block_tokens`, all others are the stored ones."""
        n = len(block_tokens)
        pos = np.arange(c, c + n)
        h = self.embed(block_tokens)
        for l in range(self.s.n_layers):
            q, k, v = self.qkv(l, h, pos)
            kc, vc = cache[l]
            kk = np.array(kc, copy=True)
            vv = np.array(vc, copy=True)
            kk[c:c + n] = k
            vv[c:c + n] = v
            h = self.finish_layer(l, h, attention(q, kk, vv, self.p_rin))
        return self.head(h)


# --------------------------------------------------------------------------- Eq. 3, Eq. 4
def conf_pre(logits, mask_id):
    """pre_j = argmax_v p(v) (Eq. 3) and conf_j = p(pre_j) (Eq. 4) over the data vocabulary.

    The mask token is not a data token, so its logit is removed from the distribution.
    Ties go to the lowest token id.
    """
    z = np.array(logits, copy=True)
    z[:, mask_id] = -np.inf
    pre = np.argmax(z, axis=-1)           # numpy returns the first maximum
    p = softmax(z, axis=-1)
    conf = p[np.arange(len(pre)), pre]
    return conf.astype(logits.dtype), pre.astype(np.int64)


# --------------------------------------------------------------------------- filter f_theta (Sec. 3.2)
def filter_depth(flt):
    """Number of layers of a filter given as {"w1", "b1", ..., "wN", "bN"}."""
    n = 0
    while f"w{n + 1}" in flt:
        n += 1
    assert n >= 1 and all(f"b{k}" in flt for k in range(1, n + 1))
    return n


def filter_prob(conf_in, flt):
    """The filter's output for the block's confidence vector c: an MLP with ReLU between its layers
    and a sigmoid at the end.  Two layers, sigmoid(W2 relu(W1 c + b1) + b2), is the paper's filter
    (Sec. 3.2, Sec. 4.1); one layer, sigmoid(W1 c + b1), and four are the variants of Table 3."""
    dt = conf_in.dtype
    n = filter_depth(flt)
    a = conf_in
    for k in range(1, n):
        a = np.maximum(widen(flt[f"w{k}"], dt) @ a + widen(flt[f"b{k}"], dt), 0)
    z = widen(flt[f"w{n}"], dt) @ a + widen(flt[f"b{n}"], dt)
    return sigmoid(z)


def filter_param_count(block_len, hidden, n_layers=2):
    dims = [block_len] + [hidden] * (n_layers - 1) + [block_len]
    return sum(dims[k + 1] * dims[k] + dims[k + 1] for k in range(n_layers))


# --------------------------------------------------------------------------- one denoising step (Alg. 2 loop body)
def apply_bias(logits, gen_pos0, bias):
    """Test hook of the workloads: add `value` to one token's logit at generation positions >= from."""
    if bias is None or bias[2] == 0.0:
        return logits
    token_id, pos_from, value = bias
    out = np.array(logits, copy=True)
    for j in range(out.shape[0]):
        if gen_pos0 + j >= pos_from:
            out[j, token_id] += out.dtype.type(value)
    return out


def decide(block_tokens, logits, mask_id, flt, tau):
    """Unmask decision of one step for one block.

    Returns dict(conf, pre, p, sel).  sel[j] is true when position j is unmasked now:
    it is masked and p_j > tau (strict), or it is the masked position of highest
    confidence (lowest index on ties), which is always taken so that the loop ends.
    """
    masked = np.asarray(block_tokens) == mask_id
    conf, pre = conf_pre(logits, mask_id)
    cin = np.where(masked, conf, conf.dtype.type(1.0))
    p = filter_prob(cin, flt)
    sel = masked & (p > p.dtype.type(tau))
    if masked.any():
        cm = np.where(masked, conf, -np.inf)
        sel[int(np.argmax(cm))] = True
    return dict(conf=conf, pre=pre, p=p, sel=sel, masked=masked)


def denoise_step(model, X, prompt_len, b, block_len, mask_id, flt, tau, bias=None, cache=None, dual=False):
    """One pass of the while-loop body of Alg. 2 for block b of sequence X (modified in place).
    `cache` is None (full recompute), a prefix cache, or with `dual` a dual cache."""
    lo = prompt_len + b * block_len
    if cache is None:
        logits = model.forward(X, lo, block_len)
    elif dual:
        logits = model.forward_block_dual(cache, X[lo:lo + block_len], lo)
    else:
        logits = model.forward_block_cached(cache, X[lo:lo + block_len], lo)
    logits = apply_bias(logits, b * block_len, bias)
    d = decide(X[lo:lo + block_len], logits, mask_id, flt, tau)
    for j in np.nonzero(d["sel"])[0]:
        X[lo + j] = d["pre"][j]
    d["logits"] = logits
    return d


# --------------------------------------------------------------------------- Sec. 3.3 (step-granular EoTP)
def first_eot(X, prompt_len, eos_id):
    """Index in X of the first end-of-text token of the response region, or None."""
    hit = np.nonzero(np.asarray(X[prompt_len:]) == eos_id)[0]
    return prompt_len + int(hit[0]) if len(hit) else None


def denoise_step_shortened(model, X, t_eff, prompt_len, b, block_len, mask_id, flt, tau, bias=None):
    """One step of block b on the shortened sequence X[0:t_eff] (X modified in place).  Only the
    n = min(block_len, t_eff - lo) positions of the block that still exist are predicted; the filter
    sees block_len inputs, the discarded ones as 1.0."""
    lo = prompt_len + b * block_len
    n = min(block_len, t_eff - lo)
    logits = model.forward(X[:t_eff], lo, n)
    logits = apply_bias(logits, b * block_len, bias)
    conf, pre = conf_pre(logits, mask_id)
    masked = np.asarray(X[lo:lo + n]) == mask_id
    cin = np.ones(block_len, dtype=conf.dtype)
    cin[:n] = np.where(masked, conf, conf.dtype.type(1.0))
    p = filter_prob(cin, flt)[:n]
    sel = masked & (p > p.dtype.type(tau))
    if masked.any():
        cm = np.where(masked, conf, -np.inf)
        sel[int(np.argmax(cm))] = True
    for j in np.nonzero(sel)[0]:
        X[lo + j] = pre[j]
    return dict(conf=conf, pre=pre, p=p, sel=sel, masked=masked, logits=logits, n=n)


def generate_eotp_step(model, prompt, gen_len, block_len, mask_id, eos_id, flt, tau, bias=None, trace=None):
    """Alg. 2 with the step-granular EoTP of Sec. 3.3 (full recompute).  Returns
    (response[gen_len], steps, decoded_len)."""
    assert gen_len % block_len == 0
    P = len(prompt)
    X = np.concatenate([np.asarray(prompt, dtype=np.int64), np.full(gen_len, mask_id, dtype=np.int64)])
    t_eff = P + gen_len
    steps = 0
    for b in range(gen_len // block_len):
        lo = P + b * block_len
        while np.any(X[lo:min(lo + block_len, t_eff)] == mask_id):
            before = X.copy() if trace is not None else None
            d = denoise_step_shortened(model, X, t_eff, P, b, block_len, mask_id, flt, tau, bias)
            steps += 1
            if trace is not None:
                d.update(X_before=before, block=b, t_eff=t_eff)
                trace.append(d)
            e = first_eot(X[:t_eff], P, eos_id)
            if e is not None:
                t_eff = e + 1                     # everything after the first end-of-text is discarded
        if first_eot(X[:t_eff], P, eos_id) is not None:
            break
    resp = X[P:P + gen_len].copy()
    resp[t_eff - P:] = mask_id
    return resp, steps, t_eff - P


# --------------------------------------------------------------------------- Alg. 2 / Alg. 3
def generate(model, prompt, gen_len, block_len, mask_id, eos_id, flt, tau, eotp=False,
             bias=None, prefix_cache=False, trace=None, dual_cache=False):
    """Decode one prompt.  Returns (response[gen_len], steps, decoded_len).

    `trace`, if a list, receives one record per step: the state before the step and the
    step's conf / pre / p / sel, for teacher-forced comparison.
    """
    assert gen_len % block_len == 0
    P = len(prompt)
    X = np.concatenate([np.asarray(prompt, dtype=np.int64),
                        np.full(gen_len, mask_id, dtype=np.int64)])
    steps = 0
    decoded_len = gen_len
    for b in range(gen_len // block_len):
        lo = P + b * block_len
        assert not (prefix_cache and dual_cache)
        cache = model.prefix_kv(X[:lo]) if prefix_cache else (model.full_kv(X) if dual_cache else None)
        while np.any(X[lo:lo + block_len] == mask_id):
            before = X.copy() if trace is not None else None
            d = denoise_step(model, X, P, b, block_len, mask_id, flt, tau, bias, cache, dual_cache)
            steps += 1
            if trace is not None:
                d.update(X_before=before, block=b)
                trace.append(d)
        if eotp and np.any(X[P:lo + block_len] == eos_id):
            decoded_len = (b + 1) * block_len
            break
    return X[P:P + gen_len].copy(), steps, decoded_len


def tail_all_eos(response, eos_id, decoded_len):
    """True when every decoded position from the first end-of-text token on holds end-of-text."""
    r = np.asarray(response)[:decoded_len]
    hit = np.nonzero(r == eos_id)[0]
    return bool(len(hit) and np.all(r[hit[0]:] == eos_id))


# --------------------------------------------------------------------------- Alg. 1: EGP rollout
def egp_step(model, X, prompt_len, b, block_len, mask_id, reference, bias=None):
    """One pass of Alg. 1's while-loop body without the parameter update: predict, compare with the
    reference answer, unmask where they agree (X modified in place).  Returns the training row:
    cin[s] (confidence of masked positions, 1.0 for committed ones) and y[s] (1 = may be unmasked)."""
    lo = prompt_len + b * block_len
    logits = apply_bias(model.forward(X, lo, block_len), b * block_len, bias)
    conf, pre = conf_pre(logits, mask_id)
    masked = np.asarray(X[lo:lo + block_len]) == mask_id
    ref = np.asarray(reference[b * block_len:(b + 1) * block_len])
    match = masked & (pre == ref)
    cin = np.where(masked, conf, conf.dtype.type(1.0))
    y = np.where(masked, match, True).astype(conf.dtype)
    sel = match.copy()
    if masked.any() and not match.any():
        cm = np.where(masked, conf, -np.inf)
        sel[int(np.argmax(cm))] = True            # progress: the reference token, labelled 0
    for j in np.nonzero(sel)[0]:
        X[lo + j] = ref[j]
    return dict(cin=cin, y=y, sel=sel, conf=conf, pre=pre, masked=masked, logits=logits)


def egp_rollout(model, prompt, reference, gen_len, block_len, mask_id, bias=None, trace=None):
    """EGP decoding of one prompt against its reference answer.  Returns (C[n, s], Y[n, s], steps
    per block); the decoded response equals the reference by construction."""
    assert gen_len % block_len == 0 and len(reference) == gen_len
    P = len(prompt)
    X = np.concatenate([np.asarray(prompt, dtype=np.int64), np.full(gen_len, mask_id, dtype=np.int64)])
    rows_c, rows_y, per_block = [], [], []
    for b in range(gen_len // block_len):
        lo = P + b * block_len
        n = 0
        while np.any(X[lo:lo + block_len] == mask_id):
            before = X.copy() if trace is not None else None
            d = egp_step(model, X, P, b, block_len, mask_id, reference, bias)
            rows_c.append(d["cin"])
            rows_y.append(d["y"])
            n += 1
            if trace is not None:
                d.update(X_before=before, block=b)
                trace.append(d)
        per_block.append(n)
    assert np.array_equal(X[P:], np.asarray(reference))
    return np.array(rows_c), np.array(rows_y), per_block


# --------------------------------------------------------------------------- Eq. 6 and the optimiser
def bce_loss_and_grad(flt, C, Y, dtype=np.float64):
    """Mean binary cross-entropy (Eq. 6) of sigmoid(f_theta(c)) against y over all entries of the
    rows C[n, s], Y[n, s], and its gradient with respect to every w_k, b_k of the filter.
    `dtype` is the precision everything is evaluated in (float64 by default)."""
    C = np.asarray(C, dtype=dtype)
    Y = np.asarray(Y, dtype=dtype)
    n = filter_depth(flt)
    W = [None] + [np.asarray(flt[f"w{k}"], dtype=dtype) for k in range(1, n + 1)]
    Bv = [None] + [np.asarray(flt[f"b{k}"], dtype=dtype) for k in range(1, n + 1)]
    acts = [C]                               # acts[k] = input of layer k+1, rows [n, width]
    pre = [None]                             # pre[k] = pre-activation of layer k
    for k in range(1, n):
        pre.append(acts[-1] @ W[k].T + Bv[k])
        acts.append(np.maximum(pre[-1], 0.0))
    Z = acts[-1] @ W[n].T + Bv[n]            # [n, s]
    m = C.dtype.type(Z.size)
    # -[y log sigma(z) + (1 - y) log(1 - sigma(z))] = softplus(z) - y z
    loss = float(np.sum(np.maximum(Z, 0.0) + np.log1p(np.exp(-np.abs(Z))) - Y * Z) / m)
    d = (sigmoid(Z) - Y) / m                 # dL/d(pre-activation) of the layer at hand
    g = {}
    for k in range(n, 0, -1):
        g[f"w{k}"] = d.T @ acts[k - 1]
        g[f"b{k}"] = d.sum(axis=0)
        if k > 1:
            d = (d @ W[k]) * (pre[k - 1] > 0.0)
    return loss, g


def adamw_step(param, grad, m, v, t, lr, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01):
    """One AdamW update (decoupled weight decay) at step t >= 1.  Returns (param, m, v)."""
    m = beta1 * m + (1.0 - beta1) * grad
    v = beta2 * v + (1.0 - beta2) * grad * grad
    mh = m / (1.0 - beta1 ** t)
    vh = v / (1.0 - beta2 ** t)
    param = param - lr * (mh / (np.sqrt(vh) + eps) + weight_decay * param)
    return param, m, v


def train_filter(flt, C, Y, epochs, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01,
                 dtype=np.float64):
    """`epochs` full-batch AdamW steps on Eq. 6.  Returns (filter, losses[epochs]) in `dtype`
    (float64 by default; float32 shows how far single precision alone moves the result)."""
    n = filter_depth(flt)
    ft = np.dtype(dtype).type
    lr, beta1, beta2, eps, weight_decay = (ft(x) for x in (lr, beta1, beta2, eps, weight_decay))
    th = {f"{c}{k}": np.array(flt[f"{c}{k}"], dtype=dtype) for k in range(1, n + 1) for c in "wb"}
    m = {k: np.zeros_like(x) for k, x in th.items()}
    v = {k: np.zeros_like(x) for k, x in th.items()}
    losses = []
    for t in range(1, epochs + 1):
        loss, g = bce_loss_and_grad(th, C, Y, dtype)
        losses.append(loss)
        for k in th:
            th[k], m[k], v[k] = adamw_step(th[k], g[k], m[k], v[k], t, lr, beta1, beta2, eps, weight_decay)
    return th, np.array(losses)
