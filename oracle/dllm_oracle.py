"""CPU oracle for the denoise-step path of masked-diffusion LLM decoding.  TEST INFRASTRUCTURE ONLY.

This file is the plain definition of what the HIP path computes, written out in numpy float64.
It is slow on purpose, shares no code with the HIP path, and must only be imported by tests, by
the smoke check and by the benchmark's CPU-baseline leg.  Nothing in the product path may call it.

What follows which passage of the paper (d3LLM, arxiv 2601.07568):
  * bidirectional (unmasked) attention between all tokens present in a forward  -- Section 1
    ("bidirectional attention") and the appendix on the serving-engine integration, item (i);
  * a cache of the key/value states of the prompt and of completed blocks, and forward passes
    that do not use the cache and rewrite it -- Section 3.2, "KV-Cache and KV-Refresh Mechanism"
    and the description of the "Completed but Stabilizing" state;
  * selecting, in every forward, the tokens whose prediction is confident enough, and decoding
    at least a minimum number per forward regardless of the threshold -- Section 3.2,
    "Entropy-Based Multi-Block Parallel Decoding"; the max-probability form of the rule is the
    threshold rule Section 2 attributes to Fast-dLLM;
  * unmasking exactly one token per step (the teacher's trajectory) -- Section 3.1; this is the
    same step with a threshold above 1 and a floor of 1;
  * block size 32, greedy decoding -- appendix, "Inference Settings".
The paper does not describe the transformer itself (it names LLaDA / Dream).  The layer used here
is the usual pre-norm one: RMSNorm, rotary position embedding in the half-split pairing,
multi-/grouped-query attention, SwiGLU MLP, untied LM head, no biases.

Parity pins (tests/test_oracle_*.py): brute-force attention, an independent float64 composition
out of torch library routines, closed forms of the confidence, cache == recompute, rotary shift
invariance, non-causality, selection invariants and a sort-based selection.  The paper prints no
numerical value for any of these functions, so beyond those pins the numbers are unpinned by the
paper itself.

Weights are dicts of arrays, linear weights [out_features, in_features].  `model` is any object
with .ms (shape record with n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ff, vocab,
mask_id, rms_eps, rope_base), .layer(l) -> dict and ["tok_emb" | "final_norm" | "lm_head"].
All inputs are converted to float64 on entry (the conversion function is passed in by the
caller, default: numpy's astype).

Storage precision.  All arithmetic is float64.  A model whose activations are handed from kernel
to kernel in a narrower type decides its arg max and its unmask set on values that went through
that type, so those decisions have to be taken in the same precision here: every forward takes
an optional `store` function (e.g. round-to-bfloat16) that is applied exactly where the data
layout of the library stores an activation -- the GEMM input of a normalised layer (x * gain is
what is stored; the row's factor rsqrt(mean(x^2) + eps) is a scalar that stays in full precision
and multiplies the product), q and k after the rotary embedding, v, the attention output, and
silu(gate)*up -- and nowhere else (the residual stream, scores, probabilities and logits are never
rounded).  store=None is the exact definition.
"""
from __future__ import annotations

import numpy as np


def _f64(a, widen=None):
    if widen is not None:
        a = widen(a)
    return np.asarray(a, dtype=np.float64)


# --------------------------------------------------------------------------- layer pieces

def rmsnorm(x, gain, eps):
    """x * rsqrt(mean(x^2) + eps) * gain over the last axis."""
    x = np.asarray(x, dtype=np.float64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gain


def rope(v, pos, base):
    """Rotary embedding, half-split pairing.  v: [S, H, dh]; pos: [S] absolute positions.
    Pair (j, j + dh/2) is rotated by the angle pos * base**(-2j/dh)."""
    v = np.asarray(v, dtype=np.float64)
    S, H, dh = v.shape
    half = dh // 2
    j = np.arange(half, dtype=np.float64)
    theta = base ** (-2.0 * j / dh)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * theta[None, :]       # [S, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    a, b = v[..., :half], v[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def attention(q, k, v):
    """softmax(q k^T / sqrt(dh)) v with no mask.  q: [Sq, H, dh]; k, v: [Sk, Hkv, dh].
    Query head h reads key/value head h // (H / Hkv)."""
    Sq, H, dh = q.shape
    Hkv = k.shape[1]
    group = H // Hkv
    out = np.empty((Sq, H, dh), dtype=np.float64)
    for h in range(H):
        kh = h // group
        s = q[:, h, :] @ k[:, kh, :].T / np.sqrt(dh)                        # [Sq, Sk]
        s = s - s.max(axis=-1, keepdims=True)
        p = np.exp(s)
        p = p / p.sum(axis=-1, keepdims=True)
        out[:, h, :] = p @ v[:, kh, :]
    return out


def silu(x):
    return x / (1.0 + np.exp(-x))


def _st(a, store):
    return a if store is None else np.asarray(store(a), dtype=np.float64)


def norm_input(x, gain, eps, store=None):
    """RMSNorm as the input of a linear layer.  Exactly rmsnorm(x, gain, eps); with a storage function the stored
    activation is x * gain and the row factor is applied in full precision (it commutes with the linear layer)."""
    if store is None:
        return rmsnorm(x, gain, eps)
    x = np.asarray(x, dtype=np.float64)
    return _st(x * gain, store) / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)


def layer_qkv(ms, lw, x, pos, widen=None, store=None):
    """Normalised input -> rotated q, rotated k, v for the rows of x at absolute positions pos."""
    S = x.shape[0]
    h = norm_input(x, _f64(lw["attn_norm"], widen), ms.rms_eps, store)
    q = (h @ _f64(lw["wq"], widen).T).reshape(S, ms.n_q_heads, ms.head_dim)
    k = (h @ _f64(lw["wk"], widen).T).reshape(S, ms.n_kv_heads, ms.head_dim)
    v = (h @ _f64(lw["wv"], widen).T).reshape(S, ms.n_kv_heads, ms.head_dim)
    return _st(rope(q, pos, ms.rope_base), store), _st(rope(k, pos, ms.rope_base), store), _st(v, store)


def layer_finish(ms, lw, x, o, widen=None, store=None):
    """Output projection + residual, then SwiGLU MLP + residual."""
    S = x.shape[0]
    x = x + _st(o, store).reshape(S, -1) @ _f64(lw["wo"], widen).T
    h = norm_input(x, _f64(lw["mlp_norm"], widen), ms.rms_eps, store)
    g = h @ _f64(lw["w_gate"], widen).T
    u = h @ _f64(lw["w_up"], widen).T
    return x + _st(silu(g) * u, store) @ _f64(lw["w_down"], widen).T


def head_logits(model, x, widen=None, store=None):
    """Final norm and LM head: raw logits [rows, vocab] (row i predicts position i, no shift)."""
    ms = model.ms
    h = norm_input(x, _f64(model["final_norm"], widen), ms.rms_eps, store)
    return h @ _f64(model["lm_head"], widen).T


# --------------------------------------------------------------------------- forwards

def forward_full(model, tokens, n_layers=None, widen=None, want_logits=True, pos0=0, store=None):
    """No-cache forward over one sequence: every token attends to every token.
    Returns (logits [S, V] or None, K [L][S, Hkv, dh], V [L][...], hidden [S, d])."""
    ms = model.ms
    L = ms.n_layers if n_layers is None else n_layers
    tokens = np.asarray(tokens)
    S = tokens.shape[0]
    pos = np.arange(S) + pos0
    x = _f64(np.asarray(model["tok_emb"])[tokens], widen)
    Ks, Vs = [], []
    for l in range(L):
        lw = model.layer(l)
        q, k, v = layer_qkv(ms, lw, x, pos, widen, store)
        Ks.append(k)
        Vs.append(v)
        x = layer_finish(ms, lw, x, attention(q, k, v), widen, store)
    logits = head_logits(model, x, widen, store) if want_logits else None
    return logits, Ks, Vs, x


def prefill(model, tokens, n_cache=None, n_layers=None, widen=None, store=None):
    """Key/value states of the first n_cache positions taken from a no-cache forward over
    `tokens` (which may extend past n_cache, e.g. include in-flight blocks)."""
    _, Ks, Vs, _ = forward_full(model, tokens, n_layers, widen, want_logits=False, store=store)
    n = len(tokens) if n_cache is None else n_cache
    return [k[:n] for k in Ks], [v[:n] for v in Vs]


def forward_cached(model, block_tokens, cache_k, cache_v, n_layers=None, widen=None,
                   want_logits=True, stop_layer=None, store=None):
    """Denoise-step forward: the Q block tokens sit at positions P..P+Q-1 and attend to the
    cached prefix (P = cache length) and to themselves.  Returns (logits [Q, V], hidden [Q, d])."""
    ms = model.ms
    L = ms.n_layers if n_layers is None else n_layers
    if stop_layer is not None:
        L = stop_layer
    block_tokens = np.asarray(block_tokens)
    Q = block_tokens.shape[0]
    P = cache_k[0].shape[0] if len(cache_k) else 0
    pos = np.arange(Q) + P
    x = _f64(np.asarray(model["tok_emb"])[block_tokens], widen)
    for l in range(L):
        lw = model.layer(l)
        q, k, v = layer_qkv(ms, lw, x, pos, widen, store)
        kk = np.concatenate([_f64(cache_k[l], widen), k], axis=0)
        vv = np.concatenate([_f64(cache_v[l], widen), v], axis=0)
        x = layer_finish(ms, lw, x, attention(q, kk, vv), widen, store)
    logits = head_logits(model, x, widen, store) if want_logits else None
    return logits, x


# --------------------------------------------------------------------------- confidence + select

def confidence(logits, mask_id):
    """Per row: candidate token (arg max, lowest id on ties), its softmax probability, and the
    entropy of the row in nats.  The mask id itself can never be predicted: its column is
    taken out of the softmax."""
    z = np.array(logits, dtype=np.float64, copy=True)
    z[:, mask_id] = -np.inf
    cand = np.argmax(z, axis=-1)
    zmax = z[np.arange(z.shape[0]), cand]
    e = np.exp(z - zmax[:, None])
    lse = np.log(e.sum(axis=-1)) + zmax
    p = np.exp(z - lse[:, None])
    conf = np.exp(zmax - lse)
    zz = np.where(np.isfinite(z), z, 0.0)
    entropy = lse - (p * zz).sum(axis=-1)
    return cand.astype(np.int64), conf, entropy, p


def unmask(tokens, cand, conf, mask_id, tau, m):
    """Threshold + floor selection on one block.  Masked positions with conf >= tau are
    unmasked, and so are the m' = min(m, #masked) most confident masked positions (highest
    confidence first, lowest index first among equals; a NaN confidence passes no threshold and ranks
    behind every number).  Returns (new tokens, chosen indices)."""
    tokens = np.array(tokens, copy=True)
    masked = [i for i in range(len(tokens)) if tokens[i] == mask_id]
    chosen = {i for i in masked if conf[i] >= tau}
    order = sorted(masked, key=lambda i: (1, 0.0, i) if conf[i] != conf[i] else (0, -conf[i], i))
    chosen.update(order[:min(m, len(masked))])
    for i in chosen:
        tokens[i] = cand[i]
    return tokens, sorted(chosen)


def unmask_entropy(tokens, cand, entropy, mask_id, theta, m):
    """Entropy-threshold selection on one block (Section 3.2, entropy-based decoding; Appendix,
    inference settings: theta between 0.4 and 0.5 nats).  Masked positions with entropy <= theta
    are unmasked, and so are the m' = min(m, #masked) masked positions of lowest entropy (lowest
    index first among equals).  m = 0 is the threshold-only strategy of an "Activated" block,
    m >= 1 the strategy of a "Fully-Activated" one.  Returns (new tokens, chosen indices)."""
    tokens = np.array(tokens, copy=True)
    masked = [i for i in range(len(tokens)) if tokens[i] == mask_id]
    chosen = {i for i in masked if entropy[i] <= theta}
    order = sorted(masked, key=lambda i: (1, 0.0, i) if entropy[i] != entropy[i] else (0, entropy[i], i))   # NaN last
    chosen.update(order[:min(m, len(masked))])
    for i in chosen:
        tokens[i] = cand[i]
    return tokens, sorted(chosen)


def denoise_step(model, block_tokens, cache_k, cache_v, tau, m, block_len=None, widen=None,
                 n_layers=None, store=None, rule="prob"):
    """One whole step on a window of one or more blocks: forward, confidence of the masked
    rows, selection per block (rule "prob": max-probability >= tau; rule "entropy": entropy <=
    tau).  Returns dict with new tokens, cand, conf, entropy, chosen, logits."""
    ms = model.ms
    block_tokens = np.asarray(block_tokens)
    Q = len(block_tokens)
    bl = Q if block_len is None else block_len
    logits, _ = forward_cached(model, block_tokens, cache_k, cache_v, n_layers, widen, store=store)
    cand, conf, ent, _ = confidence(logits, ms.mask_id)
    new = np.array(block_tokens, copy=True)
    chosen_all = []
    for b0 in range(0, Q, bl):
        sl = slice(b0, b0 + bl)
        if rule == "entropy":
            new[sl], ch = unmask_entropy(block_tokens[sl], cand[sl], ent[sl], ms.mask_id, tau, m)
        else:
            new[sl], ch = unmask(block_tokens[sl], cand[sl], conf[sl], ms.mask_id, tau, m)
        chosen_all += [b0 + i for i in ch]
    return {"tokens": new, "cand": cand, "conf": conf, "entropy": ent, "chosen": chosen_all,
            "logits": logits}


def decode(model, prompt, n_blocks, block_len, tau, m, widen=None, n_layers=None,
           record=None, store=None, rule="prob"):
    """Sequential-block decoding: cache the prompt, then for each block append block_len mask
    ids, run denoise steps until none is left, refresh the cache with a no-cache forward over
    everything decoded so far, go on.  Returns (all tokens, number of forwards with cache)."""
    ms = model.ms
    seq = np.array(prompt, dtype=np.int64, copy=True)
    ck, cv = prefill(model, seq, None, n_layers, widen, store)
    steps = 0
    for _ in range(n_blocks):
        blk = np.full(block_len, ms.mask_id, dtype=np.int64)
        while (blk == ms.mask_id).any():
            r = denoise_step(model, blk, ck, cv, tau, m, None, widen, n_layers, store, rule)
            if record is not None:
                record.append({"before": blk.copy(), **r})
            blk = r["tokens"]
            steps += 1
        seq = np.concatenate([seq, blk])
        ck, cv = prefill(model, seq, None, n_layers, widen, store)      # refresh at the block boundary
    return seq, steps


# ---------------------------------------------------------------------------------------------
# Multi-block decoding (Section 3.2, "Entropy-Based Multi-Block Parallel Decoding"; thresholds from
# the appendix, "Inference Settings": block-add 0.1, decoded-token 0.95, cache delay 1-2 rounds).
#
# The paper gives the five block states and the transition rules in one paragraph.  What it leaves
# open is fixed here (and listed with the other readings in the design notes):
#   * the first block starts Fully-Activated (its "preceding block" is the prompt, which is complete);
#   * "X % completion" = unmasked positions / block length >= X;
#   * a round's forward does not use the cache iff some block is Stabilizing at the start of the
#     round; otherwise it uses the cache of the prompt and the Completed blocks;
#   * transitions are evaluated after the round's unmasking, in block order, on the new tokens;
#     a newly added block whose predecessor is already >= 95 % complete starts Fully-Activated;
#   * a Stabilizing block counts the no-cache rounds since it filled up and becomes Completed after
#     `delay` of them, but not before its predecessor is Completed (the cache grows in order);
#   * decoding ends when no [MASK] is left.
INACTIVE, ACTIVATED, FULLY_ACTIVATED, STABILIZING, COMPLETED = 0, 1, 2, 3, 4


def fsm_update(state, counter, filled, block_len, add_at, full_at, delay, nocache_round):
    """State transitions of one sequence after a round.  state, counter: per-block lists; filled[b] =
    unmasked positions of block b after the round's unmasking; nocache_round: the round's forward
    did not use the cache.  Returns (new state, new counter) as lists."""
    nb = len(state)
    st, ct = list(state), list(counter)
    for b in range(nb):
        done_prev = 1.0 if b == 0 else filled[b - 1] / block_len
        if st[b] == STABILIZING:
            if nocache_round:
                ct[b] -= 1
            if ct[b] <= 0 and (b == 0 or st[b - 1] == COMPLETED):
                st[b] = COMPLETED
        elif st[b] in (ACTIVATED, FULLY_ACTIVATED):
            if filled[b] == block_len:
                st[b], ct[b] = STABILIZING, delay
            elif st[b] == ACTIVATED and done_prev >= full_at:
                st[b] = FULLY_ACTIVATED
        elif st[b] == INACTIVE:
            if b > 0 and st[b - 1] != INACTIVE and done_prev >= add_at:
                st[b] = FULLY_ACTIVATED if done_prev >= full_at else ACTIVATED
            break                                   # only the first inactive block can be added
    return st, ct


def fsm_plan(state, counter, block_len, base_len, refresh_every, since, was_nocache):
    """What the next round of one sequence looks like, from its block states after the transitions of the round just
    done.  since: cached rounds since the last forward without cache, before the round just done; was_nocache: that
    round's forward did not use the cache.  Returns (since updated, whether the next forward must skip the cache,
    how many positions the cache holds after such a forward).
    The next forward skips the cache if a block is Stabilizing, or if refresh_every > 0 cached rounds have passed
    since the last one that did (the periodic refresh of Section 3.2: the cache is updated every few rounds).  A
    forward without cache rewrites the cache of the prompt and of every block that is Completed once its round's
    transitions are done: the Completed blocks, and the Stabilizing ones behind them whose count-down ends with it."""
    since = 0 if was_nocache else since + 1
    nocache = any(s == STABILIZING for s in state) or (refresh_every > 0 and since >= refresh_every)
    done = 0
    for b, s in enumerate(state):
        if s == COMPLETED or (s == STABILIZING and counter[b] - 1 <= 0):
            done += 1
        else:
            break
    return since, nocache, base_len + done * block_len


def decode_multiblock(model, prompt, n_blocks, block_len, thr, rule="entropy", add_at=0.1, full_at=0.95,
                      delay=1, widen=None, n_layers=None, store=None, record=None, max_rounds=None,
                      refresh_every=0):
    """Multi-block decoding of n_blocks blocks after the prompt.  Every round: one forward over the
    window of Activated / Fully-Activated blocks (against the cache, or without it while a block is
    Stabilizing, in which case the cache is rewritten from that forward), selection per block with
    a floor of 0 (Activated) or 1 (Fully-Activated), then the state transitions.
    refresh_every > 0: the periodic refresh, a forward without cache after that many cached rounds in a row.
    Every forward without cache rewrites the cache of the prompt and of the blocks Completed at the end of its round
    (Section 3.2, multi-block paragraph: such a forward is also what renews the earlier caches).
    Returns (tokens of prompt + generation, number of forwards)."""
    ms = model.ms
    prompt = np.asarray(prompt, dtype=np.int64)
    P = len(prompt)
    since = 0                                                           # cached rounds since the last forward without cache
    gen = np.full(n_blocks * block_len, ms.mask_id, dtype=np.int64)
    state = [INACTIVE] * n_blocks
    counter = [0] * n_blocks
    state[0] = FULLY_ACTIVATED
    ck, cv = prefill(model, prompt, None, n_layers, widen, store)       # cache of the prompt
    n_done = 0                                                          # Completed blocks (in the cache)
    rounds = 0
    limit = max_rounds if max_rounds is not None else 4 * n_blocks * block_len + 8 * n_blocks
    while (gen == ms.mask_id).any():
        assert rounds < limit, "multi-block decoding does not terminate"
        active = [b for b in range(n_blocks) if state[b] in (ACTIVATED, FULLY_ACTIVATED)]
        lo, hi = active[0], active[-1]
        nocache = any(s == STABILIZING for s in state) or (refresh_every > 0 and since >= refresh_every)
        since = 0 if nocache else since + 1
        if nocache:
            seq = np.concatenate([prompt, gen[:(hi + 1) * block_len]])
            logits_all, Ks, Vs, _ = forward_full(model, seq, n_layers, widen, store=store)
            logits = logits_all[P + lo * block_len:]
        else:
            assert lo == n_done
            window = gen[lo * block_len:(hi + 1) * block_len]
            logits, _ = forward_cached(model, window, ck, cv, n_layers, widen, store=store)
        cand, conf, ent, _ = confidence(logits, ms.mask_id)
        before = gen.copy()
        chosen = []
        for b in active:
            off = (b - lo) * block_len
            sl = slice(b * block_len, (b + 1) * block_len)
            floor = 1 if state[b] == FULLY_ACTIVATED else 0
            if rule == "entropy":
                gen[sl], ch = unmask_entropy(gen[sl], cand[off:off + block_len], ent[off:off + block_len],
                                             ms.mask_id, thr, floor)
            else:
                gen[sl], ch = unmask(gen[sl], cand[off:off + block_len], conf[off:off + block_len],
                                     ms.mask_id, thr, floor)
            chosen += [b * block_len + i for i in ch]
        filled = [int((gen[b * block_len:(b + 1) * block_len] != ms.mask_id).sum()) for b in range(n_blocks)]
        new_state, counter = fsm_update(state, counter, filled, block_len, add_at, full_at, delay, nocache)
        n_done_new = sum(1 for s in new_state if s == COMPLETED)
        if nocache:
            # the blocks that became Completed take their K/V from this round's no-cache forward, which
            # also rewrites the cache of everything before them
            n = P + n_done_new * block_len
            ck, cv = [k[:n] for k in Ks], [v[:n] for v in Vs]
        if record is not None:
            record.append({"before": before, "lo": lo, "hi": hi, "nocache": nocache, "state": list(state),
                           "n_cached": P + n_done_new * block_len if nocache else P + n_done * block_len,
                           "cand": cand, "conf": conf, "entropy": ent, "chosen": chosen,
                           "state_after": list(new_state), "counter_after": list(counter)})
        state, n_done = new_state, n_done_new
        rounds += 1
    return np.concatenate([prompt, gen]), rounds


def round_batches(prompts, gens, states, nocache, n_commit_plan, block_len, max_window=None):
    """How one round of multi-block decoding looks for a batch of sequences that each follow decode_multiblock
    (Section 3.2, multi-block paragraph): sequence b with an active block runs either the cached step over its window
    (nocache[b] false) or the forward without cache over prompt + generation up to the end of the window, which also
    rewrites the first n_commit_plan[b] cached positions.  Returns a list, per sequence, of None (no active block: no
    forward) or a dict with the window (lo, hi in blocks), the forward type, the tokens the forward runs over, the
    number of cached positions it attends to (cached step) or rewrites (forward without cache), and the index of the
    window's first row within those tokens."""
    out = []
    for b, (prompt, gen, st) in enumerate(zip(prompts, gens, states)):
        active = [k for k, s in enumerate(st) if s in (ACTIVATED, FULLY_ACTIVATED)]
        if not active:
            out.append(None)
            continue
        lo, hi = active[0], active[-1]
        if max_window is not None:
            hi = min(hi, lo + max_window - 1)
        P = len(prompt)
        if nocache[b]:
            toks = np.concatenate([np.asarray(prompt), np.asarray(gen)[:(hi + 1) * block_len]])
            out.append({"lo": lo, "hi": hi, "nocache": True, "tokens": toks, "n_cached": int(n_commit_plan[b]),
                        "window_row": P + lo * block_len})
        else:
            out.append({"lo": lo, "hi": hi, "nocache": False,
                        "tokens": np.asarray(gen)[lo * block_len:(hi + 1) * block_len].copy(),
                        "n_cached": P + lo * block_len, "window_row": 0})
    return out


# ---------------------------------------------------------------------------------------------
# Teacher pseudo-trajectory (Section 3.1; appendix "Extracting Pseudo Trajectory of the Teacher
# dLLM") and early stopping (Section 3.2, "Early Stopping on EOS Token").

def teacher_trajectory(model, prompt, n_blocks, block_len, widen=None, n_layers=None, store=None):
    """The teacher's decoding order: exactly one token is unmasked per step (the most confident
    masked position of the current block; threshold above 1, floor 1), generation runs for the
    full length n = n_blocks * block_len whatever is decoded (no stop at an end-of-sequence token).
    Returns (tokens [n], order [n]) with order[i] = the step (1 .. n) that unmasked position i, so
    that trajectory state T_j has position i decoded iff order[i] <= j."""
    rec = []
    seq, steps = decode(model, prompt, n_blocks, block_len, 2.0, 1, widen, n_layers, rec, store)
    n = n_blocks * block_len
    assert steps == n
    order = np.zeros(n, dtype=np.int64)
    for j, r in enumerate(rec):
        (i,) = r["chosen"]
        order[(j // block_len) * block_len + i] = j + 1
    return seq[len(prompt):], order


def noisy_sequence(y, order, s, k, t, mask_id):
    """Noisy training sequence of Section 3.1 (the displayed case formula): with the decoding window
    {s, ..., s + k} and ratio t, position i (1-based in the paper) keeps the ground truth y_i if
    i <= s, is [MASK] if i > s + k, and inside the window keeps y_i iff the teacher's trajectory
    state T_{s + ceil(k t)} has it decoded.  Where the two printed cases overlap, the window bounds
    decide.  Indices here are 0-based: position j is the paper's i = j + 1."""
    y = np.asarray(y)
    m = s + int(np.ceil(k * t))
    out = np.array(y, copy=True)
    for j in range(len(y)):
        i = j + 1
        if i <= s:
            continue
        if i > s + k or order[j] > m:
            out[j] = mask_id
    return out


def eos_state(gen, eos_id, mask_id):
    """Early stop: a sequence is finished once an end-of-sequence token has been decoded with no
    [MASK] left before it (so everything up to it is final).  Returns (finished, index of that token
    or -1)."""
    for p, tok in enumerate(gen):
        if tok == mask_id:
            return False, -1
        if tok == eos_id:
            return True, p
    return False, -1


def live_sequences(gens, eos_id, mask_id):
    """Early stop over a batch (Section 3.2, "Early Stopping on EOS Token"): indices, in order, of the sequences that
    are not finished; a finished sequence takes part in no further forward."""
    return [b for b, gen in enumerate(gens) if not eos_state(gen, eos_id, mask_id)[0]]


def gather_rows(src, index, fill):
    """Compaction of a batch array: row i of the result is row index[i] of src for i < len(index); the remaining
    rows hold `fill`."""
    src = np.asarray(src)
    out = np.full_like(src, fill)
    for i, j in enumerate(index):
        out[i] = src[j]
    return out


def scatter_rows(dst, index, src):
    """The way back: row index[i] of the result is row i of src for i < len(index); other rows are those of dst."""
    out = np.array(dst, copy=True)
    for i, j in enumerate(index):
        out[j] = np.asarray(src)[i]
    return out
