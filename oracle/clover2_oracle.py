"""CPU oracle for one Clover-2 speculative step.  TEST INFRASTRUCTURE ONLY.

Plain NumPy, one sequence at a time, no blocking, no fusion.  Only the tests,
the smoke check and the benchmark's CPU-baseline leg may import this file; the
product (the HIP library and its Python binding) never does, and this file
imports nothing from the product.

What is computed, and where the paper defines it
------------------------------------------------
* Target model: a LLaMA-style decoder (the paper's targets are Vicuna-7B and
  LLaMA3-8B, Sec. 4.1 "Models and baselines").
* Tree attention (Sec. 2.1): the causal mask over the candidate tokens is the
  tree's ancestor-or-self matrix; cached tokens are visible to every node.
* Attention Decoder (Appendix A.3 listing; Sec. 3.2 removes the SiLU): RMSNorm
  on x, q from x, k and v from y, one cosine similarity per head between q and
  k that scales that head's slice of v, residual add of x.
* Draft head wiring (Sec. 3, Sec. 3.1, 3.2, 3.3, "Other details"): AD1 merges
  the target's last-block hidden state with the embedding of the token that
  followed it; the Augmenting Block (decoder layers with their own KV cache)
  runs on that; head 0 is a plain FC on the block's last row.  For a node u of
  depth >= 1 that has children: s_u = AD2(x = s_parent(u), y = emb(tok_u)), i.e.
  the state handed down by u's parent (the root hands down the block's last
  row) and the embedding of u's OWN token; then FC_j over [s_u ; emb(tok_u)],
  an RMSNorm and the shared LM head give the logits whose ranked ids become
  u's children.  s_u (not the FC's output) is what u hands down (Sec. 3.2).
  Token embeddings are rows of the LM head weight.
* Greedy verification (Sec. 2.1; Table 1 caption, temperature 0): walk from the
  root, descend while a child carries the target's argmax, emit one bonus token.

Pins (tests/test_oracle_pins.py): chain tree == token-by-token decoding; tree
verify == every root-to-leaf path run alone; speculative greedy == plain greedy;
compacted KV == KV of a fresh prefill; identity-style draft head reproduces the
target's logits; Attention-Decoder algebra; HF `LlamaForCausalLM` and
`scaled_dot_product_attention` cross-checks; top-k and the accept walk against
brute force; the matrices a regressive update and the Augmenting Block multiply
by, priced against the cost figures of Sec. 3.3; the draft wiring (which token
embedding and whose state AD1 / AD2 / FC_j receive, what is handed down) against
a closed form in the tokens alone for additive Attention Decoders, a pin that
planted wiring mistakes are shown to fail; the dynamic (score-pruned) tree
against brute force over every prefix of the full static tree, normalisation of
its scores, and the lossless property; sampled verification against the target
distribution (exact enumeration over the uniforms' outcomes and a seeded
Monte-Carlo run), its zero-temperature limit, and the library inverse-CDF.  The paper prints no worked numeric
example, so no pin compares against printed values.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Callable, Dict, List, Optional, Sequence, Tuple

import numpy as np


# ----------------------------------------------------------------------------
# configuration and weights
# ----------------------------------------------------------------------------
@dataclass
class OracleConfig:
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    vocab: int
    rope_base: float
    rms_eps: float
    aug_layers: int
    ad_heads: int
    draft_depths: int
    max_seq: int
    dtype: type = np.float64

    @staticmethod
    def from_shape(s, max_seq: int, dtype=np.float64) -> "OracleConfig":
        return OracleConfig(s.n_layers, s.hidden, s.n_q_heads, s.n_kv_heads, s.head_dim, s.ffn,
                            s.vocab, s.rope_base, s.rms_eps, s.aug_layers,
                            s.ad_heads or s.n_q_heads, s.draft_depths, max_seq, dtype)


class Weights:
    """Name -> array lookup.  `getter(name)` must return float32/float64 values;
    arrays are converted to the oracle dtype on first use and cached unless
    `cache=False` (large models: convert per use to bound memory)."""

    def __init__(self, getter: Callable[[str], np.ndarray], dtype=np.float64, cache: bool = True):
        self._get = getter
        self._dtype = dtype
        self._cache_on = cache
        self._cache: Dict[str, np.ndarray] = {}

    def __call__(self, name: str) -> np.ndarray:
        if name in self._cache:
            return self._cache[name]
        a = np.asarray(self._get(name)).astype(self._dtype, copy=False)
        if self._cache_on:
            self._cache[name] = a
        return a


# ----------------------------------------------------------------------------
# tree helpers (dense, by definition)
# ----------------------------------------------------------------------------
def tree_depths(parent: Sequence[int]) -> np.ndarray:
    n = len(parent)
    d = np.zeros(n, dtype=np.int64)
    for u in range(1, n):
        assert 0 <= parent[u] < u, "nodes must be in breadth-first order"
        d[u] = d[parent[u]] + 1
    return d


def ancestor_matrix(parent: Sequence[int]) -> np.ndarray:
    """A[u, w] is True iff w is u or an ancestor of u (the 2-D tree mask, Sec. 2.1)."""
    n = len(parent)
    a = np.zeros((n, n), dtype=bool)
    for u in range(n):
        w = u
        while w >= 0:
            a[u, w] = True
            w = parent[w]
    return a


def interval_labels(parent: Sequence[int]):
    """Linear-size tree mask (Appendix A.1: the mask relation is confirmed by numerical comparison instead of a
    2-D matrix; the paper's figure is not available, this is the reading taken): two integers per node from a
    depth-first numbering, enter[u] = the step at which u is first visited (children in index order),
    exit[u] = the largest enter value inside u's subtree.  Then w is u or an ancestor of u exactly when
    enter[w] <= enter[u] <= exit[w]."""
    n = len(parent)
    kids = children_of(parent)
    enter = np.zeros(n, dtype=np.int64)
    exit_ = np.zeros(n, dtype=np.int64)
    clock = 0
    stack = [(0, 0)]           # (node, index of the next child to visit)
    enter[0] = 0
    while stack:
        u, i = stack.pop()
        if i < len(kids[u]):
            stack.append((u, i + 1))
            c = kids[u][i]
            clock += 1
            enter[c] = clock
            stack.append((c, 0))
        else:
            exit_[u] = clock
    return enter, exit_


def mask_from_intervals(enter: np.ndarray, exit_: np.ndarray) -> np.ndarray:
    """The 2-D tree mask rebuilt from the interval labels: A[u, w] = enter[w] <= enter[u] <= exit[w]."""
    e = np.asarray(enter)
    return (e[None, :] <= e[:, None]) & (e[:, None] <= np.asarray(exit_)[None, :])


def children_of(parent: Sequence[int]) -> List[List[int]]:
    ch: List[List[int]] = [[] for _ in parent]
    for u in range(1, len(parent)):
        ch[parent[u]].append(u)
    return ch


# ----------------------------------------------------------------------------
# building blocks
# ----------------------------------------------------------------------------
def rmsnorm(x: np.ndarray, w: np.ndarray, eps: float) -> np.ndarray:
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps) * w


def rope(x: np.ndarray, pos: np.ndarray, base: float) -> np.ndarray:
    """Rotary embedding, half-split pairing: dim i pairs with dim i + d/2.
    x: [rows, heads, d]; pos: [rows]."""
    d = x.shape[-1]
    half = d // 2
    inv = base ** (-(np.arange(half, dtype=np.float64) * 2.0) / d)
    ang = pos.astype(np.float64)[:, None] * inv[None, :]
    cos = np.cos(ang).astype(x.dtype)[:, None, :]
    sin = np.sin(ang).astype(x.dtype)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * cos - x2 * sin, x2 * cos + x1 * sin], axis=-1)


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def softmax_rows(s: np.ndarray) -> np.ndarray:
    s = s - s.max(axis=-1, keepdims=True)
    e = np.exp(s)
    return e / e.sum(axis=-1, keepdims=True)


class KVCache:
    """K and V of every layer of one stack for one sequence: [layers, max_seq, n_kv, d]."""

    def __init__(self, n_layers: int, cfg: OracleConfig):
        shp = (n_layers, cfg.max_seq, cfg.n_kv_heads, cfg.head_dim)
        self.k = np.zeros(shp, dtype=cfg.dtype)
        self.v = np.zeros(shp, dtype=cfg.dtype)

    def copy(self) -> "KVCache":
        c = object.__new__(KVCache)
        c.k = self.k.copy()
        c.v = self.v.copy()
        return c


def decoder_layer(W: Weights, prefix: str, cfg: OracleConfig, x: np.ndarray, cache: KVCache, li: int,
                  L: int, pos: np.ndarray, slot: np.ndarray, vis_new: np.ndarray) -> np.ndarray:
    """One LLaMA decoder layer on `rows` new rows.

    Row r is rotated to position pos[r]; its K/V are stored at slot[r]; it sees
    every cached slot < L and new row c iff vis_new[r, c]."""
    rows = x.shape[0]
    nq, nkv, d = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    a = rmsnorm(x, W(prefix + "attn_norm"), cfg.rms_eps)
    q = (a @ W(prefix + "wq").T).reshape(rows, nq, d)
    k = (a @ W(prefix + "wk").T).reshape(rows, nkv, d)
    v = (a @ W(prefix + "wv").T).reshape(rows, nkv, d)
    q = rope(q, pos, cfg.rope_base)
    k = rope(k, pos, cfg.rope_base)
    cache.k[li, slot] = k
    cache.v[li, slot] = v
    keys = np.concatenate([cache.k[li, :L], cache.k[li, slot]], axis=0)   # [L+rows, nkv, d]
    vals = np.concatenate([cache.v[li, :L], cache.v[li, slot]], axis=0)
    vis = np.concatenate([np.ones((rows, L), dtype=bool), vis_new], axis=1)
    o = np.zeros((rows, nq, d), dtype=x.dtype)
    group = nq // nkv
    for h in range(nq):
        g = h // group
        s = (q[:, h, :] @ keys[:, g, :].T) / np.sqrt(float(d))
        s = np.where(vis, s, -np.inf)
        o[:, h, :] = softmax_rows(s) @ vals[:, g, :]
    x = x + o.reshape(rows, nq * d) @ W(prefix + "wo").T
    f = rmsnorm(x, W(prefix + "ffn_norm"), cfg.rms_eps)
    h1 = silu(f @ W(prefix + "w_gate").T) * (f @ W(prefix + "w_up").T)
    return x + h1 @ W(prefix + "w_down").T


def attention_decoder(W: Weights, prefix: str, cfg: OracleConfig, x: np.ndarray, y: np.ndarray) -> np.ndarray:
    """Attention Decoder (Appendix A.3).  x, y: [rows, H].

    The norm acts on x only; y (a token embedding) is used as is.  The gate is
    one cosine similarity per head, each vector norm clamped below at 1e-8."""
    rows, H = x.shape
    nh = cfg.ad_heads
    hd = H // nh
    xn = rmsnorm(x, W(prefix + "norm"), cfg.rms_eps)
    q = (xn @ W(prefix + "wq").T + W(prefix + "bq")).reshape(rows, nh, hd)
    k = (y @ W(prefix + "wk").T + W(prefix + "bk")).reshape(rows, nh, hd)
    v = (y @ W(prefix + "wv").T + W(prefix + "bv")).reshape(rows, nh, hd)
    nq_ = np.maximum(np.sqrt((q * q).sum(-1)), 1e-8)
    nk_ = np.maximum(np.sqrt((k * k).sum(-1)), 1e-8)
    att = (q * k).sum(-1) / (nq_ * nk_)                                  # [rows, nh]
    return x + (v * att[..., None]).reshape(rows, H)


def ranked_ids(z: np.ndarray, k: int) -> np.ndarray:
    """Ids of the k largest entries, ordered by (value descending, id ascending)."""
    order = np.argsort(-z, kind="stable")
    return order[:k].astype(np.int64)


# ----------------------------------------------------------------------------
# per-sequence state
# ----------------------------------------------------------------------------
class SeqState:
    """KV caches and lengths of one sequence (target stack and augmenting block)."""

    def __init__(self, cfg: OracleConfig):
        self.cfg = cfg
        self.kv = KVCache(cfg.n_layers, cfg)
        self.aug_kv = KVCache(cfg.aug_layers, cfg)
        self.L = 0          # target cache length
        self.aug_L = 0      # augmenting-block cache length


# ----------------------------------------------------------------------------
# the three calls
# ----------------------------------------------------------------------------
def verify_tree(W: Weights, cfg: OracleConfig, seq: SeqState, tokens: Sequence[int],
                parent: Sequence[int]) -> Tuple[np.ndarray, np.ndarray]:
    """Target forward over all tree nodes at once (Sec. 2.1).

    Node u sits at position L + depth(u) and its K/V go to slot L + u.  Returns
    (hidden [N,H] before the final norm, logits [N,V]).  seq.L is unchanged."""
    n = len(tokens)
    L = seq.L
    assert L + n <= cfg.max_seq
    depth = tree_depths(parent)
    pos = L + depth
    slot = L + np.arange(n)
    vis = ancestor_matrix(parent)
    x = W("embed")[np.asarray(tokens, dtype=np.int64)].astype(cfg.dtype)
    for li in range(cfg.n_layers):
        x = decoder_layer(W, f"layers.{li}.", cfg, x, seq.kv, li, L, pos, slot, vis)
    logits = rmsnorm(x, W("final_norm"), cfg.rms_eps) @ W("lm_head").T
    return x, logits


def draft_tree(W: Weights, cfg: OracleConfig, seq: SeqState, hid_acc: np.ndarray, next_tok: Sequence[int],
               parent: Sequence[int], rank: Sequence[int],
               forced_tokens: Optional[Sequence[int]] = None) -> Tuple[np.ndarray, Dict[int, np.ndarray]]:
    """Propose the token tree from the m newly accepted rows.

    hid_acc[i] is the target's pre-final-norm hidden state of accepted row i and
    next_tok[i] the token that followed it (the last one is the new root).
    Returns (tokens [N], {node u: draft logits z_u for every node with children}).
    With `forced_tokens`, node tokens are taken from it instead of from the
    ranking (used by the tests to follow a tolerated near-tie choice); the
    returned logits are still the oracle's own."""
    m = hid_acc.shape[0]
    n = len(parent)
    next_tok = np.asarray(next_tok, dtype=np.int64)
    assert m >= 1 and len(next_tok) == m
    lm = W("lm_head")
    emb = lambda t: lm[np.asarray(t, dtype=np.int64)].astype(cfg.dtype)   # embedding = LM-head rows
    # AD1: pre-integrate hidden state and the token the target produced after it (Sec. 3.1)
    u = attention_decoder(W, "ad1.", cfg, hid_acc.astype(cfg.dtype), emb(next_tok))
    # Augmenting Block: causal decoder layer(s) over its own cache (Sec. 3.3)
    L0 = seq.aug_L
    assert L0 + m <= cfg.max_seq
    pos = L0 + np.arange(m)
    causal = np.tril(np.ones((m, m), dtype=bool))
    a = u
    for li in range(cfg.aug_layers):
        a = decoder_layer(W, f"aug.{li}.", cfg, a, seq.aug_kv, li, L0, pos, pos, causal)
    seq.aug_L = L0 + m

    depth = tree_depths(parent)
    kids = children_of(parent)
    tokens = np.zeros(n, dtype=np.int64)
    tokens[0] = next_tok[m - 1]
    if forced_tokens is not None:
        assert int(forced_tokens[0]) == int(tokens[0])
    state: Dict[int, np.ndarray] = {0: a[m - 1]}
    zs: Dict[int, np.ndarray] = {}

    def expand(node: int, z: np.ndarray) -> None:
        zs[node] = z
        need = 1 + max(rank[c] for c in kids[node])
        top = ranked_ids(z, need)
        for c in kids[node]:
            tokens[c] = top[rank[c]] if forced_tokens is None else int(forced_tokens[c])

    # head 0: FC straight on the augmented state (Sec. 3.1)
    if kids[0]:
        g = W("fc0.w") @ state[0] + W("fc0.b")
        expand(0, W("lm_head") @ rmsnorm(g, W("head_norm"), cfg.rms_eps))
    # later depths: regressive update through AD2, then FC over [state ; embedding] (Sec. 3.2)
    for node in range(1, n):
        if not kids[node]:
            continue
        j = int(depth[node])
        assert 1 <= j <= cfg.draft_depths - 1
        e = emb(tokens[node])
        s = attention_decoder(W, "ad2.", cfg, state[int(parent[node])][None, :], e[None, :])[0]
        state[node] = s
        g = W(f"fc.{j}.w") @ np.concatenate([s, e]) + W(f"fc.{j}.b")
        expand(node, W("lm_head") @ rmsnorm(g, W("head_norm"), cfg.rms_eps))
    return tokens, zs


def log_softmax(z: np.ndarray) -> np.ndarray:
    z = z - z.max()
    return z - np.log(np.exp(z).sum())


def draft_tree_dynamic(W: Weights, cfg: OracleConfig, seq: SeqState, hid_acc: np.ndarray, next_tok: Sequence[int],
                       topk: int, frontier: int, n_nodes: int, follow: Optional[dict] = None) -> dict:
    """Score-pruned dynamic tree (Sec. 4.1: the tree is constructed the way EAGLE constructs it; the reading
    taken here is the expand-and-rerank scheme below).

    Same draft head as `draft_tree` (AD1, Augmenting Block, head 0, regressive AD2/FC_j updates, shared LM
    head), but the topology is chosen per call from the draft's own probabilities:
      * a candidate's score is the sum of the draft log-probabilities (log-softmax of its parent's logits at
        its token) along its root path; the root has score 0;
      * the root expands into its `topk` most probable tokens (ids by value descending, id ascending);
      * at every depth j = 1 .. D-1 the `frontier` best candidates of that depth (score descending, older
        candidate first) are expanded, each into its `topk` most probable tokens;
      * of all candidates the n_nodes - 1 best (score descending, shallower first, older first) form the
        tree together with the root; a child never outscores its parent, so the set is closed under parents;
      * nodes are numbered breadth-first: by depth, then by the parent's number, then by rank under the parent.
    Candidates are numbered in creation order: 0 = root, depth-1 candidates in rank order, then for each
    depth the children of the expanded candidates in (expansion order, rank) order.

    `follow` = dict(tokens=[per candidate], frontier=[[candidate ids per depth 1..D-1]], keep=[candidate ids])
    makes the oracle take those decisions instead of its own (tests follow a tolerated near-tie choice of the
    other side); every score and logit returned is still the oracle's own.

    Returns dict(tokens, parent, rank [n_nodes]; cand_token, cand_parent, cand_depth, cand_rank, cand_score
    [per candidate]; frontier [[ids]]; keep [candidate id of every tree node]; logits {candidate id: z})."""
    m = hid_acc.shape[0]
    next_tok = np.asarray(next_tok, dtype=np.int64)
    assert m >= 1 and len(next_tok) == m and topk >= 1 and frontier >= 1 and n_nodes >= 1
    D = cfg.draft_depths
    lm = W("lm_head")
    emb = lambda t: lm[np.asarray(t, dtype=np.int64)].astype(cfg.dtype)
    u = attention_decoder(W, "ad1.", cfg, hid_acc.astype(cfg.dtype), emb(next_tok))
    L0 = seq.aug_L
    assert L0 + m <= cfg.max_seq
    pos = L0 + np.arange(m)
    causal = np.tril(np.ones((m, m), dtype=bool))
    a = u
    for li in range(cfg.aug_layers):
        a = decoder_layer(W, f"aug.{li}.", cfg, a, seq.aug_kv, li, L0, pos, pos, causal)
    seq.aug_L = L0 + m

    c_tok, c_par, c_dep, c_rank, c_score = [int(next_tok[m - 1])], [-1], [0], [0], [0.0]
    state: Dict[int, np.ndarray] = {0: a[m - 1]}
    zs: Dict[int, np.ndarray] = {}
    fronts: List[List[int]] = []

    def expand(c: int, z: np.ndarray) -> None:
        zs[c] = z
        lp = log_softmax(z.astype(np.float64))
        top = ranked_ids(z, topk)
        for i in range(topk):
            cid = len(c_tok)
            t = int(top[i]) if follow is None else int(follow["tokens"][cid])
            c_tok.append(t); c_par.append(c); c_dep.append(c_dep[c] + 1); c_rank.append(i)
            c_score.append(c_score[c] + float(lp[t]))

    g = W("fc0.w") @ state[0] + W("fc0.b")
    expand(0, W("lm_head") @ rmsnorm(g, W("head_norm"), cfg.rms_eps))
    for j in range(1, D):
        level = [c for c in range(len(c_tok)) if c_dep[c] == j]
        if follow is None:
            chosen = sorted(level, key=lambda c: (-c_score[c], c))[:frontier]
        else:
            chosen = [int(c) for c in follow["frontier"][j - 1]]
            assert all(c_dep[c] == j for c in chosen) and len(set(chosen)) == len(chosen) <= frontier
        fronts.append(chosen)
        for c in chosen:
            e = emb(c_tok[c])
            s = attention_decoder(W, "ad2.", cfg, state[c_par[c]][None, :], e[None, :])[0]
            state[c] = s
            g = W(f"fc.{j}.w") @ np.concatenate([s, e]) + W(f"fc.{j}.b")
            expand(c, W("lm_head") @ rmsnorm(g, W("head_norm"), cfg.rms_eps))

    cands = list(range(1, len(c_tok)))
    assert len(cands) >= n_nodes - 1, "fewer candidates than tree nodes"
    if follow is None:
        keep = [0] + sorted(cands, key=lambda c: (-c_score[c], c_dep[c], c))[:n_nodes - 1]
    else:
        keep = [int(c) for c in follow["keep"]]
        assert keep[0] == 0 and len(set(keep)) == len(keep) == n_nodes
    kept = set(keep)
    assert all(c == 0 or c_par[c] in kept for c in keep), "selection is not closed under parents"
    # breadth-first numbering: by depth, then the parent's number, then the rank under the parent
    number: Dict[int, int] = {0: 0}
    order = [0]
    for j in range(1, D + 1):
        level = sorted((c for c in keep if c_dep[c] == j), key=lambda c: (number[c_par[c]], c_rank[c]))
        for c in level:
            number[c] = len(order)
            order.append(c)
    tokens = np.asarray([c_tok[c] for c in order], dtype=np.int64)
    parent = np.asarray([-1] + [number[c_par[c]] for c in order[1:]], dtype=np.int64)
    rank = np.asarray([c_rank[c] for c in order], dtype=np.int64)
    return dict(tokens=tokens, parent=parent, rank=rank, cand_token=c_tok, cand_parent=c_par, cand_depth=c_dep,
                cand_rank=c_rank, cand_score=c_score, frontier=fronts, keep=order, logits=zs)


def accept_greedy(tokens: Sequence[int], logits: np.ndarray, parent: Sequence[int],
                  argmax_override: Optional[Dict[int, int]] = None) -> Tuple[List[int], int]:
    """Longest root path whose every token is the target's greedy choice (Sec. 2.1).

    Returns (path of node indices starting at the root, bonus token)."""
    kids = children_of(parent)
    u = 0
    path = [0]
    while True:
        t = int(ranked_ids(logits[u], 1)[0])
        if argmax_override is not None and u in argmax_override:
            t = int(argmax_override[u])
        nxt = [c for c in kids[u] if int(tokens[c]) == t]
        if not nxt:
            return path, t
        u = nxt[0]
        path.append(u)


def accept_sampled(tokens: Sequence[int], logits: np.ndarray, parent: Sequence[int], temperature: float,
                   uniforms: np.ndarray, decisions: Optional[Dict[int, dict]] = None) -> Tuple[List[int], int, Dict[int, dict]]:
    """Verification at a non-zero temperature (Table 1, temperature 1 rows; the tree is sampled the way EAGLE's
    engine does it: the candidates below a node are fixed tokens, not draws, so each is a point-mass proposal).

    At node u the target distribution is p = softmax(logits[u] / temperature).  The children of u are tried in
    index order: child c with token x is accepted with probability p(x) / (1 - mass of the children already
    refused), i.e. p(x) under the distribution that remains after the refusals; uniforms[u, i] decides the
    i-th child.  When a child is accepted the walk moves there.  When none is, the next token is drawn from what
    remains of p -- the refused tokens removed, the rest renormalised -- by inverting its cumulative sum in
    token-id order with uniforms[u, 16], and the walk ends.  A leaf draws from p itself.  The emitted token
    after every visited node is therefore distributed exactly as p (the method stays lossless).

    uniforms: [n_nodes, 17] values in [0, 1).  Returns (path, bonus token, {node: record of what was decided
    there}); `decisions` = {node: dict(accept=child position or -1, bonus=token)} overrides the decisions at those
    nodes (tests follow the other side inside a tolerance); the probabilities recorded are always the oracle's."""
    kids = children_of(parent)
    u, path, rec = 0, [0], {}
    while True:
        z = logits[u].astype(np.float64) / float(temperature)
        p = np.exp(z - z.max())
        p /= p.sum()
        refused = 0.0
        ratios = []
        accepted = -1
        for i, c in enumerate(kids[u]):
            a = p[int(tokens[c])] / max(1.0 - refused, 1e-300)
            ratios.append(a)
            if accepted < 0 and (uniforms[u, i] < a if decisions is None or u not in decisions
                                 else decisions[u]["accept"] == i):
                accepted = i
                break
            refused += p[int(tokens[c])]
        rec[u] = dict(ratios=ratios, accept=accepted)
        if accepted >= 0:
            u = kids[u][accepted]
            path.append(u)
            continue
        rest = p.copy()
        for c in kids[u]:
            rest[int(tokens[c])] = 0.0
        cdf = np.cumsum(rest)
        target = uniforms[u, 16] * cdf[-1]
        bonus = int(np.searchsorted(cdf, target, side="right"))
        bonus = min(bonus, len(p) - 1)
        while rest[bonus] == 0.0 and bonus > 0:      # a draw that lands on a removed token's zero-width step
            bonus -= 1
        if decisions is not None and u in decisions:
            bonus = int(decisions[u]["bonus"])
        rec[u].update(cdf=cdf, target=target, bonus=bonus)
        return path, bonus, rec


def compact(seq: SeqState, path: Sequence[int]) -> None:
    """Keep only the accepted rows: slot L+i receives slot L+path[i], ascending i."""
    L = seq.L
    for i, p in enumerate(path):
        seq.kv.k[:, L + i] = seq.kv.k[:, L + p]
        seq.kv.v[:, L + i] = seq.kv.v[:, L + p]
    seq.L = L + len(path)


def accept_and_compact(cfg: OracleConfig, seq: SeqState, tokens: Sequence[int], logits: np.ndarray,
                       hidden: np.ndarray, parent: Sequence[int],
                       argmax_override: Optional[Dict[int, int]] = None, sampled: Optional[Tuple[List[int], int]] = None):
    """Greedy acceptance (or a path and next token already chosen by `accept_sampled`), KV compaction and the
    hand-off to the next draft call.

    Returns dict(m, path, new_tokens, hid_acc, next_tok)."""
    path, bonus = sampled if sampled is not None else accept_greedy(tokens, logits, parent, argmax_override)
    compact(seq, path)
    new_tokens = [int(tokens[p]) for p in path[1:]] + [bonus]
    return dict(m=len(path), path=path, new_tokens=new_tokens,
                hid_acc=hidden[np.asarray(path)].copy(), next_tok=list(new_tokens))


def accept_forced(seq: SeqState, tokens: Sequence[int], logits: np.ndarray, hidden: np.ndarray,
                  n_rows: int, forced_next: int):
    """Prefill hand-off for a chain of prompt tokens: accept the first n_rows nodes
    unconditionally.  The token following the last row is `forced_next`, or the
    target's greedy choice there when forced_next < 0."""
    path = list(range(n_rows))
    last = forced_next if forced_next >= 0 else int(ranked_ids(logits[n_rows - 1], 1)[0])
    compact(seq, path)
    new_tokens = [int(t) for t in tokens[1:n_rows]] + [int(last)]
    return dict(m=n_rows, path=path, new_tokens=new_tokens,
                hid_acc=hidden[:n_rows].copy(), next_tok=list(new_tokens))


# ----------------------------------------------------------------------------
# drivers built from the calls
# ----------------------------------------------------------------------------
def prefill(W: Weights, cfg: OracleConfig, seq: SeqState, prompt: Sequence[int], chunk: int,
            parent_tree: Sequence[int], rank_tree: Sequence[int]):
    """Feed the prompt as chain-shaped trees of at most `chunk` tokens; returns the
    first draft tree (tokens, zs) and the hand-off state of the last chunk."""
    prompt = [int(t) for t in prompt]
    out = None
    i = 0
    while i < len(prompt):
        part = prompt[i:i + chunk]
        n = len(part)
        chain = list(range(-1, n - 1))
        hidden, logits = verify_tree(W, cfg, seq, part, chain)
        nxt = prompt[i + n] if i + n < len(prompt) else -1
        acc = accept_forced(seq, part, logits, hidden, n, nxt)
        i += n
        if i < len(prompt):
            draft_tree(W, cfg, seq, acc["hid_acc"], acc["next_tok"], chain[:1], [0])
        else:
            out = (acc, draft_tree(W, cfg, seq, acc["hid_acc"], acc["next_tok"], parent_tree, rank_tree))
    return out


def speculative_generate(W: Weights, cfg: OracleConfig, prompt: Sequence[int], parent, rank, steps: int,
                         chunk: int = 16, tree_hook=None):
    """Prefill, then `steps` speculative steps.  Returns (emitted tokens, per-step m, seq).
    `tree_hook(step, tokens)` may replace the proposed tree's tokens (tests inject trees)."""
    seq = SeqState(cfg)
    acc, (tokens, _) = prefill(W, cfg, seq, prompt, chunk, parent, rank)
    emitted = [acc["new_tokens"][-1]]
    ms = []
    for step in range(steps):
        if tree_hook is not None:
            tokens = np.asarray(tree_hook(step, tokens.copy()))
        hidden, logits = verify_tree(W, cfg, seq, tokens, parent)
        acc = accept_and_compact(cfg, seq, tokens, logits, hidden, parent)
        emitted.extend(acc["new_tokens"])
        ms.append(acc["m"])
        tokens, _ = draft_tree(W, cfg, seq, acc["hid_acc"], acc["next_tok"], parent, rank)
    return emitted, ms, seq


def plain_greedy(W: Weights, cfg: OracleConfig, prompt: Sequence[int], n_new: int):
    """Token-by-token greedy decoding of the target alone (the definition the
    speculative result must equal).  Returns (new tokens, seq)."""
    seq = SeqState(cfg)
    out: List[int] = []
    last_logits = None
    for t in prompt:
        _, lg = verify_tree(W, cfg, seq, [int(t)], [-1])
        seq.L += 1
        last_logits = lg[0]
    for _ in range(n_new):
        t = int(ranked_ids(last_logits, 1)[0])
        out.append(t)
        _, lg = verify_tree(W, cfg, seq, [t], [-1])
        seq.L += 1
        last_logits = lg[0]
    return out, seq
