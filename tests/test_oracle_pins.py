"""Pins for the CPU oracle: it is checked against what the method's definition and
plain mathematics fix, never against itself or the HIP path.

P1 chain tree == token-by-token decoding            (tree positions, slots, mask)
P2 tree verify == each root-to-leaf path run alone  (ancestor mask; brute force)
P3 speculative greedy == plain greedy               (lossless property, Sec. 1 and 2.1)
P4 compacted KV == KV of a fresh prefill            (compaction indices, aug cache length)
P5 identity-style draft head (limit of the init table, Appendix A.2) reproduces target logits
P6 Attention-Decoder algebra                        (Appendix A.3)
P7 HF LlamaForCausalLM / SDPA cross-checks          (library special case)
P8 ranking and accept walk vs brute force
P9 matrices used by one regressive update / the Augmenting Block vs the cost figures of Sec. 3.3
P11 dynamic (score-pruned) tree == best prefixes of the complete static tree by brute force; invariants; lossless
P12 verification at temperature > 0 emits the target distribution (Monte-Carlo, quadrature), zero-temperature limit
P10 draft wiring in closed form (additive Attention Decoders): which token and whose state each step receives;
    the pin is shown to fail on planted wiring mistakes (mutants of the oracle's source, CPU only)
"""
import itertools

import numpy as np
import pytest

from oracle import clover2_oracle as O
from paper_2408_00264_amd import synth

TINY = synth.CONFIGS[1]


def make(shape=TINY, max_seq=160, gain_jitter=0.1, overrides=None, dtype=np.float64):
    ws = synth.WeightStore(shape, gain_jitter=gain_jitter, overrides=overrides)
    cfg = O.OracleConfig.from_shape(shape, max_seq, dtype)
    return ws, cfg, O.Weights(ws.get_f32, dtype)


def rand_tree(rng, n):
    parent = np.full(n, -1, dtype=np.int64)
    for u in range(1, n):
        parent[u] = rng.integers(0, u)
    # renumber breadth-first (depth-major, parent index ascending)
    depth = np.zeros(n, dtype=np.int64)
    for u in range(1, n):
        depth[u] = depth[parent[u]] + 1
    order = sorted(range(n), key=lambda u: (depth[u], u))
    new = {old: i for i, old in enumerate(order)}
    p2 = np.full(n, -1, dtype=np.int64)
    for old in range(1, n):
        p2[new[old]] = new[parent[old]]
    assert all(p2[u] < u for u in range(1, n))
    return p2


# ---------------------------------------------------------------- P1
def test_p1_chain_equals_sequential_decoding():
    ws, cfg, W = make()
    rng = np.random.default_rng(0)
    prompt = rng.integers(0, TINY.vocab, 9)
    chain_tok = rng.integers(0, TINY.vocab, 7)
    # (a) all at once as a chain-shaped tree after a chain prefill
    a = O.SeqState(cfg)
    O.verify_tree(W, cfg, a, prompt, list(range(-1, 8)))
    a.L = 9
    hid_a, log_a = O.verify_tree(W, cfg, a, chain_tok, list(range(-1, 6)))
    # (b) one token at a time
    b = O.SeqState(cfg)
    logs, hids = [], []
    for t in list(prompt) + list(chain_tok):
        h, lg = O.verify_tree(W, cfg, b, [t], [-1])
        b.L += 1
        logs.append(lg[0]); hids.append(h[0])
    np.testing.assert_allclose(log_a, np.stack(logs[9:]), atol=1e-10)
    np.testing.assert_allclose(hid_a, np.stack(hids[9:]), atol=1e-10)
    np.testing.assert_allclose(a.kv.k[:, :16], b.kv.k[:, :16], atol=1e-10)
    np.testing.assert_allclose(a.kv.v[:, :16], b.kv.v[:, :16], atol=1e-10)


def test_p1_prefill_state_does_not_depend_on_the_chunking():
    """Sec. 1 (prefill, then decode) with Sec. 3.1 / 3.3: whatever the pass size, a prompt leaves the same target
    cache, the same augmenting-block cache (position i paired with token i+1, also across pass boundaries) and the
    same first draft tree.  The GPU's prefill call is compared with the oracle at a different pass size on this basis."""
    ws, cfg, W = make()
    parent, rank = synth.tree_for(TINY)
    prompt = np.random.default_rng(5).integers(0, TINY.vocab, 23)
    outs = []
    for chunk in (1, 5, 23):
        seq = O.SeqState(cfg)
        acc, (tokens, zs) = O.prefill(W, cfg, seq, prompt, chunk, parent, rank)
        assert seq.L == 23 and seq.aug_L == 23
        outs.append((seq, tokens, acc["new_tokens"][-1]))
    ref = outs[-1]
    for seq, tokens, first in outs[:-1]:
        assert first == ref[2] and list(tokens) == list(ref[1])
        np.testing.assert_allclose(seq.kv.k[:, :23], ref[0].kv.k[:, :23], atol=1e-10)
        np.testing.assert_allclose(seq.kv.v[:, :23], ref[0].kv.v[:, :23], atol=1e-10)
        np.testing.assert_allclose(seq.aug_kv.k[:, :23], ref[0].aug_kv.k[:, :23], atol=1e-10)
        np.testing.assert_allclose(seq.aug_kv.v[:, :23], ref[0].aug_kv.v[:, :23], atol=1e-10)


# ---------------------------------------------------------------- P2
@pytest.mark.parametrize("seed", [0, 1])
def test_p2_tree_equals_each_path_alone(seed):
    ws, cfg, W = make()
    rng = np.random.default_rng(seed)
    n = 13
    parent = rand_tree(rng, n) if seed else synth.make_tree((4, 3, 2), 16)[0][:n]
    n = len(parent)
    prompt = rng.integers(0, TINY.vocab, 11)
    toks = rng.integers(0, TINY.vocab, n)
    s = O.SeqState(cfg)
    O.verify_tree(W, cfg, s, prompt, list(range(-1, 10)))
    s.L = 11
    base = s.kv.copy()
    hid, log = O.verify_tree(W, cfg, s, toks, parent)
    kids = O.children_of(parent)
    leaves = [u for u in range(n) if not kids[u]]
    seen = set()
    for leaf in leaves:
        path = []
        u = leaf
        while u >= 0:
            path.append(u); u = parent[u]
        path = path[::-1]
        t = O.SeqState(cfg)
        t.kv = base.copy(); t.L = 11
        h2, l2 = O.verify_tree(W, cfg, t, toks[path], list(range(-1, len(path) - 1)))
        np.testing.assert_allclose(l2, log[path], atol=1e-10)
        np.testing.assert_allclose(h2, hid[path], atol=1e-10)
        # K/V rows of the tree nodes equal the rows of the path run
        np.testing.assert_allclose(t.kv.k[:, 11:11 + len(path)], s.kv.k[:, 11 + np.asarray(path)], atol=1e-10)
        seen.update(path)
    assert seen == set(range(n))


# ---------------------------------------------------------------- P3 / P4
def _plain(W, cfg, prompt, n_new):
    return O.plain_greedy(W, cfg, prompt, n_new)


def test_p3_speculative_equals_plain_greedy_config1():
    ws, cfg, W = make(gain_jitter=0.0, max_seq=260)
    parent, rank = synth.tree_for(TINY)
    prompt = synth.make_prompts(TINY)[0]
    emitted, ms, seq = O.speculative_generate(W, cfg, prompt, parent, rank, steps=TINY.steps, chunk=16)
    ref, _ = _plain(W, cfg, prompt, len(emitted))
    assert emitted == ref
    assert sum(ms) + 1 == len(emitted)
    assert seq.L == seq.aug_L == len(prompt) + sum(ms)


def test_p3_paper_size_head_two_aug_layers_five_depths():
    """The head at the paper's size (Sec. 3.3 and 4.1: two augmenting layers, five heads): still lossless,
    and both caches advance together."""
    shape = synth.scaled(TINY, name="tiny-paper-head", aug_layers=2, draft_depths=5, tree_k=(3, 2, 2, 2, 1),
                         tree_nodes=20, seed=23)
    ws, cfg, W = make(shape=shape, gain_jitter=0.0, max_seq=200)
    parent, rank = synth.tree_for(shape)
    depth = [0] * len(parent)
    for u in range(1, len(parent)):
        depth[u] = depth[parent[u]] + 1
    assert len(parent) == 20 and max(depth) == 5
    prompt = synth.make_prompts(shape)[0][:40]
    emitted, ms, seq = O.speculative_generate(W, cfg, prompt, parent, rank, steps=4, chunk=16)
    ref, _ = _plain(W, cfg, prompt, len(emitted))
    assert emitted == ref
    assert seq.L == seq.aug_L == len(prompt) + sum(ms)


@pytest.mark.parametrize("pattern", ["deep", "mixed", "none"])
def test_p3_p4_injected_trees(pattern):
    """Trees built from the true continuation with controlled corruption: accept
    lengths 1..D+1 all occur; the emitted text is still the plain greedy text and the
    compacted cache equals the cache of a fresh prefill of that text."""
    ws, cfg, W = make(max_seq=200)
    parent, rank = synth.tree_for(TINY)
    depth = O.tree_depths(parent)
    kids = O.children_of(parent)
    height = np.zeros(len(parent), dtype=np.int64)
    for u_ in range(len(parent) - 1, 0, -1):
        height[parent[u_]] = max(height[parent[u_]], height[u_] + 1)
    prompt = synth.make_prompts(TINY, seed=7)[0][:20]
    truth, _ = _plain(W, cfg, prompt, 64)
    # truth[i] is the token at absolute position len(prompt)+i
    state = {"emitted": 1}
    want = {"deep": [4, 4, 4, 4], "mixed": [1, 2, 3, 4, 2, 1], "none": [1, 1, 1]}[pattern]

    def hook(step, tokens):
        # root = truth[emitted-1]; put the true continuation on one root-to-leaf path,
        # correct for want-1 levels, wrong (id+1) below.
        e = state["emitted"]
        assert int(tokens[0]) == truth[e - 1]
        rng = np.random.default_rng(step)
        tokens[1:] = (np.asarray(truth[e:e + 1] * (len(tokens) - 1)) + 1 + rng.integers(1, 50, len(tokens) - 1)) % TINY.vocab
        u = 0
        for lvl in range(want[step] - 1):
            # deepest subtree first; among equals the last child, so the walk must search siblings
            if not kids[u]:
                break
            c = max(kids[u], key=lambda c_: (height[c_], c_))
            tokens[c] = truth[e + lvl]
            u = c
        return tokens

    steps = len(want)

    emitted, ms, seq = None, None, None

    def run():
        nonlocal emitted, ms, seq
        out = []
        s = O.SeqState(cfg)
        acc, (tokens, _) = O.prefill(W, cfg, s, prompt, 16, parent, rank)
        out.append(acc["new_tokens"][-1])
        mlist = []
        for step in range(steps):
            tokens = hook(step, np.asarray(tokens).copy())
            hidden, logits = O.verify_tree(W, cfg, s, tokens, parent)
            acc = O.accept_and_compact(cfg, s, tokens, logits, hidden, parent)
            out.extend(acc["new_tokens"]); mlist.append(acc["m"])
            state["emitted"] = len(out)
            tokens, _ = O.draft_tree(W, cfg, s, acc["hid_acc"], acc["next_tok"], parent, rank)
        emitted, ms, seq = out, mlist, s

    run()
    assert ms == [min(w, 1 + max(depth)) for w in want]
    assert emitted == truth[:len(emitted)]
    # P4: compacted target cache == cache of a plain token-by-token run over the same text
    full = list(prompt) + emitted[:-1]
    assert seq.L == len(full) == seq.aug_L
    fresh = O.SeqState(cfg)
    for t in full:
        O.verify_tree(W, cfg, fresh, [int(t)], [-1]); fresh.L += 1
    np.testing.assert_allclose(seq.kv.k[:, :seq.L], fresh.kv.k[:, :seq.L], atol=1e-9)
    np.testing.assert_allclose(seq.kv.v[:, :seq.L], fresh.kv.v[:, :seq.L], atol=1e-9)


def test_p4_compaction_overlapping_moves():
    """dst slot of one move is the src slot of an earlier one: ascending order keeps it right."""
    ws, cfg, W = make()
    s = O.SeqState(cfg)
    s.L = 5
    rng = np.random.default_rng(3)
    s.kv.k[:] = rng.standard_normal(s.kv.k.shape)
    s.kv.v[:] = rng.standard_normal(s.kv.v.shape)
    k0, v0 = s.kv.k.copy(), s.kv.v.copy()
    path = [0, 1, 3, 9]
    O.compact(s, path)
    for i, p in enumerate(path):
        np.testing.assert_array_equal(s.kv.k[:, 5 + i], k0[:, 5 + p])
        np.testing.assert_array_equal(s.kv.v[:, 5 + i], v0[:, 5 + p])
    assert s.L == 9


# ---------------------------------------------------------------- P5
def _identity_overrides(shape, fc_pick="state"):
    H = shape.hidden
    z = lambda *s: np.zeros(s, np.float32)
    ov = {}
    for ad in ("ad1", "ad2"):
        ov[f"{ad}.wv"] = z(H, H); ov[f"{ad}.bv"] = z(H)
    ov["aug.0.wo"] = z(H, shape.n_q_heads * shape.head_dim)
    ov["aug.0.w_down"] = z(H, shape.ffn)
    ov["fc0.w"] = np.eye(H, dtype=np.float32); ov["fc0.b"] = z(H)
    for j in range(1, shape.draft_depths):
        w = z(H, 2 * H)
        if fc_pick == "state":
            w[:, :H] = np.eye(H)
        else:
            w[:, H:] = np.eye(H)
        ov[f"fc.{j}.w"] = w; ov[f"fc.{j}.b"] = z(H)
    return ov


def test_p5_identity_draft_reproduces_target_logits():
    base = synth.WeightStore(TINY, gain_jitter=0.1)
    ov = _identity_overrides(TINY, "state")
    ov["head_norm"] = base.get_f32("final_norm")
    ws, cfg, W = make(overrides=ov)
    parent, rank = synth.tree_for(TINY)
    kids = O.children_of(parent)
    prompt = synth.make_prompts(TINY, seed=3)[0][:24]
    s = O.SeqState(cfg)
    acc, (tokens, zs) = O.prefill(W, cfg, s, prompt, 16, parent, rank)
    # target logits at the last prompt row, computed by plain decoding
    _, ps = O.plain_greedy(W, cfg, prompt, 0)
    fresh = O.SeqState(cfg)
    lg = None
    for t in prompt:
        _, l1 = O.verify_tree(W, cfg, fresh, [int(t)], [-1]); fresh.L += 1; lg = l1[0]
    for node, z in zs.items():
        np.testing.assert_allclose(z, lg, atol=1e-9)   # every depth sees the same state
    top = np.argsort(-lg, kind="stable")
    assert tokens[0] == top[0]
    for u in range(len(parent)):
        for c in kids[u]:
            assert tokens[c] == top[rank[c]]
    assert tokens[kids[0][0]] == tokens[0]            # rank-0 child of the root repeats the root


def test_p5b_fc_embedding_half():
    """FC_j = [0 | I]: depth-j logits are LMhead(RMSNorm(embedding of the node's token))."""
    ov = _identity_overrides(TINY, "emb")
    ws, cfg, W = make(overrides=ov)
    parent, rank = synth.tree_for(TINY)
    prompt = synth.make_prompts(TINY, seed=4)[0][:10]
    s = O.SeqState(cfg)
    acc, (tokens, zs) = O.prefill(W, cfg, s, prompt, 16, parent, rank)
    lm = ws.get_f32("lm_head").astype(np.float64)
    hn = ws.get_f32("head_norm").astype(np.float64)
    for node, z in zs.items():
        if node == 0:
            continue
        e = lm[tokens[node]]
        g = e / np.sqrt((e ** 2).mean() + TINY.rms_eps) * hn
        np.testing.assert_allclose(z, lm @ g, atol=1e-9)


# ---------------------------------------------------------------- P6
def test_p6_attention_decoder_algebra():
    H, nh = 256, 4
    rng = np.random.default_rng(5)
    cfg = O.OracleConfig.from_shape(TINY, 8)
    x = rng.standard_normal((3, H)); y = rng.standard_normal((3, H))
    Wd = {"a.norm": 1 + 0.1 * rng.standard_normal(H)}
    for p in "qkv":
        Wd[f"a.w{p}"] = rng.standard_normal((H, H)) * 0.05
        Wd[f"a.b{p}"] = rng.standard_normal(H) * 0.05
    W = O.Weights(Wd.__getitem__)
    out = O.attention_decoder(W, "a.", cfg, x, y)
    v = y @ Wd["a.wv"].T + Wd["a.bv"]
    assert np.all(np.abs(out - x) <= np.abs(v) + 1e-12)          # |cos| <= 1
    # gate is constant within a head
    ratio = ((out - x) / v).reshape(3, nh, H // nh)
    assert np.allclose(ratio, ratio[..., :1])
    # direct per-head recomputation with explicit loops
    xn = x / np.sqrt((x ** 2).mean(-1, keepdims=True) + cfg.rms_eps) * Wd["a.norm"]
    q = xn @ Wd["a.wq"].T + Wd["a.bq"]; k = y @ Wd["a.wk"].T + Wd["a.bk"]
    for r in range(3):
        for h in range(nh):
            sl = slice(h * 64, (h + 1) * 64)
            c = float(q[r, sl] @ k[r, sl]) / (np.linalg.norm(q[r, sl]) * np.linalg.norm(k[r, sl]))
            np.testing.assert_allclose(out[r, sl], x[r, sl] + c * v[r, sl], atol=1e-12)
    # Wv = 0, bv = 0  ->  out == x
    W0 = dict(Wd); W0["a.wv"] = np.zeros((H, H)); W0["a.bv"] = np.zeros(H)
    np.testing.assert_array_equal(O.attention_decoder(O.Weights(W0.__getitem__), "a.", cfg, x, y), x)
    # bk = 0: scaling y leaves the gate unchanged, v scales linearly (bv = 0)
    W1 = dict(Wd); W1["a.bk"] = np.zeros(H); W1["a.bv"] = np.zeros(H)
    o1 = O.attention_decoder(O.Weights(W1.__getitem__), "a.", cfg, x, y)
    o2 = O.attention_decoder(O.Weights(W1.__getitem__), "a.", cfg, x, 3.0 * y)
    np.testing.assert_allclose(o2 - x, 3.0 * (o1 - x), atol=1e-10)
    # k parallel to q in every head -> gate 1 -> out = x + v ; antiparallel -> out = x - v
    W2 = dict(Wd); W2["a.bq"] = np.zeros(H); W2["a.bk"] = np.zeros(H)
    W2["a.wq"] = np.eye(H); W2["a.wk"] = np.eye(H); W2["a.norm"] = np.ones(H)
    xn2 = x / np.sqrt((x ** 2).mean(-1, keepdims=True) + cfg.rms_eps)
    v2 = (2.5 * xn2) @ W2["a.wv"].T + W2["a.bv"]
    np.testing.assert_allclose(O.attention_decoder(O.Weights(W2.__getitem__), "a.", cfg, x, 2.5 * xn2), x + v2, atol=1e-10)
    v3 = (-xn2) @ W2["a.wv"].T + W2["a.bv"]
    np.testing.assert_allclose(O.attention_decoder(O.Weights(W2.__getitem__), "a.", cfg, x, -xn2), x - v3, atol=1e-10)


def test_p6_cosine_matches_torch():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(6)
    H = 256
    cfg = O.OracleConfig.from_shape(TINY, 8)
    x = rng.standard_normal((5, H)); y = rng.standard_normal((5, H))
    y[2] = 0.0          # zero key vector: clamp path (bk = 0 below)
    Wd = {"a.norm": np.ones(H)}
    for p in "qkv":
        Wd[f"a.w{p}"] = rng.standard_normal((H, H)) * 0.05
        Wd[f"a.b{p}"] = np.zeros(H)
    out = O.attention_decoder(O.Weights(Wd.__getitem__), "a.", cfg, x, y)
    xt, yt = torch.tensor(x), torch.tensor(y)
    xn = xt * torch.rsqrt((xt ** 2).mean(-1, keepdim=True) + cfg.rms_eps)
    q = (xn @ torch.tensor(Wd["a.wq"]).T).view(-1, 64)
    k = (yt @ torch.tensor(Wd["a.wk"]).T).view(-1, 64)
    att = torch.nn.functional.cosine_similarity(q, k).view(-1, 4, 1)
    v = (yt @ torch.tensor(Wd["a.wv"]).T).view(-1, 4, 64) * att
    ref = xt + v.view(5, H)
    np.testing.assert_allclose(out, ref.numpy(), atol=1e-12)


# ---------------------------------------------------------------- P7
def test_p7_target_matches_hf_llama():
    torch = pytest.importorskip("torch")
    tr = pytest.importorskip("transformers")
    shape = synth.scaled(TINY, n_kv_heads=2)          # exercise grouped-query attention too
    ws, cfg, W = make(shape=shape)
    hf_cfg = tr.LlamaConfig(vocab_size=shape.vocab, hidden_size=shape.hidden, intermediate_size=shape.ffn,
                            num_hidden_layers=shape.n_layers, num_attention_heads=shape.n_q_heads,
                            num_key_value_heads=shape.n_kv_heads, head_dim=shape.head_dim,
                            rms_norm_eps=shape.rms_eps, rope_theta=shape.rope_base,
                            max_position_embeddings=256, attention_bias=False, mlp_bias=False,
                            tie_word_embeddings=False, attn_implementation="eager")
    try:
        hf_cfg.rope_parameters = {"rope_type": "default", "rope_theta": shape.rope_base}
    except Exception:
        pass
    model = tr.LlamaForCausalLM(hf_cfg).double().eval()
    sd = {"model.embed_tokens.weight": "embed", "model.norm.weight": "final_norm", "lm_head.weight": "lm_head"}
    for i in range(shape.n_layers):
        p = f"model.layers.{i}."
        sd.update({p + "input_layernorm.weight": f"layers.{i}.attn_norm",
                   p + "self_attn.q_proj.weight": f"layers.{i}.wq", p + "self_attn.k_proj.weight": f"layers.{i}.wk",
                   p + "self_attn.v_proj.weight": f"layers.{i}.wv", p + "self_attn.o_proj.weight": f"layers.{i}.wo",
                   p + "post_attention_layernorm.weight": f"layers.{i}.ffn_norm",
                   p + "mlp.gate_proj.weight": f"layers.{i}.w_gate", p + "mlp.up_proj.weight": f"layers.{i}.w_up",
                   p + "mlp.down_proj.weight": f"layers.{i}.w_down"})
    state = {k: torch.tensor(ws.get_f32(v).astype(np.float64)) for k, v in sd.items()}
    missing = model.load_state_dict(state, strict=False)
    assert not [k for k in missing.missing_keys if "rotary" not in k]
    toks = synth.make_prompts(shape, seed=9)[0][:33]
    with torch.no_grad():
        out = model(torch.tensor(toks[None].astype(np.int64)), output_hidden_states=True)
    s = O.SeqState(cfg)
    hid, log = O.verify_tree(W, cfg, s, toks, list(range(-1, 32)))
    # HF keeps its rotary tables in float32 even in a double model: agreement to ~2e-7
    np.testing.assert_allclose(log, out.logits[0].numpy(), atol=2e-6)


def test_p7_tree_attention_matches_sdpa():
    torch = pytest.importorskip("torch")
    shape = synth.scaled(TINY, n_layers=1)
    ws, cfg, W = make(shape=shape)
    rng = np.random.default_rng(11)
    n, L = 12, 7
    parent = rand_tree(rng, n)
    s = O.SeqState(cfg)
    s.kv.k[:] = rng.standard_normal(s.kv.k.shape); s.kv.v[:] = rng.standard_normal(s.kv.v.shape)
    s.L = L
    toks = rng.integers(0, shape.vocab, n)
    x0 = ws.get_f32("embed")[toks].astype(np.float64)
    k_before = s.kv.k.copy()
    hid, _ = O.verify_tree(W, cfg, s, toks, parent)
    # recompute the attention of that single layer with torch SDPA and an explicit bool mask
    P = "layers.0."
    g = lambda nme: torch.tensor(ws.get_f32(P + nme).astype(np.float64))
    xt = torch.tensor(x0)
    a = xt * torch.rsqrt((xt ** 2).mean(-1, keepdim=True) + shape.rms_eps) * g("attn_norm")
    d, nh = shape.head_dim, shape.n_q_heads
    q = (a @ g("wq").T).view(n, nh, d); k = (a @ g("wk").T).view(n, nh, d); v = (a @ g("wv").T).view(n, nh, d)
    depth = O.tree_depths(parent)
    pos = torch.tensor(L + depth, dtype=torch.float64)
    inv = 1.0 / (shape.rope_base ** (torch.arange(0, d, 2, dtype=torch.float64) / d))
    ang = pos[:, None] * inv[None]
    cos = torch.cat([ang.cos(), ang.cos()], -1)[:, None]; sin = torch.cat([ang.sin(), ang.sin()], -1)[:, None]
    rot = lambda t: torch.cat([-t[..., d // 2:], t[..., :d // 2]], -1)
    q = q * cos + rot(q) * sin; k = k * cos + rot(k) * sin
    K = torch.cat([torch.tensor(k_before[0, :L]), k], 0); V = torch.cat([torch.tensor(s.kv.v[0, :L]), v], 0)
    mask = torch.tensor(np.concatenate([np.ones((n, L), bool), O.ancestor_matrix(parent)], 1))
    o = torch.nn.functional.scaled_dot_product_attention(q.transpose(0, 1)[None], K.transpose(0, 1)[None],
                                                         V.transpose(0, 1)[None], attn_mask=mask[None, None])
    x1 = xt + o[0].transpose(0, 1).reshape(n, nh * d) @ g("wo").T
    f = x1 * torch.rsqrt((x1 ** 2).mean(-1, keepdim=True) + shape.rms_eps) * g("ffn_norm")
    x2 = x1 + (torch.nn.functional.silu(f @ g("w_gate").T) * (f @ g("w_up").T)) @ g("w_down").T
    np.testing.assert_allclose(hid, x2.numpy(), atol=1e-10)


# ---------------------------------------------------------------- P8
def test_p8_ranked_ids_bruteforce():
    rng = np.random.default_rng(8)
    z = rng.integers(0, 6, 200).astype(np.float64)      # many exact ties
    want = sorted(range(200), key=lambda i: (-z[i], i))[:9]
    assert list(O.ranked_ids(z, 9)) == want
    assert O.ranked_ids(z, 1)[0] == int(np.flatnonzero(z == z.max())[0])


def test_p8_accept_walk_bruteforce():
    rng = np.random.default_rng(12)
    V = 5
    for trial in range(200):
        n = int(rng.integers(1, 12))
        parent = rand_tree(rng, n)
        # children of one node carry distinct tokens (as ranked children do)
        kids = O.children_of(parent)
        tokens = np.zeros(n, dtype=np.int64)
        tokens[0] = rng.integers(0, V)
        for u in range(n):
            perm = rng.permutation(V)
            for i, c in enumerate(kids[u]):
                tokens[c] = perm[i % V]
        logits = rng.standard_normal((n, V))
        path, bonus = O.accept_greedy(tokens, logits, parent)
        am = logits.argmax(-1)
        # brute force: among all root-anchored paths, those whose every non-root node
        # carries the argmax of its parent; take the longest (unique since siblings differ)
        best = [0]
        for u in range(n):
            p = []; w = u
            while w >= 0:
                p.append(w); w = parent[w]
            p = p[::-1]
            if all(tokens[p[i]] == am[p[i - 1]] for i in range(1, len(p))) and len(p) > len(best):
                best = p
        assert path == best and bonus == am[best[-1]]


def test_tree_generator():
    parent, rank = synth.tree_for(TINY)
    assert len(parent) == 16 and parent[0] == -1
    assert all(0 <= parent[u] < u for u in range(1, 16))
    depth = O.tree_depths(parent)
    assert list(depth) == sorted(depth) and depth.max() <= 3
    assert all(rank[u] < TINY.tree_k[depth[u] - 1] for u in range(1, 16))
    # siblings have distinct ranks
    kids = O.children_of(parent)
    for u in range(16):
        assert len({int(rank[c]) for c in kids[u]}) == len(kids[u])
    for cid in (2, 4, 5):
        p, r = synth.tree_for(synth.CONFIGS[cid])
        s = synth.CONFIGS[cid]
        assert len(p) == s.tree_nodes and O.tree_depths(p).max() == s.draft_depths


def test_bf16_rounding_bits():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.140625, 1e-3], dtype=np.float32)
    b = synth.f32_to_bf16_bits(x)
    back = synth.bf16_bits_to_f32(b)
    # 1 + 2^-8 is a tie between 1 and 1+2^-7 -> even (1.0); 1 + 3*2^-8 ties to 1+2^-6
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == 1.015625 and back[3] == -2.5
    assert np.all(np.abs(back - x) <= np.abs(x) * 2.0 ** -8)
    torch = pytest.importorskip("torch")
    r = np.random.default_rng(0).standard_normal(10000).astype(np.float32)
    t = torch.tensor(r).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(synth._f32_to_bf16_bits_np(r), t)
    big = np.random.default_rng(1).standard_normal(1 << 20).astype(np.float32)
    np.testing.assert_array_equal(synth.f32_to_bf16_bits(big), synth._f32_to_bf16_bits_np(big))


# ---------------------------------------------------------------- cost figures the paper states
def _golden(name):
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "draft_cost_ratios.txt")
    for line in open(path):
        f = line.split()
        if f and f[0] == name:
            return float(f[1]), float(f[2])
    raise KeyError(name)


def test_draft_head_cost_matches_the_papers_figures():
    """Which weight matrices the oracle's draft step actually multiplies by, priced at the paper's two model shapes,
    against the two cost statements of Sec. 3.3 (tests/golden/draft_cost_ratios.txt).  A different reading of the head
    (an output projection inside the Attention Decoder, an FC over the state alone, per-depth Attention Decoders that
    also project the embedding twice, an augmenting block that is not a decoder layer) moves the ratio out of range."""
    ws, cfg, W0 = make(gain_jitter=0.0, max_seq=64)
    used = []
    W = O.Weights(lambda n: (used.append(n), ws.get_f32(n))[1], np.float64, cache=False)
    seq = O.SeqState(cfg)
    rng = np.random.default_rng(3)
    hid = rng.standard_normal((2, TINY.hidden))
    # root with one child: AD1, augmenting block, head 0 only
    O.draft_tree(W, cfg, seq, hid, [5, 9], [-1, 0], [0, 0])
    first = list(used)
    used.clear()
    # a chain root -> a -> b: the second call adds exactly ONE regressive update (node a has a child)
    seq2 = O.SeqState(cfg)
    O.draft_tree(W, cfg, seq2, hid, [5, 9], [-1, 0, 1], [0, 0, 0])
    extra = list(used)
    for n in first:
        extra.remove(n)
    mats = lambda names: sorted(n for n in names if len(ws.shapes[n]) == 2 and n not in ("lm_head", "embed"))
    update = mats(extra)
    assert update == ["ad2.wk", "ad2.wq", "ad2.wv", "fc.1.w"], update
    aug = [n for n in mats(first) if n.startswith("aug.")]
    layer_names = sorted(f"aug.0.{k}" for k, v in synth.layer_tensor_shapes(TINY).items() if len(v) == 2)
    assert aug == layer_names
    want, tol = _golden("aug_block_in_decoder_layers")
    assert abs(len(aug) / len(layer_names) / TINY.aug_layers - want) <= tol
    want, tol = _golden("decoder_layer_over_per_depth_update")
    for c in (2, 3):                       # the paper's two targets: Vicuna-7B and LLaMA3-8B shapes
        shapes = synth.weight_shapes(synth.CONFIGS[c])
        size = lambda n: int(np.prod(shapes[n]))
        layer = sum(size(f"layers.0.{k}") for k, v in synth.layer_tensor_shapes(synth.CONFIGS[c]).items() if len(v) == 2)
        upd = sum(size(n) for n in update)
        assert abs(layer / upd - want) <= tol, (c, layer / upd)


# ---------------------------------------------------------------- P10: the draft head's wiring (Sec. 3.1, 3.2, App. A.3)
def _additive_overrides(shape, rng):
    """A head whose result has a closed form in the tokens alone.  Both Attention Decoders get Wq = Wk = 0 and
    bq = bk = one non-zero vector (every head's cosine is exactly 1), Wv = I, bv = 0: AD(x, y) = x + y.  The
    augmenting layer keeps its attention but projects to zero (Wo = W_down = 0), so it returns its input and only
    fills its cache.  FC_j = [2I | 0] without bias, head-norm gains 1."""
    H = shape.hidden
    z = lambda *s: np.zeros(s, np.float32)
    c = (0.5 + rng.random(H)).astype(np.float32)
    ov = {}
    for ad in ("ad1", "ad2"):
        ov[f"{ad}.wq"] = z(H, H); ov[f"{ad}.wk"] = z(H, H)
        ov[f"{ad}.bq"] = c; ov[f"{ad}.bk"] = c
        ov[f"{ad}.wv"] = np.eye(H, dtype=np.float32); ov[f"{ad}.bv"] = z(H)
    for l in range(shape.aug_layers):
        ov[f"aug.{l}.wo"] = z(H, shape.n_q_heads * shape.head_dim)
        ov[f"aug.{l}.w_down"] = z(H, shape.ffn)
    for j in range(1, shape.draft_depths):
        w = z(H, 2 * H)
        w[:, :H] = 2.0 * np.eye(H)
        ov[f"fc.{j}.w"] = w; ov[f"fc.{j}.b"] = z(H)
    ov["head_norm"] = np.ones(H, np.float32)
    return ov


def _wiring_pin(draft_tree_fn):
    """Runs `draft_tree_fn` on the additive head and checks every returned logit vector and the augmenting block's
    cached V rows against values computed here from the tokens alone:
        s_root = h_{m-1} + E[n_{m-1}]                       (AD1 pairs row i with the token that followed it)
        s_u    = s_root + sum of E[tok_w] over the nodes w != root on the path root -> u   (AD2 chains the STATE,
                 and adds the node's OWN token embedding)
        z_root = W_lm RMSNorm(FC0 s_root + b0),   z_u = W_lm RMSNorm(2 s_u)
        V_aug[i] = Wv_aug RMSNorm(h_i + E[n_i]; attn_norm)   (no rotation on V: shows the pairing of every row)
    with E = rows of the LM-head weight."""
    rng = np.random.default_rng(41)
    shape = TINY
    ws, cfg, W = make(shape=shape, gain_jitter=0.1, overrides=_additive_overrides(shape, rng), max_seq=64)
    parent, rank = synth.tree_for(shape)
    n, H, m = len(parent), shape.hidden, 3
    hid = rng.standard_normal((m, H))
    nxt = [int(t) for t in rng.integers(0, shape.vocab, m)]
    seq = O.SeqState(cfg)
    tokens, zs = draft_tree_fn(W, cfg, seq, hid, nxt, parent, rank)
    lm = ws.get_f32("lm_head").astype(np.float64)
    rms = lambda v: v / np.sqrt(np.mean(v * v) + shape.rms_eps)
    kids = O.children_of(parent)
    assert tokens[0] == nxt[-1]
    s_root = hid[m - 1] + lm[nxt[m - 1]]
    checked_deep = 0
    for u in range(n):
        if not kids[u]:
            continue
        s = s_root.copy()
        w = u
        while w > 0:                          # explicit walk up the path, own token of every node on it
            s += lm[int(tokens[w])]
            w = int(parent[w])
        if u == 0:
            g = ws.get_f32("fc0.w").astype(np.float64) @ s + ws.get_f32("fc0.b").astype(np.float64)
        else:
            g = 2.0 * s
            checked_deep += int(parent[u] != 0)
        np.testing.assert_allclose(zs[u], lm @ rms(g), atol=1e-9, err_msg=f"node {u}")
        # children carry the ranked ids of exactly these logits
        order = sorted(range(shape.vocab), key=lambda i: (-zs[u][i], i))
        for c in kids[u]:
            assert tokens[c] == order[rank[c]]
    assert checked_deep >= 1                  # a node whose parent is not the root: chaining is exercised
    wv = ws.get_f32("aug.0.wv").astype(np.float64)
    gain = ws.get_f32("aug.0.attn_norm").astype(np.float64)
    for i in range(m):
        want = wv @ (rms(hid[i] + lm[nxt[i]]) * gain)
        np.testing.assert_allclose(seq.aug_kv.v[0, i].reshape(-1), want, atol=1e-9, err_msg=f"aug V row {i}")
    assert seq.aug_L == m


def test_p10_draft_wiring_closed_form():
    _wiring_pin(O.draft_tree)


def _mutant(replacements):
    """draft_tree with one line of its source replaced (a planted wiring mistake), compiled beside the oracle."""
    import inspect
    src = inspect.getsource(O.draft_tree)
    for old, new in replacements:
        assert src.count(old) == 1, old
        src = src.replace(old, new)
    ns = dict(vars(O))
    exec(compile(src, "<mutant draft_tree>", "exec"), ns)
    return ns["draft_tree"]


@pytest.mark.parametrize("name,replacements", [
    # AD2 / FC_j fed the PARENT's token embedding instead of the node's own
    ("parent_token", [("e = emb(tokens[node])", "e = emb(tokens[int(parent[node])])")]),
    # the FC's output handed to the next depth instead of the Attention Decoder's state
    ("chain_fc_output", [("expand(node, W(\"lm_head\") @ rmsnorm(g, W(\"head_norm\"), cfg.rms_eps))\n    return",
                          "state[node] = g\n        expand(node, W(\"lm_head\") @ rmsnorm(g, W(\"head_norm\"), cfg.rms_eps))\n    return")]),
    # AD1 pairs hidden row i with the token of row i-1 (shifted pairing)
    ("ad1_shifted_pairing", [("emb(next_tok))", "emb(np.roll(next_tok, 1)))")]),
    # AD2 takes the ROOT's state instead of the parent's
    ("root_state", [("state[int(parent[node])][None, :]", "state[0][None, :]")]),
    # only an EARLIER accepted row is paired with the wrong token (visible in the augmenting block's cache alone)
    ("ad1_earlier_row_mispaired", [("emb(next_tok))", "emb(np.array([next_tok[0], next_tok[0], next_tok[2]])))")]),
], ids=lambda v: v if isinstance(v, str) else "")
def test_p10_pin_detects_planted_wiring_mistakes(name, replacements):
    mutant = _mutant(replacements)
    with pytest.raises(AssertionError):
        _wiring_pin(mutant)


# ---------------------------------------------------------------- P11: the dynamic (score-pruned) tree, Sec. 4.1
def _full_static_tree(k, D):
    """Complete k-ary tree of depth D in breadth-first order with ranks 0..k-1 under every parent."""
    parent, rank, depth = [-1], [0], [0]
    level = [0]
    for _ in range(D):
        nxt = []
        for u in level:
            for i in range(k):
                parent.append(u); rank.append(i); depth.append(depth[u] + 1)
                nxt.append(len(parent) - 1)
        level = nxt
    return np.asarray(parent), np.asarray(rank), np.asarray(depth)


def _path_key(parent, rank, u):
    out = []
    while u > 0:
        out.append(int(rank[u])); u = int(parent[u])
    return tuple(out[::-1])


def _dynamic_case(seed=5, m=2):
    ws, cfg, W = make(gain_jitter=0.1, max_seq=64)
    rng = np.random.default_rng(seed)
    hid = rng.standard_normal((m, TINY.hidden))
    nxt = [int(t) for t in rng.integers(0, TINY.vocab, m)]
    return ws, cfg, W, hid, nxt


def _brute_scores(W, cfg, hid, nxt, k, D):
    """Cumulative draft log-probability of EVERY node of the complete k-ary tree, from the static-tree oracle's
    logits (pinned by P5/P10) and a log-softmax written out here."""
    parent, rank, depth = _full_static_tree(k, D)
    seq = O.SeqState(cfg)
    tokens, zs = O.draft_tree(W, cfg, seq, hid, nxt, parent, rank)
    score = np.zeros(len(parent))
    for u in range(1, len(parent)):
        z = zs[int(parent[u])].astype(np.float64)
        lse = np.log(np.sum(np.exp(z - z.max()))) + z.max()
        score[u] = score[parent[u]] + z[tokens[u]] - lse
    return parent, rank, depth, tokens, score


def test_p11_dynamic_tree_is_the_best_prefixes_of_the_full_tree():
    """No frontier pruning (every candidate of a depth is expanded): the dynamic tree must be exactly the
    n_nodes - 1 most probable prefixes among ALL prefixes of the complete tree, found here by brute force."""
    k, D, N = 3, TINY.draft_depths, 14
    ws, cfg, W, hid, nxt = _dynamic_case()
    parent, rank, depth, tokens, score = _brute_scores(W, cfg, hid, nxt, k, D)
    order = sorted(range(1, len(parent)), key=lambda u: (-score[u], depth[u], u))[:N - 1]
    want = {_path_key(parent, rank, u): int(tokens[u]) for u in order}
    dyn = O.draft_tree_dynamic(W, cfg, O.SeqState(cfg), hid, nxt, topk=k, frontier=k ** D, n_nodes=N)
    got = {_path_key(dyn["parent"], dyn["rank"], u): int(dyn["tokens"][u]) for u in range(1, N)}
    assert got == want
    assert dyn["tokens"][0] == nxt[-1] and len(dyn["tokens"]) == N
    # scores reported per candidate equal the brute-force ones
    by_path = {_path_key(parent, rank, u): score[u] for u in range(1, len(parent))}
    for c in range(1, len(dyn["cand_token"])):
        path, w = [], c
        while w > 0:
            path.append(dyn["cand_rank"][w]); w = dyn["cand_parent"][w]
        assert abs(dyn["cand_score"][c] - by_path[tuple(path[::-1])]) < 1e-9


def test_p11_frontier_pruning_bruteforce():
    """frontier = 2: at every depth only the two best candidates (among the children of the previous frontier)
    are expanded; checked against the complete tree's brute-force scores."""
    k, D, N, K = 3, TINY.draft_depths, 10, 2
    ws, cfg, W, hid, nxt = _dynamic_case(seed=6, m=1)
    parent, rank, depth, tokens, score = _brute_scores(W, cfg, hid, nxt, k, D)
    kids = O.children_of(parent)
    alive = list(kids[0])                       # generated candidates of the current depth
    generated = list(alive)
    for j in range(1, D):
        front = sorted(alive, key=lambda u: (-score[u], u))[:K]
        alive = [c for u in front for c in kids[u]]
        generated += alive
    keep = sorted(generated, key=lambda u: (-score[u], depth[u], u))[:N - 1]
    want = {_path_key(parent, rank, u): int(tokens[u]) for u in keep}
    dyn = O.draft_tree_dynamic(W, cfg, O.SeqState(cfg), hid, nxt, topk=k, frontier=K, n_nodes=N)
    got = {_path_key(dyn["parent"], dyn["rank"], u): int(dyn["tokens"][u]) for u in range(1, N)}
    assert got == want
    assert len(dyn["cand_token"]) == 1 + k + (D - 1) * K * k


def test_p11_scores_are_normalised_log_probabilities():
    """topk = whole vocabulary on a tiny head: the exp(score) of all depth-1 candidates sum to 1, and those of
    the children of any expanded candidate sum to that candidate's own probability."""
    shape = synth.scaled(TINY, name="tiny-v32", vocab=32, seed=3)
    ws, cfg, W = make(shape=shape, gain_jitter=0.1, max_seq=32)
    rng = np.random.default_rng(1)
    hid = rng.standard_normal((1, shape.hidden))
    dyn = O.draft_tree_dynamic(W, cfg, O.SeqState(cfg), hid, [7], topk=32, frontier=3, n_nodes=20)
    sc, par, dep = np.asarray(dyn["cand_score"]), np.asarray(dyn["cand_parent"]), np.asarray(dyn["cand_depth"])
    assert abs(np.exp(sc[dep == 1]).sum() - 1.0) < 1e-12
    for front in dyn["frontier"]:
        for c in front:
            assert abs(np.exp(sc[par == c]).sum() - np.exp(sc[c])) < 1e-12
    assert len({dyn["cand_token"][c] for c in range(len(sc)) if par[c] == 0}) == 32   # all distinct tokens


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_p11_dynamic_tree_invariants(seed):
    ws, cfg, W, hid, nxt = _dynamic_case(seed=10 + seed, m=3)
    N = 16
    dyn = O.draft_tree_dynamic(W, cfg, O.SeqState(cfg), hid, nxt, topk=4, frontier=3, n_nodes=N)
    parent, rank, toks = dyn["parent"], dyn["rank"], dyn["tokens"]
    assert parent[0] == -1 and all(0 <= parent[u] < u for u in range(1, N))
    assert all(parent[u] >= parent[u - 1] for u in range(2, N))                  # breadth-first: children contiguous
    depth = O.tree_depths(parent)
    assert list(depth) == sorted(depth) and depth.max() <= TINY.draft_depths
    kids = O.children_of(parent)
    for u in range(N):
        assert [int(rank[c]) for c in kids[u]] == sorted({int(rank[c]) for c in kids[u]})   # distinct, ascending
        assert len({int(toks[c]) for c in kids[u]}) == len(kids[u])
    sc = {n: dyn["cand_score"][c] for n, c in enumerate(dyn["keep"])}
    assert all(sc[u] <= sc[int(parent[u])] + 1e-12 for u in range(1, N))         # a child never outscores its parent
    # every kept candidate beats every candidate that was left out
    left = [c for c in range(1, len(dyn["cand_token"])) if c not in set(dyn["keep"])]
    assert min(sc[u] for u in range(1, N)) >= max(dyn["cand_score"][c] for c in left) - 1e-12
    # follow mode reproduces the same tree from the recorded decisions
    again = O.draft_tree_dynamic(W, cfg, O.SeqState(cfg), hid, nxt, topk=4, frontier=3, n_nodes=N,
                                 follow=dict(tokens=dyn["cand_token"], frontier=dyn["frontier"], keep=dyn["keep"]))
    np.testing.assert_array_equal(again["tokens"], toks)
    np.testing.assert_array_equal(again["parent"], parent)


def test_p11_dynamic_tree_is_lossless():
    """Greedy speculative decoding with a dynamic tree per step emits the plain greedy text (Sec. 2.1)."""
    ws, cfg, W = make(gain_jitter=0.0, max_seq=200)
    prompt = synth.make_prompts(TINY, seed=9)[0][:24]
    seq = O.SeqState(cfg)
    acc, _ = O.prefill(W, cfg, seq, prompt, 16, [-1], [0])
    emitted = [acc["new_tokens"][-1]]
    seq.aug_L -= acc["m"]                             # the last chunk's rows are drafted again below (same values)
    for step in range(6):
        dyn = O.draft_tree_dynamic(W, cfg, seq, acc["hid_acc"], acc["next_tok"], topk=3, frontier=3, n_nodes=12)
        hidden, logits = O.verify_tree(W, cfg, seq, dyn["tokens"], dyn["parent"])
        acc = O.accept_and_compact(cfg, seq, dyn["tokens"], logits, hidden, dyn["parent"])
        emitted.extend(acc["new_tokens"])
        assert seq.aug_L == seq.L - acc["m"]          # the augmenting block catches up in the next draft call
    ref, _ = O.plain_greedy(W, cfg, prompt, len(emitted))
    assert emitted == ref


# ---------------------------------------------------------------- P12: verification at temperature > 0 (Table 1, T = 1)
def _chi2_ok(counts, probs, z=5.0):
    """Pearson statistic within z standard deviations of its mean (dof = k - 1; fixed seeds, so deterministic)."""
    n = counts.sum()
    exp = n * probs
    stat = ((counts - exp) ** 2 / exp).sum()
    dof = len(probs) - 1
    return stat <= dof + z * np.sqrt(2 * dof)


def test_p12_sampled_acceptance_emits_the_target_distribution():
    """Whatever the tree offers, the token emitted after a visited node is distributed as softmax(logits / T) of
    that node (the method stays lossless at T > 0): seeded Monte-Carlo over the uniforms, at the root and, given the
    walk reached it, at a depth-1 node."""
    rng = np.random.default_rng(12)
    V, T = 7, 1.0
    parent = [-1, 0, 0, 0, 1, 1, 2]
    tokens = [3, 2, 4, 1, 3, 5, 6]
    logits = rng.standard_normal((7, V)) * 1.5
    first = np.zeros(V)
    second = {1: np.zeros(V), 2: np.zeros(V)}
    for _ in range(30000):
        path, bonus, _ = O.accept_sampled(tokens, logits, parent, T, rng.random((7, 17)))
        out = [tokens[c] for c in path[1:]] + [bonus]
        first[out[0]] += 1
        if len(path) > 1 and path[1] in second:
            second[path[1]][out[1]] += 1
    soft = lambda z: np.exp(z - z.max()) / np.exp(z - z.max()).sum()
    assert _chi2_ok(first, soft(logits[0] / T))
    for node, cnt in second.items():
        assert cnt.sum() > 2000
        assert _chi2_ok(cnt, soft(logits[node] / T))
    # and at another temperature
    first[:] = 0
    for _ in range(20000):
        path, bonus, _ = O.accept_sampled(tokens, logits, parent, 0.6, rng.random((7, 17)))
        first[tokens[path[1]] if len(path) > 1 else bonus] += 1
    assert _chi2_ok(first, soft(logits[0] / 0.6))


def test_p12_one_child_exact_by_quadrature():
    """One candidate below the root: the outcome as a function of the two uniforms, integrated on a midpoint grid,
    reproduces the target probabilities to the grid's resolution (no formula of the procedure is used here)."""
    rng = np.random.default_rng(3)
    V, G = 5, 120
    logits = rng.standard_normal((2, V))
    parent, tokens = [-1, 0], [0, 3]
    cnt = np.zeros(V)
    u = np.zeros((2, 17))
    for i in range(G):
        for j in range(G):
            u[0, 0] = (i + 0.5) / G
            u[0, 16] = (j + 0.5) / G
            path, bonus, _ = O.accept_sampled(tokens, logits, parent, 1.0, u)
            cnt[tokens[path[1]] if len(path) > 1 else bonus] += 1
    p = np.exp(logits[0] - logits[0].max()); p /= p.sum()
    assert np.abs(cnt / G ** 2 - p).max() <= 2.5 / G


def test_p12_zero_temperature_limit_is_greedy_acceptance():
    rng = np.random.default_rng(5)
    V = 9
    for trial in range(100):
        n = int(rng.integers(1, 10))
        parent = rand_tree(rng, n)
        kids = O.children_of(parent)
        tokens = np.zeros(n, dtype=np.int64)
        for u in range(n):
            perm = rng.permutation(V)
            for i, c in enumerate(kids[u]):
                tokens[c] = perm[i]
        logits = rng.standard_normal((n, V))
        path, bonus, _ = O.accept_sampled(tokens, logits, parent, 1e-4, rng.random((n, 17)))
        assert (path, bonus) == O.accept_greedy(tokens, logits, parent)


def test_p12_leaf_draw_inverts_the_cumulative_sum():
    rng = np.random.default_rng(8)
    V = 50
    logits = rng.standard_normal((1, V)) * 2
    p = np.exp(logits[0] - logits[0].max()); p /= p.sum()
    for _ in range(200):
        u = rng.random((1, 17))
        _, bonus, _ = O.accept_sampled([0], logits, [-1], 1.0, u)
        acc, want = 0.0, V - 1
        for t in range(V):                  # plain loop: first token whose running sum passes the uniform
            acc += p[t]
            if acc > u[0, 16]:
                want = t
                break
        assert bonus == want


# ---------------------------------------------------------------- P13: linear-size tree mask (Appendix A.1)
def test_p13_interval_labels_rebuild_the_tree_mask():
    """The two-integers-per-node labels give exactly the 2-D tree mask (built independently by walking parent
    pointers), for random trees, a chain and a star; plus what a depth-first numbering fixes: enter is a permutation
    of 0..n-1 with the root first, exit - enter + 1 is the subtree size, a chain's intervals are nested and a star's
    leaves are single points."""
    rng = np.random.default_rng(3)
    trees = [rand_tree(rng, n) for n in (2, 5, 16, 64, 96, 200)]
    trees.append(np.arange(-1, 40))                       # chain
    trees.append(np.array([-1] + [0] * 30))               # star
    trees.append(np.asarray(synth.tree_for(synth.CONFIGS[5])[0]))
    for parent in trees:
        n = len(parent)
        enter, exit_ = O.interval_labels(parent)
        walked = np.zeros((n, n), dtype=bool)             # by parent pointers, not through the oracle's own matrix
        for u in range(n):
            w = u
            while w >= 0:
                walked[u, w] = True
                w = int(parent[w])
        assert np.array_equal(O.mask_from_intervals(enter, exit_), walked)
        assert np.array_equal(O.ancestor_matrix(parent), walked)
        assert sorted(enter.tolist()) == list(range(n)) and enter[0] == 0 and exit_[0] == n - 1
        size = walked.sum(axis=0)                          # nodes that have w on their path = subtree size of w
        assert np.array_equal(exit_ - enter + 1, size)
    enter, exit_ = O.interval_labels(np.arange(-1, 39))   # a chain of 40 nodes
    assert np.array_equal(enter, np.arange(40)) and np.all(exit_ == 39)
    enter, exit_ = O.interval_labels(np.array([-1] + [0] * 30))
    assert np.array_equal(enter[1:], exit_[1:])


def test_p13_a_wrong_comparison_is_caught():
    """Planted mistakes in the comparison (strict instead of inclusive, exit of the wrong node) break the mask."""
    parent = rand_tree(np.random.default_rng(4), 24)
    enter, exit_ = O.interval_labels(parent)
    good = O.ancestor_matrix(parent)
    e = enter
    strict = (e[None, :] < e[:, None]) & (e[:, None] <= exit_[None, :])
    swapped = (e[None, :] <= e[:, None]) & (e[:, None] <= exit_[:, None])
    assert not np.array_equal(strict, good) and not np.array_equal(swapped, good)
