"""Lock-step parity harness: the HIP path (through the C ABI) beside the CPU oracle.

Both sides get identical seeded weights and inputs every call.  Integer results must be
identical except inside the tie zone: a GPU argmax / rank choice is tolerated only if, under the
ORACLE's logits, its value is within `tol` of the oracle's own choice; the oracle then follows
the GPU's choice so later calls stay comparable.  Everything else is compared element-wise.
"""
from __future__ import annotations

from typing import Callable, Dict, List, Optional

import numpy as np

from oracle import clover2_oracle as O
from paper_2408_00264_amd import clover, synth


def bfs_tree_random(rng, n, max_depth, max_kids=4):
    """Random rooted tree in true breadth-first order with distinct sibling ranks."""
    parent, rank, depth = [-1], [0], [0]
    frontier = [0]
    while len(parent) < n and frontier:
        nxt = []
        for u in frontier:
            if depth[u] >= max_depth:
                continue
            k = int(rng.integers(0, max_kids + 1))
            if u == 0 or (not nxt and u == frontier[-1]):
                k = max(k, 1)
            ranks = rng.permutation(8)[:k]
            for r in sorted(ranks):
                if len(parent) >= n:
                    break
                parent.append(u); rank.append(int(r)); depth.append(depth[u] + 1)
                nxt.append(len(parent) - 1)
        frontier = nxt
    return np.asarray(parent, np.int32), np.asarray(rank, np.int32)


class Lockstep:
    def __init__(self, shape, parent, rank, max_seq: int, flags: int = 0, gain_jitter: float = 0.0,
                 oracle_dtype=np.float64, max_nodes: Optional[int] = None, batch: int = 1,
                 overrides: Optional[Dict[str, np.ndarray]] = None, dynamic: Optional[tuple] = None,
                 prefill_rows: int = 0):
        self.shape = shape
        self.dyn = dynamic                  # (n_nodes, topk, frontier): score-pruned tree, new topology per draft call
        self.parent = np.asarray(parent, np.int32)
        self.rank = np.asarray(rank, np.int32)
        self.tol = 3e-2 if shape.bf16 else 1e-4
        self.store = synth.WeightStore(shape, gain_jitter=gain_jitter, overrides=overrides)
        self.ocfg = O.OracleConfig.from_shape(shape, max_seq, oracle_dtype)
        self.W = O.Weights(self.store.get_f32, oracle_dtype)
        self.B = batch
        self.R = max_nodes or len(parent)
        self.dev_w = clover.upload_weights(self.store)
        self.gpu = clover.Clover(shape, self.dev_w, self.parent, self.rank, batch, max_seq, self.R, flags,
                                 prefill_rows=prefill_rows)
        self.seqs = [O.SeqState(self.ocfg) for _ in range(batch)]
        self.parents = [self.parent for _ in range(batch)]      # topology per sequence (differs with a dynamic tree)
        self.score_tol = 5e-3 if shape.bf16 else 1e-4           # cumulative draft log-probabilities (up to D terms)
        self.acc: List[dict] = [None] * batch
        self.tie_events = 0
        self.max_logit_err = 0.0
        self.max_hidden_err = 0.0
        self.max_draft_logit_err = 0.0
        self.max_kv_err = 0.0
        # tolerances: logits as the target states them; K/V rows and hidden states are not bounded by it, the
        # bounds below are what 16 mantissa bits through the stack give with a wide margin (a lost low plane
        # of the split-bf16 cache alone is ~2^-9 |x| ~ 1e-2 and fails them)
        self.kv_atol = 2e-3 if shape.bf16 else 1e-4
        self.hidden_atol = 1e-2 if shape.bf16 else 1e-4
        self.gpu.capture_draft_logits(True)

    @property
    def n_nodes(self) -> int:
        return self.dyn[0] if self.dyn is not None else len(self.parent)

    # ------------------------------------------------------------------------------------
    def _check_draft(self, b: int, gpu_tokens: np.ndarray, parent, rank) -> None:
        """Oracle draft for sequence b on the oracle's own hand-off state, following the GPU's tokens."""
        if self.dyn is not None:
            return self._check_draft_dynamic(b, gpu_tokens)
        acc = self.acc[b]
        toks, zs = O.draft_tree(self.W, self.ocfg, self.seqs[b], acc["hid_acc"], acc["next_tok"], parent, rank,
                                forced_tokens=gpu_tokens)
        assert int(gpu_tokens[0]) == int(acc["next_tok"][-1]), "root token"
        kids = O.children_of(parent)
        # every draft logit the GPU ranked, element by element (internal nodes in index order are grouped by depth)
        cap = self.gpu.draft_logits
        if cap is not None and zs:
            depth = O.tree_depths(parent)
            internal = sorted(zs)
            by_depth: Dict[int, List[int]] = {}
            for u in internal:
                by_depth.setdefault(int(depth[u]), []).append(u)
            start = 0
            for j in sorted(by_depth):
                nodes = by_depth[j]
                base = self.B * start + b * len(nodes)
                got = cap[base:base + len(nodes)].cpu().numpy()
                for r, u in enumerate(nodes):
                    err = float(np.abs(got[r] - zs[u]).max())
                    self.max_draft_logit_err = max(self.max_draft_logit_err, err)
                    assert err <= self.tol, f"seq {b} node {u} (depth {j}): draft logits max-abs error {err:.3e}"
                start += len(nodes)
        for u, z in zs.items():
            need = 1 + max(rank[c] for c in kids[u])
            top = O.ranked_ids(z, need)
            got = [int(gpu_tokens[c]) for c in kids[u]]
            assert len(set(got)) == len(got), f"duplicate sibling tokens under node {u}"
            for c in kids[u]:
                want = int(top[rank[c]])
                if int(gpu_tokens[c]) != want:
                    gap = abs(float(z[want]) - float(z[int(gpu_tokens[c])]))
                    assert gap <= self.tol, (f"seq {b} node {c} (rank {rank[c]} of node {u}): gpu token "
                                             f"{int(gpu_tokens[c])} vs oracle {want}, oracle logit gap {gap:.3e}")
                    self.tie_events += 1

    def _check_draft_dynamic(self, b: int, gpu_tokens: np.ndarray) -> None:
        """Dynamic tree: the oracle follows the GPU's decisions (candidate tokens, expanded candidates, kept set)
        and every decision must be (near-)optimal under the ORACLE's logits and scores; the breadth-first
        numbering that follows from the kept set must be identical."""
        n_nodes, topk, front = self.dyn
        gt = self.gpu.read_dynamic_tree(b)
        D = self.shape.draft_depths
        F, n_cand = [1], topk
        for j in range(1, D):
            F.append(min(front, n_cand)); n_cand = F[-1] * topk
        C = 1 + topk + sum(F[j] * topk for j in range(1, D))
        follow = dict(tokens=[int(t) for t in gt["cand_token"][:C]],
                      frontier=[[int(c) for c in gt["frontier"][j][:F[j]]] for j in range(1, D)],
                      keep=[int(c) for c in gt["keep"]])
        acc = self.acc[b]
        assert follow["tokens"][0] == int(acc["next_tok"][-1]) == int(gpu_tokens[0]), "root token"
        dyn = O.draft_tree_dynamic(self.W, self.ocfg, self.seqs[b], acc["hid_acc"], acc["next_tok"], topk, front, n_nodes,
                                   follow=follow)
        score = np.asarray(dyn["cand_score"]); par = np.asarray(dyn["cand_parent"]); dep = np.asarray(dyn["cand_depth"])
        # (1) tokens of every expansion against the oracle's ranking of that candidate's logits (tie zone allowed)
        for c, z in dyn["logits"].items():
            kids = [k for k in range(C) if par[k] == c and k != 0]
            got = [follow["tokens"][k] for k in kids]
            assert len(set(got)) == len(got) == topk, f"candidate {c}: children {got}"
            top = O.ranked_ids(z, topk)
            for i, k in enumerate(kids):
                if got[i] != int(top[i]):
                    gap = abs(float(z[int(top[i])]) - float(z[got[i]]))
                    assert gap <= self.tol, f"seq {b} candidate {k}: token {got[i]} vs oracle {int(top[i])}, gap {gap:.3e}"
                    self.tie_events += 1
        # (2) scores
        err = float(np.abs(gt["cand_score"][1:C] - score[1:C]).max())
        self.max_score_err = max(getattr(self, "max_score_err", 0.0), err)
        assert err <= self.score_tol, f"seq {b}: cumulative draft log-probabilities differ by {err:.3e}"
        # (3) expanded candidates per depth: none left out that beats a chosen one by more than the tolerance
        for j in range(1, D):
            level = [c for c in range(C) if dep[c] == j]
            chosen = follow["frontier"][j - 1]
            out = [c for c in level if c not in set(chosen)]
            if out:
                slack = max(score[c] for c in out) - min(score[c] for c in chosen)
                assert slack <= 2 * self.score_tol, f"seq {b} depth {j}: a left-out candidate beats an expanded one by {slack:.3e}"
                self.tie_events += int(slack > 0)
            order = [score[c] for c in chosen]
            assert all(order[i] >= order[i + 1] - 2 * self.score_tol for i in range(len(order) - 1)), "frontier order"
        # (4) kept set
        kept = set(follow["keep"])
        left = [c for c in range(1, C) if c not in kept]
        if left:
            slack = max(score[c] for c in left) - min(score[c] for c in kept if c != 0)
            assert slack <= 2 * self.score_tol, f"seq {b}: a left-out candidate beats a kept one by {slack:.3e}"
            self.tie_events += int(slack > 0)
        # numbering: fully determined by the kept set
        np.testing.assert_array_equal(dyn["keep"], gt["keep"])
        np.testing.assert_array_equal(dyn["parent"], gt["parent"])
        np.testing.assert_array_equal(dyn["rank"], gt["rank"])
        np.testing.assert_array_equal(dyn["tokens"], gpu_tokens[:n_nodes])
        self.parents[b] = np.asarray(dyn["parent"], np.int32)
        # (5) every draft logit the GPU ranked
        cap = self.gpu.draft_logits
        if cap is not None:
            start = 0
            for j in range(D):
                nodes = [0] if j == 0 else follow["frontier"][j - 1]
                base = self.B * start + b * len(nodes)
                got = cap[base:base + len(nodes)].cpu().numpy()
                for r, c in enumerate(nodes):
                    e = float(np.abs(got[r] - dyn["logits"][c]).max())
                    self.max_draft_logit_err = max(self.max_draft_logit_err, e)
                    assert e <= self.tol, f"seq {b} candidate {c} (depth {j}): draft logits max-abs error {e:.3e}"
                start += len(nodes)

    def _follow_sampled(self, b: int, tokens, o_logits, o_hidden, gpu_path, gpu_bonus, temperature, uni) -> dict:
        """Sampled verification: the oracle runs on the same uniforms; where the GPU decided otherwise, its decision
        must lie within the tolerance of the oracle's own threshold (an acceptance ratio, or a step of the cumulative
        sum), and the oracle then follows it."""
        parent = self.parents[b]
        kids = O.children_of(parent)
        path, bonus, rec = O.accept_sampled(tokens, o_logits, parent, temperature, uni)
        if path != gpu_path or bonus != gpu_bonus:
            # relative slack of a probability computed from logits that may differ by `tol`
            slack = np.expm1(2 * self.tol / temperature)
            decisions = {}
            for i, u in enumerate(gpu_path):
                nxt = gpu_path[i + 1] if i + 1 < len(gpu_path) else -1
                decisions[u] = dict(accept=kids[u].index(nxt) if nxt >= 0 else -1, bonus=gpu_bonus)
            path2, bonus2, rec2 = O.accept_sampled(tokens, o_logits, parent, temperature, uni, decisions=decisions)
            assert path2 == gpu_path and bonus2 == gpu_bonus
            for u in gpu_path:                      # every forced decision must be a near-threshold one
                r = rec2[u]
                for i, a in enumerate(r["ratios"]):
                    took = r["accept"] == i
                    natural = uni[u, i] < a
                    if took != natural:
                        assert abs(uni[u, i] - a) <= slack * a + 1e-7, \
                            f"seq {b} node {u} child {i}: uniform {uni[u, i]:.6f} vs ratio {a:.6f}"
                        self.tie_events += 1
                    if took:
                        break
                if "cdf" in r:
                    cdf, target, t = r["cdf"], r["target"], gpu_bonus
                    lo = cdf[t - 1] if t > 0 else 0.0
                    d = slack * cdf[-1] + 1e-7
                    assert cdf[t] > lo, f"seq {b} node {u}: the GPU drew token {t}, which has no probability left"
                    if not (lo <= target < cdf[t]):
                        assert lo - d <= target <= cdf[t] + d, f"seq {b} node {u}: drawn token {t} outside its step"
                        self.tie_events += 1
            path, bonus = path2, bonus2
        return O.accept_and_compact(self.ocfg, self.seqs[b], tokens, o_logits, o_hidden, parent, sampled=(path, bonus))

    def prefill(self, prompts: List[np.ndarray], chunk: int) -> None:
        g = self.gpu
        g.prefill(prompts, self.parent, self.rank, chunk, dynamic=self.dyn)
        self._check_prefill(prompts, chunk)

    def prefill_prompts(self, prompts: List[np.ndarray], oracle_chunk: int = 64) -> None:
        """The library's own prefill call (many-row passes, causal attention, LM head on the last row only) against
        the oracle's chunked chain prefill: the state after a prompt does not depend on how it was chunked."""
        g = self.gpu
        g.prefill_prompts(prompts, self.parent, self.rank, dynamic=self.dyn)
        self._check_prefill(prompts, oracle_chunk, last_row=True)

    def _check_prefill(self, prompts: List[np.ndarray], chunk: int, last_row: bool = False) -> None:
        g = self.gpu
        g.torch.cuda.synchronize()
        toks = g.tree_tokens.cpu().numpy()
        lens = g.seq_len()
        for b, p in enumerate(prompts):
            # oracle prefill in chunks (a chain is plain decoding whatever the chunking)
            seq = self.seqs[b]
            n_chunks_b = (len(p) + chunk - 1) // chunk
            acc = None
            for ci in range(n_chunks_b):
                part = [int(t) for t in p[ci * chunk:(ci + 1) * chunk]]
                chain = list(range(-1, len(part) - 1))
                hidden, logits = O.verify_tree(self.W, self.ocfg, seq, part, chain)
                nxt = int(p[(ci + 1) * chunk]) if (ci + 1) * chunk < len(p) else -1
                if nxt < 0:
                    # the bonus token is an argmax: follow the GPU inside the tie zone
                    gpu_bonus = int(toks[b, 0])
                    best = int(O.ranked_ids(logits[len(part) - 1], 1)[0])
                    if gpu_bonus != best:
                        gap = float(logits[len(part) - 1][best] - logits[len(part) - 1][gpu_bonus])
                        assert gap <= self.tol, f"prefill bonus token: gpu {gpu_bonus} oracle {best} gap {gap:.3e}"
                        self.tie_events += 1
                    nxt_eff = gpu_bonus
                    if last_row:
                        # the prefill call hands back the last row's logits and hidden state: element by element
                        got = g.logits[b, 0].cpu().numpy()
                        err = float(np.abs(got - logits[len(part) - 1]).max())
                        self.max_logit_err = max(self.max_logit_err, err)
                        assert err <= self.tol, f"seq {b}: last-row logits max-abs error {err:.3e}"
                        herr = float(np.abs(g.hid_acc[b, 0].cpu().numpy() - hidden[len(part) - 1]).max())
                        self.max_hidden_err = max(self.max_hidden_err, herr)
                        assert herr <= self.hidden_atol, f"seq {b}: last-row hidden state max-abs error {herr:.3e}"
                        assert int(g.next_tok[b, 0]) == gpu_bonus
                else:
                    nxt_eff = nxt
                acc = O.accept_forced(seq, part, logits, hidden, len(part), nxt_eff)
                if ci < n_chunks_b - 1:
                    O.draft_tree(self.W, self.ocfg, seq, acc["hid_acc"], acc["next_tok"], [-1], [0])
            self.acc[b] = acc
            assert lens[b] == seq.L == len(p), (lens[b], seq.L, len(p))
            self._check_draft(b, toks[b, :self.n_nodes], self.parent, self.rank)
            assert seq.aug_L == seq.L
            self.compare_kv(b, 0, seq.L)

    def seed_cache(self, lengths: List[int], seed: int) -> None:
        """Instead of a prefill: the state right after a prompt of lengths[b] tokens, with seeded random cache rows
        (N(0, 0.6) keys and values, each a sum of two bf16 numbers so that both sides hold identical values): L rows
        in the target cache, L - 1 in the augmenting block's, and one seeded (hidden state, next token) hand-off
        row per sequence, on which the draft head then runs on both sides."""
        g, torch = self.gpu, self.gpu.torch
        nkv, d = self.shape.n_kv_heads, self.shape.head_dim

        def two_bf16(a: np.ndarray) -> np.ndarray:
            hi = synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(a))
            lo = synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(a - hi))
            return hi + lo

        hid = np.zeros((self.B, self.R, self.shape.hidden), np.float32)
        nxt = np.zeros((self.B, self.R), np.int32)
        for b, L in enumerate(lengths):
            rng = np.random.default_rng([seed, b])
            seq = self.seqs[b]
            for stack, n_layers, kv in ((0, self.shape.n_layers, seq.kv), (1, self.shape.aug_layers, seq.aug_kv)):
                rows = L - stack
                for l in range(n_layers):
                    k = two_bf16((rng.standard_normal((rows, nkv, d), dtype=np.float32) * 0.6).astype(np.float32))
                    v = two_bf16((rng.standard_normal((rows, nkv, d), dtype=np.float32) * 0.6).astype(np.float32))
                    kv.k[l, :rows] = k
                    kv.v[l, :rows] = v
                    g.write_kv(stack, l, b, 0, k, v)
            seq.L, seq.aug_L = L, L - 1
            hid[b, 0] = rng.standard_normal(self.shape.hidden, dtype=np.float32)
            nxt[b, 0] = int(rng.integers(0, self.shape.vocab))
            self.acc[b] = dict(m=1, path=[0], new_tokens=[int(nxt[b, 0])], hid_acc=hid[b, :1].astype(np.float64),
                               next_tok=[int(nxt[b, 0])])
        full = list(lengths) + [0] * (self.B - len(lengths))
        g.set_seq_len(full, [max(v - 1, 0) for v in full])
        g.hid_acc.copy_(torch.from_numpy(hid))
        g.next_tok.copy_(torch.from_numpy(nxt))
        g.m.copy_(torch.from_numpy(np.ones(self.B, np.int32)))
        g.draft_tree(len(lengths))
        torch.cuda.synchronize()
        toks = g.tree_tokens.cpu().numpy()
        lens = g.seq_len()
        for b, L in enumerate(lengths):
            assert lens[b] == L
            self._check_draft(b, toks[b, :self.n_nodes], self.parent, self.rank)
            assert self.seqs[b].aug_L == L
            self.compare_kv(b, L - 1, L, stacks=(1,))

    def compare_kv(self, b: int, slot0: int, slot1: int, atol: Optional[float] = None, stacks=(0, 1)) -> None:
        """Target and augmenting-block cache rows [slot0, slot1) against the oracle's."""
        atol = atol if atol is not None else self.kv_atol
        if slot1 <= slot0:
            return
        seq = self.seqs[b]
        for stack, n_layers, kv in ((0, self.shape.n_layers, seq.kv), (1, self.shape.aug_layers, seq.aug_kv)):
            if stack not in stacks:
                continue
            for l in range(n_layers):
                k, v = self.gpu.read_kv(stack, l, b, slot0, slot1 - slot0)
                ek = np.abs(k - kv.k[l, slot0:slot1]).max()
                ev = np.abs(v - kv.v[l, slot0:slot1]).max()
                self.max_kv_err = max(self.max_kv_err, float(ek), float(ev))
                assert ek <= atol and ev <= atol, f"KV stack {stack} layer {l} seq {b}: |dK| {ek:.3e} |dV| {ev:.3e}"

    def step(self, tree_hook: Optional[Callable[[int, np.ndarray], np.ndarray]] = None,
             check_compaction_bits: bool = True, sampled: Optional[tuple] = None) -> List[int]:
        """One speculative step on both sides; returns the accepted lengths.  sampled = (temperature, seed) verifies
        at that temperature with seeded uniforms handed to both sides."""
        g, B = self.gpu, self.B
        N = self.dyn[0] if self.dyn is not None else len(self.parent)
        torch = g.torch
        if tree_hook is not None:
            t = g.tree_tokens.cpu().numpy()
            for b in range(B):
                t[b, :N] = tree_hook(b, t[b, :N].copy())
            g.tree_tokens.copy_(torch.from_numpy(t))
        tokens = g.tree_tokens.cpu().numpy()
        L_before = g.seq_len()
        g.verify_tree(B)
        torch.cuda.synchronize()
        logits = g.logits.cpu().numpy()
        hidden = g.hidden.cpu().numpy()
        pre_kv = [[g.read_kv(0, l, b, int(L_before[b]), N) for l in range(self.shape.n_layers)] for b in range(B)]
        uni = None
        if sampled is not None:
            uni = np.random.default_rng([int(sampled[1]), 17]).random((B, g.R, 17), dtype=np.float32)
            g.accept_and_compact_sampled(B, float(sampled[0]), torch.from_numpy(uni).to(g.dev))
        else:
            g.accept_and_compact(B)
        torch.cuda.synchronize()
        m = g.m.cpu().numpy(); acc_idx = g.acc_idx.cpu().numpy(); new_tokens = g.new_tokens.cpu().numpy()
        next_tok = g.next_tok.cpu().numpy(); hid_acc = g.hid_acc.cpu().numpy()
        L_after = g.seq_len()
        ms = []
        for b in range(B):
            seq = self.seqs[b]
            assert seq.L == L_before[b]
            o_hidden, o_logits = O.verify_tree(self.W, self.ocfg, seq, tokens[b, :N], self.parents[b])
            le = float(np.abs(logits[b, :N] - o_logits).max())
            he = float(np.abs(hidden[b, :N] - o_hidden).max())
            self.max_logit_err = max(self.max_logit_err, le)
            self.max_hidden_err = max(self.max_hidden_err, he)
            assert le <= self.tol, f"seq {b}: logits max-abs error {le:.3e} > {self.tol}"
            assert he <= self.hidden_atol, f"seq {b}: hidden-state max-abs error {he:.3e} > {self.hidden_atol}"
            # uncompacted tree rows of the cache (read back before the GPU compacted them)
            atol = self.kv_atol
            for l in range(self.shape.n_layers):
                ek = np.abs(pre_kv[b][l][0] - seq.kv.k[l, seq.L:seq.L + N]).max()
                ev = np.abs(pre_kv[b][l][1] - seq.kv.v[l, seq.L:seq.L + N]).max()
                self.max_kv_err = max(self.max_kv_err, float(ek), float(ev))
                assert ek <= atol and ev <= atol, f"tree KV rows layer {l} seq {b}: |dK| {ek:.3e} |dV| {ev:.3e}"
            # acceptance: the GPU's implied argmax at each visited node must be (near-)optimal for the oracle
            mb = int(m[b])
            path = [int(a) for a in acc_idx[b, :mb]]
            assert mb >= 1 and path[0] == 0
            if sampled is not None:
                acc = self._follow_sampled(b, tokens[b, :N], o_logits, o_hidden, path, int(new_tokens[b, mb - 1]),
                                           float(sampled[0]), uni[b].astype(np.float64))
                assert acc["new_tokens"] == [int(t) for t in new_tokens[b, :mb]]
                assert acc["next_tok"] == [int(t) for t in next_tok[b, :mb]]
                assert L_after[b] == seq.L
                np.testing.assert_array_equal(hid_acc[b, :mb], hidden[b, path])
                if check_compaction_bits:
                    for l in range(self.shape.n_layers):
                        k2, v2 = g.read_kv(0, l, b, int(L_before[b]), mb)
                        np.testing.assert_array_equal(k2, pre_kv[b][l][0][path])
                        np.testing.assert_array_equal(v2, pre_kv[b][l][1][path])
                self.acc[b] = acc
                ms.append(mb)
                continue
            implied = {}
            for i, u in enumerate(path):
                implied[u] = int(tokens[b, path[i + 1]]) if i + 1 < mb else int(new_tokens[b, mb - 1])
            override = {}
            for u, t in implied.items():
                best = int(O.ranked_ids(o_logits[u], 1)[0])
                if t != best:
                    gap = float(o_logits[u][best] - o_logits[u][t])
                    assert gap <= self.tol, f"seq {b} node {u}: gpu argmax {t} vs oracle {best}, gap {gap:.3e}"
                    override[u] = t
                    self.tie_events += 1
            acc = O.accept_and_compact(self.ocfg, seq, tokens[b, :N], o_logits, o_hidden, self.parents[b], override)
            assert acc["path"] == path, f"seq {b}: accepted path gpu {path} oracle {acc['path']}"
            assert acc["new_tokens"] == [int(t) for t in new_tokens[b, :mb]]
            assert acc["next_tok"] == [int(t) for t in next_tok[b, :mb]]
            assert L_after[b] == seq.L
            he2 = float(np.abs(hid_acc[b, :mb] - acc["hid_acc"]).max())
            assert he2 <= max(he, 1e-12) + 1e-12
            np.testing.assert_array_equal(hid_acc[b, :mb], hidden[b, path])       # the gather itself is exact
            if check_compaction_bits:
                for l in range(self.shape.n_layers):
                    k2, v2 = g.read_kv(0, l, b, int(L_before[b]), mb)
                    np.testing.assert_array_equal(k2, pre_kv[b][l][0][path])      # compaction moves bits
                    np.testing.assert_array_equal(v2, pre_kv[b][l][1][path])
            self.acc[b] = acc
            ms.append(mb)
        g.draft_tree(B)
        torch.cuda.synchronize()
        toks = g.tree_tokens.cpu().numpy()
        for b in range(B):
            self._check_draft(b, toks[b, :N], self.parent, self.rank)
            assert self.seqs[b].aug_L == self.seqs[b].L
            self.compare_kv(b, self.seqs[b].L - ms[b], self.seqs[b].L)
        return ms


def truth_hook_factory(ls: Lockstep, want: List[int]):
    """tree_hook that plants the target's true greedy continuation (computed by the oracle from
    its current state, token by token) down one root path for want[step]-1 levels and wrong
    tokens elsewhere (random-init drafts almost never match on their own)."""
    state = {"step": 0}

    def shape_of(b: int):
        parent = ls.parents[b]
        n = len(parent)
        height = np.zeros(n, dtype=np.int64)
        for u in range(n - 1, 0, -1):
            height[parent[u]] = max(height[parent[u]], height[u] + 1)
        return O.children_of(parent), n, height

    def continuation(seq, root: int, k: int) -> List[int]:
        c = O.SeqState(ls.ocfg)
        c.kv = seq.kv.copy()
        c.L = seq.L
        out, t = [], int(root)
        for _ in range(k):
            _, lg = O.verify_tree(ls.W, ls.ocfg, c, [t], [-1])
            c.L += 1
            t = int(O.ranked_ids(lg[0], 1)[0])
            out.append(t)
        return out

    def hook(b: int, tokens: np.ndarray) -> np.ndarray:
        kids, n, height = shape_of(b)
        w = want[state["step"]]
        truth = continuation(ls.seqs[b], int(tokens[0]), max(w, 1))
        rng = np.random.default_rng(1000 * state["step"] + b)
        tokens[1:] = (truth[0] + 1 + rng.integers(1, 50, n - 1)) % ls.shape.vocab
        u = 0
        for lvl in range(w - 1):
            if not kids[u]:
                break
            c = max(kids[u], key=lambda c_: (height[c_], c_))
            tokens[c] = truth[lvl]
            for s_ in kids[u]:                      # siblings stay distinct from the planted token
                if s_ != c and tokens[s_] == tokens[c]:
                    tokens[s_] = (tokens[s_] + 1) % ls.shape.vocab
            u = c
        if b == ls.B - 1:
            state["step"] += 1
        return tokens

    return hook
