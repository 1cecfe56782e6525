"""Thin ctypes binding of libclover.so (include/clover.h).

Argument marshalling only: every step of the speculative step runs in the HIP
kernels behind the C ABI.  PyTorch is used for device memory and the stream.
There is no CPU fallback: loading fails loudly if the library is missing.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libclover.so")

OK, E_NULL, E_CONFIG, E_TREE, E_CAPACITY, E_SHAPE, E_HIP, E_STATE = 0, -1, -2, -3, -4, -5, -6, -7
DTYPE_F32, DTYPE_BF16 = 0, 1
FLAG_GENERIC = 1
FLAG_INTERVAL_MASK = 2      # linear-size tree mask (two integers per node); lifts max_nodes to 256
STATIC_SCRATCH_BYTES = 32 << 20

EXPORTS = [
    "clover_workspace_bytes", "clover_init", "clover_destroy", "clover_reset", "clover_set_tree",
    "draft_tree", "verify_tree", "accept_and_compact", "accept_and_compact_sampled", "clover_accept_forced", "clover_prefill", "clover_set_page_table", "clover_seq_len",
    "clover_read_kv", "clover_write_kv", "clover_set_seq_len", "clover_capture_draft_logits", "clover_set_dynamic_tree", "clover_read_dynamic_tree", "clover_path_info", "clover_profile_enable", "clover_profile_collect", "clover_kernel_class_count",
    "clover_kernel_class_name", "clover_last_error", "clover_last_global_error",
    "clover_op_gemm_scratch_bytes", "clover_op_gemm", "clover_op_gemm_static",
]


class Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "ffn", "vocab")] + \
               [("rope_base", C.c_float), ("rms_eps", C.c_float)] + \
               [(n, C.c_int32) for n in ("dtype", "aug_layers", "ad_heads", "draft_depths", "max_batch", "max_seq",
                                         "max_nodes", "flags", "prefill_rows")]


class Tree(C.Structure):
    _fields_ = [("n_nodes", C.c_int32), ("parent", C.POINTER(C.c_int32)), ("rank", C.POINTER(C.c_int32))]


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")]


class ADWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("norm", "wq", "bq", "wk", "bk", "wv", "bv")]


class Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("layers", C.POINTER(LayerWeights)), ("final_norm", C.c_void_p),
                ("lm_head", C.c_void_p), ("ad1", ADWeights), ("ad2", ADWeights), ("aug", C.POINTER(LayerWeights)),
                ("fc0_w", C.c_void_p), ("fc0_b", C.c_void_p), ("fc_w", C.POINTER(C.c_void_p)),
                ("fc_b", C.POINTER(C.c_void_p)), ("head_norm", C.c_void_p)]


_lib = None


def load_library(path: Optional[str] = None) -> C.CDLL:
    """dlopen libclover.so and declare the prototypes.  Raises if it is not built."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or LIB_PATH
    if not os.path.exists(p):
        raise RuntimeError(f"{p} is missing: build it with `python -m paper_2408_00264_amd.build` "
                           "(there is no CPU fallback)")
    lib = C.CDLL(p)
    vp, i32, i32p, f32p = C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p
    lib.clover_workspace_bytes.argtypes = [C.POINTER(Config), C.POINTER(C.c_size_t)]
    lib.clover_init.argtypes = [C.POINTER(Config), C.POINTER(Weights), C.POINTER(Tree), vp, C.c_size_t, vp,
                                C.POINTER(vp)]
    lib.clover_destroy.argtypes = [vp]
    lib.clover_reset.argtypes = [vp]
    lib.clover_set_tree.argtypes = [vp, C.POINTER(Tree)]
    lib.draft_tree.argtypes = [vp, i32, f32p, i32p, i32p, i32p]
    lib.verify_tree.argtypes = [vp, i32, i32p, f32p, f32p]
    lib.accept_and_compact.argtypes = [vp, i32, i32p, f32p, f32p, i32p, i32p, i32p, f32p, i32p]
    lib.accept_and_compact_sampled.argtypes = [vp, i32, i32p, f32p, f32p, C.c_float, f32p, i32p, i32p, i32p, f32p, i32p]
    lib.clover_accept_forced.argtypes = [vp, i32, i32p, f32p, f32p, i32p, i32p, i32p, i32p, i32p, f32p, i32p]
    lib.clover_seq_len.argtypes = [vp, C.POINTER(C.c_int32)]
    lib.clover_read_kv.argtypes = [vp, i32, i32, i32, i32, i32, vp, vp]
    lib.clover_write_kv.argtypes = [vp, i32, i32, i32, i32, i32, vp, vp]
    lib.clover_set_seq_len.argtypes = [vp, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
    lib.clover_capture_draft_logits.argtypes = [vp, vp, C.c_size_t]
    lib.clover_set_dynamic_tree.argtypes = [vp, i32, i32, i32]
    lib.clover_read_dynamic_tree.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp, vp]
    lib.clover_path_info.argtypes = [vp]
    lib.clover_profile_enable.argtypes = [vp, i32]
    lib.clover_profile_collect.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_int64), i32]
    lib.clover_kernel_class_count.argtypes = []
    lib.clover_kernel_class_name.argtypes = [i32]
    lib.clover_kernel_class_name.restype = C.c_char_p
    lib.clover_last_error.argtypes = [vp]
    lib.clover_last_error.restype = C.c_char_p
    lib.clover_last_global_error.argtypes = []
    lib.clover_last_global_error.restype = C.c_char_p
    lib.clover_op_gemm_scratch_bytes.argtypes = [i32, i32, i32]
    lib.clover_op_gemm_scratch_bytes.restype = C.c_size_t
    lib.clover_op_gemm.argtypes = [i32, i32, vp, vp, vp, i32, i32, i32, i32, vp, C.c_size_t, vp]
    lib.clover_op_gemm_static.argtypes = [i32, i32, vp, vp, vp, i32, i32, i32, i32, vp]
    for n in EXPORTS:
        getattr(lib, n)  # every declared symbol must be exported
    if _lib is None:
        _lib = lib          # the first library loaded serves the whole process
    return lib


class CloverError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"clover error {code}: {msg}")
        self.code = code


def make_config(shape, max_batch: int, max_seq: int, max_nodes: int, flags: int = 0, prefill_rows: int = 0) -> Config:
    """Config from a synth.ModelShape-like object."""
    return Config(shape.n_layers, shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.ffn,
                  shape.vocab, float(shape.rope_base), float(shape.rms_eps),
                  DTYPE_BF16 if shape.bf16 else DTYPE_F32, shape.aug_layers, shape.ad_heads or shape.n_q_heads,
                  shape.draft_depths, max_batch, max_seq, max_nodes, flags, prefill_rows)


def _tree_struct(parent: Sequence[int], rank: Sequence[int]):
    p = np.ascontiguousarray(parent, dtype=np.int32)
    r = np.ascontiguousarray(rank, dtype=np.int32)
    t = Tree(len(p), p.ctypes.data_as(C.POINTER(C.c_int32)), r.ctypes.data_as(C.POINTER(C.c_int32)))
    return t, (p, r)


class Clover:
    """One library context plus the torch-owned device buffers of a speculative loop."""

    def __init__(self, shape, weights: Dict[str, "object"], parent, rank, max_batch: int, max_seq: int,
                 max_nodes: int, flags: int = 0, device: str = "cuda:0", prefill_rows: int = 0):
        import torch
        self.torch = torch
        self.lib = load_library()
        self.shape = shape
        self.dev = torch.device(device)
        self.cfg = make_config(shape, max_batch, max_seq, max_nodes, flags, prefill_rows)
        self.B, self.R, self.H, self.V = max_batch, max_nodes, shape.hidden, shape.vocab
        self._w = weights                       # name -> device tensor (kept alive: the library borrows them)
        ptr = lambda n: C.c_void_p(weights[n].data_ptr())

        def layer(prefix: str) -> LayerWeights:
            return LayerWeights(*[weights[prefix + n].data_ptr() for n in
                                  ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")])

        def ad(prefix: str) -> ADWeights:
            return ADWeights(*[weights[prefix + n].data_ptr() for n in ("norm", "wq", "bq", "wk", "bk", "wv", "bv")])

        self._layers = (LayerWeights * shape.n_layers)(*[layer(f"layers.{i}.") for i in range(shape.n_layers)])
        self._aug = (LayerWeights * shape.aug_layers)(*[layer(f"aug.{i}.") for i in range(shape.aug_layers)])
        D = shape.draft_depths
        self._fcw = (C.c_void_p * D)(*[None if j == 0 else weights[f"fc.{j}.w"].data_ptr() for j in range(D)])
        self._fcb = (C.c_void_p * D)(*[None if j == 0 else weights[f"fc.{j}.b"].data_ptr() for j in range(D)])
        self._wstruct = Weights(ptr("embed"), self._layers, ptr("final_norm"), ptr("lm_head"), ad("ad1."), ad("ad2."),
                                self._aug, ptr("fc0.w"), ptr("fc0.b"), self._fcw, self._fcb, ptr("head_norm"))
        nbytes = C.c_size_t(0)
        rc = self.lib.clover_workspace_bytes(C.byref(self.cfg), C.byref(nbytes))
        if rc != OK:
            raise CloverError(rc, self.lib.clover_last_global_error().decode())
        self.workspace_bytes = nbytes.value
        self.workspace = torch.empty(nbytes.value + 256, dtype=torch.uint8, device=self.dev)
        base = (self.workspace.data_ptr() + 255) & ~255
        self.stream = torch.cuda.current_stream(self.dev)
        t, keep = _tree_struct(parent, rank)
        ctx = C.c_void_p()
        rc = self.lib.clover_init(C.byref(self.cfg), C.byref(self._wstruct), C.byref(t), C.c_void_p(base),
                                  nbytes.value, C.c_void_p(self.stream.cuda_stream), C.byref(ctx))
        if rc != OK:
            raise CloverError(rc, self.lib.clover_last_global_error().decode())
        self.ctx = ctx
        self.n_nodes = len(parent)
        B, R, H, V = self.B, self.R, self.H, self.V
        i32 = dict(dtype=torch.int32, device=self.dev)
        f32 = dict(dtype=torch.float32, device=self.dev)
        self.tree_tokens = torch.zeros(B, R, **i32)
        self.logits = torch.zeros(B, R, V, **f32)
        self.hidden = torch.zeros(B, R, H, **f32)
        self.m = torch.zeros(B, **i32)
        self.acc_idx = torch.zeros(B, R, **i32)
        self.new_tokens = torch.zeros(B, R, **i32)
        self.hid_acc = torch.zeros(B, R, H, **f32)
        self.next_tok = torch.zeros(B, R, **i32)
        self.n_forced = torch.zeros(B, **i32)
        self.forced_next = torch.zeros(B, **i32)

    # -- plumbing ------------------------------------------------------------------------------
    def _check(self, rc: int) -> None:
        if rc != OK:
            raise CloverError(rc, self.lib.clover_last_error(self.ctx).decode())

    def close(self) -> None:
        if getattr(self, "ctx", None):
            self.lib.clover_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @staticmethod
    def _p(t) -> C.c_void_p:
        return C.c_void_p(t.data_ptr())

    # -- the C calls ---------------------------------------------------------------------------
    def reset(self) -> None:
        self._check(self.lib.clover_reset(self.ctx))

    def set_tree(self, parent, rank) -> None:
        t, keep = _tree_struct(parent, rank)
        self._check(self.lib.clover_set_tree(self.ctx, C.byref(t)))
        self.n_nodes = len(parent)

    def draft_tree(self, batch: int) -> None:
        self._check(self.lib.draft_tree(self.ctx, batch, self._p(self.hid_acc), self._p(self.next_tok), self._p(self.m),
                                        self._p(self.tree_tokens)))

    def verify_tree(self, batch: int) -> None:
        self._check(self.lib.verify_tree(self.ctx, batch, self._p(self.tree_tokens), self._p(self.logits),
                                         self._p(self.hidden)))

    def accept_and_compact(self, batch: int) -> None:
        self._check(self.lib.accept_and_compact(self.ctx, batch, self._p(self.tree_tokens), self._p(self.logits),
                                                self._p(self.hidden), self._p(self.m), self._p(self.acc_idx),
                                                self._p(self.new_tokens), self._p(self.hid_acc), self._p(self.next_tok)))

    def accept_and_compact_sampled(self, batch: int, temperature: float, uniforms) -> None:
        """uniforms: device fp32 tensor [batch, max_nodes, 17] of the caller's random numbers in [0, 1)."""
        assert tuple(uniforms.shape) == (self.B, self.R, 17) and uniforms.dtype == self.torch.float32
        self._check(self.lib.accept_and_compact_sampled(self.ctx, batch, self._p(self.tree_tokens), self._p(self.logits),
                                                        self._p(self.hidden), C.c_float(temperature), self._p(uniforms),
                                                        self._p(self.m), self._p(self.acc_idx), self._p(self.new_tokens),
                                                        self._p(self.hid_acc), self._p(self.next_tok)))

    def accept_forced(self, batch: int) -> None:
        self._check(self.lib.clover_accept_forced(self.ctx, batch, self._p(self.tree_tokens), self._p(self.logits),
                                                  self._p(self.hidden), self._p(self.n_forced),
                                                  self._p(self.forced_next), self._p(self.m), self._p(self.acc_idx),
                                                  self._p(self.new_tokens), self._p(self.hid_acc),
                                                  self._p(self.next_tok)))

    def seq_len(self) -> np.ndarray:
        out = (C.c_int32 * self.B)()
        self._check(self.lib.clover_seq_len(self.ctx, out))
        return np.frombuffer(out, dtype=np.int32).copy()

    def read_kv(self, stack: int, layer: int, b: int, slot0: int, n_slots: int):
        nkv, d = self.shape.n_kv_heads, self.shape.head_dim
        k = np.empty((n_slots, nkv, d), dtype=np.float32)
        v = np.empty((n_slots, nkv, d), dtype=np.float32)
        per_call = max(1, (self.B * self.R * self.V // 2) // (nkv * d))   # staging area of the library
        for s0 in range(0, n_slots, per_call):
            n = min(per_call, n_slots - s0)
            self._check(self.lib.clover_read_kv(self.ctx, stack, layer, b, slot0 + s0, n,
                                                k[s0:].ctypes.data, v[s0:].ctypes.data))
        return k, v

    def write_kv(self, stack: int, layer: int, b: int, slot0: int, k: np.ndarray, v: np.ndarray) -> None:
        k = np.ascontiguousarray(k, dtype=np.float32)
        v = np.ascontiguousarray(v, dtype=np.float32)
        nkv, d = self.shape.n_kv_heads, self.shape.head_dim
        n_slots = k.shape[0]
        per_call = max(1, (self.B * self.R * self.V // 2) // (nkv * d))   # staging area of the library
        for s0 in range(0, n_slots, per_call):
            n = min(per_call, n_slots - s0)
            self._check(self.lib.clover_write_kv(self.ctx, stack, layer, b, slot0 + s0, n,
                                                 k[s0:].ctypes.data, v[s0:].ctypes.data))

    def set_seq_len(self, lens, aug_lens) -> None:
        a = (C.c_int32 * self.B)(*[int(v) for v in lens])
        b = (C.c_int32 * self.B)(*[int(v) for v in aug_lens])
        self._check(self.lib.clover_set_seq_len(self.ctx, a, b))

    def capture_draft_logits(self, on: bool = True):
        """Device buffer [batch * internal nodes, V] that every later draft_tree fills (None: off)."""
        if not on:
            self._check(self.lib.clover_capture_draft_logits(self.ctx, None, 0))
            self.draft_logits = None
            return None
        self.draft_logits = self.torch.zeros(self.B * self.R, self.V, dtype=self.torch.float32, device=self.dev)
        self._check(self.lib.clover_capture_draft_logits(self.ctx, self._p(self.draft_logits), self.draft_logits.numel()))
        return self.draft_logits

    def set_dynamic_tree(self, n_nodes: int, topk: int, frontier: int) -> None:
        self._check(self.lib.clover_set_dynamic_tree(self.ctx, n_nodes, topk, frontier))
        self.n_nodes = n_nodes
        self.dyn = (n_nodes, topk, frontier)

    def read_dynamic_tree(self, b: int) -> dict:
        n = self.dyn[0]
        parent = np.zeros(n, np.int32); rank = np.zeros(n, np.int32); keep = np.zeros(n, np.int32)
        ctok = np.zeros(256, np.int32); cscore = np.zeros(256, np.float32); cpar = np.zeros(256, np.int32)
        front = np.zeros(8 * 64, np.int32)
        self._check(self.lib.clover_read_dynamic_tree(self.ctx, b, parent.ctypes.data, rank.ctypes.data, keep.ctypes.data,
                                                      ctok.ctypes.data, cscore.ctypes.data, cpar.ctypes.data,
                                                      front.ctypes.data))
        return dict(parent=parent, rank=rank, keep=keep, cand_token=ctok, cand_score=cscore, cand_parent=cpar,
                    frontier=front.reshape(8, 64))

    def path_info(self) -> int:
        """Bit 0: MFMA path, bit 1: MFMA tree attention."""
        v = self.lib.clover_path_info(self.ctx)
        if v < 0:
            self._check(v)
        return v

    def profile_enable(self, on: bool) -> None:
        self._check(self.lib.clover_profile_enable(self.ctx, 1 if on else 0))

    def profile_collect(self) -> Dict[str, tuple]:
        n = self.lib.clover_kernel_class_count()
        ms = (C.c_double * n)()
        cnt = (C.c_int64 * n)()
        self._check(self.lib.clover_profile_collect(self.ctx, ms, cnt, n))
        return {self.lib.clover_kernel_class_name(i).decode(): (ms[i], cnt[i]) for i in range(n)}

    # -- call sequences (no arithmetic here) -----------------------------------------------------
    def prefill(self, prompts: List[np.ndarray], parent, rank, chunk: Optional[int] = None,
                dynamic: Optional[tuple] = None) -> None:
        """Feed prompts as chain-shaped trees of at most `chunk` tokens per call; afterwards
        `tree_tokens` holds the first draft tree and m/hid_acc/next_tok the hand-off state.
        Ragged batches are right-aligned in chunk time: a shorter prompt starts in a later call
        (n_rows = 0 before that), so every sequence ends in the last call, where the real tree is
        installed before the draft head runs."""
        torch = self.torch
        B = len(prompts)
        chunk = min(chunk or self.R, self.R)
        chain_p = np.arange(-1, chunk - 1, dtype=np.int32)
        chain_r = np.zeros(chunk, dtype=np.int32)
        n_chunks_b = [(len(p) + chunk - 1) // chunk for p in prompts]
        n_chunks = max(n_chunks_b)
        self.set_tree(chain_p, chain_r)
        for ci in range(n_chunks):
            toks = np.zeros((self.B, self.R), dtype=np.int32)
            nf = np.zeros(self.B, dtype=np.int32)
            fx = np.full(self.B, -1, dtype=np.int32)
            for b, p in enumerate(prompts):
                local = ci - (n_chunks - n_chunks_b[b])
                if local < 0:
                    continue
                part = p[local * chunk:(local + 1) * chunk]
                toks[b, :len(part)] = part
                nf[b] = len(part)
                if (local + 1) * chunk < len(p):
                    fx[b] = p[(local + 1) * chunk]
            self.tree_tokens.copy_(torch.from_numpy(toks))
            self.n_forced.copy_(torch.from_numpy(nf))
            self.forced_next.copy_(torch.from_numpy(fx))
            self.verify_tree(B)
            self.accept_forced(B)
            if ci == n_chunks - 1:
                if dynamic is not None:
                    self.set_dynamic_tree(*dynamic)      # (n_nodes, topk, frontier): a new topology per draft call
                else:
                    self.set_tree(parent, rank)
            self.draft_tree(B)

    def set_page_table(self, table: Optional[np.ndarray]) -> None:
        """Page table of the KV caches: int32 [max_batch * max_seq / 32], a permutation; None = identity."""
        if table is None:
            self._check(self.lib.clover_set_page_table(self.ctx, None))
            return
        t = np.ascontiguousarray(table, dtype=np.int32)
        self._check(self.lib.clover_set_page_table(self.ctx, t.ctypes.data_as(C.POINTER(C.c_int32))))

    def prefill_prompt(self, b: int, tokens) -> None:
        """clover_prefill for sequence b: `tokens` is a device int32 tensor; the last row's logits, hidden state
        and argmax go to logits[b, 0], hid_acc[b, 0] and next_tok[b, 0]; m[b] is not touched."""
        self._check(self.lib.clover_prefill(self.ctx, C.c_int32(b), C.c_void_p(tokens.data_ptr()), C.c_int32(tokens.numel()),
                                            C.c_void_p(self.logits[b, 0].data_ptr()), C.c_void_p(self.hid_acc[b, 0].data_ptr()),
                                            C.c_void_p(self.next_tok[b, 0].data_ptr())))

    def prefill_prompts(self, prompts: List[np.ndarray], parent, rank, dynamic: Optional[tuple] = None) -> None:
        """Prefill every prompt with clover_prefill (greedy first token), then one draft_tree call: the same
        hand-off state as `prefill` leaves."""
        torch = self.torch
        B = len(prompts)
        for b, p in enumerate(prompts):
            self.prefill_prompt(b, torch.from_numpy(np.ascontiguousarray(p, dtype=np.int32)).to(self.dev))
        self.m.fill_(1)
        if dynamic is not None:
            self.set_dynamic_tree(*dynamic)
        else:
            self.set_tree(parent, rank)
        self.draft_tree(B)

    def step(self, batch: int) -> None:
        self.verify_tree(batch)
        self.accept_and_compact(batch)
        self.draft_tree(batch)


def upload_weights(store, device: str = "cuda:0", names: Optional[Sequence[str]] = None,
                   keep_host: Optional[Sequence[str]] = None, threads: int = 0, group: int = 24):
    """Copy a synth.WeightStore to the GPU: bf16 tensors for bf16 models, fp32 otherwise.
    Tensors are generated `group` at a time on `threads` host threads and dropped from host
    memory after the copy unless listed in `keep_host` (None keeps all)."""
    import torch
    names = list(names or store.names())
    keep = None if keep_host is None else set(keep_host)
    threads = threads or min(16, os.cpu_count() or 1)
    out = {}
    for g0 in range(0, len(names), group):
        part = names[g0:g0 + group]
        store.prefetch(part, threads=threads)
        for n in part:
            a = store.get(n)
            if a.dtype == np.uint16:
                t = torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
            else:
                t = torch.from_numpy(a).to(device)
            out[n] = t.contiguous()
            if keep is not None and n not in keep:
                store.drop(n)
    return out
