"""GPU parity: the HIP path through the C ABI against the CPU oracle (run with -m gpu)."""
import ctypes as C

import numpy as np
import pytest

from paper_2408_00264_amd import clover, synth

pytestmark = pytest.mark.gpu

TINY = synth.CONFIGS[1]
# reduced bf16 shape with the structure of the LLaMA3-8B-shaped workload (GQA, head_dim 128)
MINI = synth.scaled(synth.CONFIGS[3], name="mini-bf16", n_layers=2, hidden=512, n_q_heads=4, n_kv_heads=2,
                    ffn=1536, vocab=8192, tree_k=(4, 3, 2, 2), tree_nodes=24, draft_depths=4, seed=11)


def _torch():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch


def say(*a):
    print(*a, flush=True)


# ------------------------------------------------------------------------------------------
# GEMM operator
# ------------------------------------------------------------------------------------------
GEMM_CASES = [
    # path, dtype, M, N, K
    (0, 0, 16, 1024, 256), (0, 0, 5, 77, 100), (0, 1, 64, 512, 512), (0, 1, 33, 130, 264),
    (1, 1, 64, 6144, 4096), (1, 1, 5, 4096, 8192), (1, 1, 16, 4096, 4096), (1, 1, 24, 1024, 512),
    (1, 1, 96, 4096, 14336), (1, 1, 256, 4096, 4096), (1, 1, 1, 32000, 4096), (1, 1, 130, 8192, 512),
    (1, 1, 64, 160, 256), (1, 1, 64, 28672, 4096), (1, 1, 48, 4096, 1536),
    # full-K panel kernel: odd block count, ragged rows, one row, LM-head width
    (3, 1, 64, 28672, 4096), (3, 1, 17, 1040, 768), (3, 1, 5, 4096, 512), (3, 1, 64, 160, 256), (3, 1, 1, 2064, 256),
    (3, 1, 33, 128256, 4096),
    # panel kernel over K ranges (the down projection's shape): full and ragged rows, one row
    (5, 1, 64, 4096, 14336), (5, 1, 37, 4096, 14336), (5, 1, 1, 4096, 14336), (5, 1, 16, 4096, 8192),
    # 65..128 rows in one weight pass (eight row blocks, 128-column stages): plain, odd rows, K ranges
    (3, 1, 128, 4096, 1024), (3, 1, 97, 28672, 4096), (5, 1, 96, 4096, 14336), (5, 1, 128, 6144, 4096),
    (5, 1, 65, 4096, 4096),
    # tiled kernel (one weight pass for up to 256 rows, 128 x 256 workgroup tiles): two row halves, a ragged second half,
    # one half only, odd widths, K ranges, one stage
    (7, 1, 256, 4096, 4096), (7, 1, 160, 6144, 4096), (7, 1, 129, 4096, 14336), (7, 1, 97, 1040, 512), (7, 1, 200, 8208, 1024),
    (7, 1, 256, 28672, 4096), (7, 1, 255, 512, 128), (7, 1, 256, 2064, 384), (7, 1, 33, 1040, 512), (7, 1, 97, 4096, 14336),
]


@pytest.mark.parametrize("path,dtype,M,N,K", GEMM_CASES)
def test_op_gemm(path, dtype, M, N, K):
    torch = _torch()
    say(f"gemm path={path} dtype={dtype} M={M} N={N} K={K}")
    lib = clover.load_library()
    rng = np.random.default_rng(M * 7 + N * 3 + K)
    X = rng.standard_normal((M, K)).astype(np.float32)
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    if dtype == 1:
        Wb = synth.f32_to_bf16_bits(W)
        Wf = synth.bf16_bits_to_f32(Wb).astype(np.float64)
        Wd = torch.from_numpy(Wb.view(np.int16)).cuda()
    else:
        Wf = W.astype(np.float64)
        Wd = torch.from_numpy(W).cuda()
    Xd = torch.from_numpy(X).cuda()
    ldy = N + 4
    Y = torch.full((M, ldy), -7.0, dtype=torch.float32, device="cuda")
    nb = lib.clover_op_gemm_scratch_bytes(M, N, K)
    scratch = torch.zeros(nb, dtype=torch.uint8, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    for rep in range(2):       # twice: the split-K counters must be back at zero
        rc = lib.clover_op_gemm(path, dtype, C.c_void_p(Xd.data_ptr()), C.c_void_p(Wd.data_ptr()),
                                C.c_void_p(Y.data_ptr()), ldy, M, N, K, C.c_void_p(scratch.data_ptr()), nb,
                                C.c_void_p(st))
        assert rc == 0, lib.clover_last_global_error()
        torch.cuda.synchronize()
        got = Y.cpu().numpy()
        assert np.all(got[:, N:] == -7.0)
        # generic path: fp32 FMA; MFMA path: activations split into two bf16 halves (16 mantissa bits)
        ref = X.astype(np.float64) @ Wf.T
        tol = (1e-5 if path == 0 else 4e-5) * np.sqrt(K) * 0.02 * 4
        err = np.abs(got[:, :N] - ref).max()
        assert err <= tol, (err, tol)


# ------------------------------------------------------------------------------------------
# whole calls, lock-step with the oracle
# ------------------------------------------------------------------------------------------
def _lockstep(shape, flags=0, gain_jitter=0.0, batch=1, max_seq=256, tree=None, max_nodes=None, dynamic=None,
              prefill_rows=0):
    from tests.parity import Lockstep
    parent, rank = tree if tree is not None else synth.tree_for(shape)
    return Lockstep(shape, parent, rank, max_seq, flags=flags, gain_jitter=gain_jitter, batch=batch,
                    max_nodes=max_nodes, dynamic=dynamic, prefill_rows=prefill_rows)


def test_config1_fp32_eight_steps():
    _torch()
    ls = _lockstep(TINY, max_seq=256)
    prompts = synth.make_prompts(TINY)
    say("config 1: prefill 64 tokens in chunks of 16")
    ls.prefill(prompts, chunk=16)
    for s in range(TINY.steps):
        ms = ls.step()
        say(f"  step {s}: m={ms} max|dlogit|={ls.max_logit_err:.2e} ties={ls.tie_events}")
    assert ls.max_logit_err <= 1e-4


def test_config1_gain_jitter_injected_accept_lengths():
    _torch()
    from tests.parity import truth_hook_factory
    ls = _lockstep(TINY, gain_jitter=0.1, max_seq=256)
    prompts = [synth.make_prompts(TINY, seed=5)[0][:37]]        # ragged last chunk
    ls.prefill(prompts, chunk=16)
    want = [4, 1, 3, 2, 4, 2]
    hook = truth_hook_factory(ls, want)
    got = []
    for s in range(len(want)):
        ties = ls.tie_events
        ms = ls.step(tree_hook=hook)
        say(f"  step {s}: want {want[s]} got {ms}")
        if ls.tie_events == ties:
            assert ms == [want[s]]
        got.append(ms[0])
    assert max(got) == 4 and min(got) == 1


@pytest.mark.parametrize("flags", [clover.FLAG_GENERIC, 0], ids=["generic", "mfma_kernels"])
def test_mini_bf16(flags):
    _torch()
    from tests.parity import truth_hook_factory
    ls = _lockstep(MINI, flags=flags, gain_jitter=0.1, max_seq=512)
    # the two variants must really run two different sets of kernels
    assert ls.gpu.path_info() == {clover.FLAG_GENERIC: 0, 0: 3}[flags]
    prompts = [synth.make_prompts(MINI, seed=3)[0][:150]]
    say(f"mini bf16 flags={flags}: prefill 150 tokens in chunks of 24")
    ls.prefill(prompts, chunk=24)
    want = [5, 1, 2, 4, 3]
    hook = truth_hook_factory(ls, want)
    for s in range(len(want)):
        ties = ls.tie_events
        ms = ls.step(tree_hook=hook)
        say(f"  step {s}: want {want[s]} got {ms} max|dlogit|={ls.max_logit_err:.2e} ties={ls.tie_events}")
        if ls.tie_events == ties:
            assert ms == [want[s]]
    for s in range(2):
        ms = ls.step()
        say(f"  free step {s}: m={ms} max|dlogit|={ls.max_logit_err:.2e}")
    assert ls.max_logit_err <= 3e-2


def test_mini_bf16_batch_ragged():
    _torch()
    shape = synth.scaled(MINI, batch=3, tree_nodes=12, tree_k=(3, 2, 2, 1), prompt_len=(20, 90), seed=13)
    ls = _lockstep(shape, batch=3, max_seq=256, max_nodes=16)
    prompts = synth.make_prompts(shape)
    say("ragged batch prompt lengths", [len(p) for p in prompts])
    ls.prefill(prompts, chunk=16)
    for s in range(3):
        ms = ls.step()
        say(f"  step {s}: m={ms} max|dlogit|={ls.max_logit_err:.2e} ties={ls.tie_events}")


def test_random_tree_and_chain_mask():
    """Tree attention against the oracle for a random topology (ancestor bit masks, tree-depth positions)."""
    _torch()
    from tests.parity import bfs_tree_random
    rng = np.random.default_rng(21)
    parent, rank = bfs_tree_random(rng, 16, 3)
    say("random tree parents", parent.tolist())
    ls = _lockstep(TINY, gain_jitter=0.1, tree=(parent, rank), max_seq=128, max_nodes=16)
    ls.prefill([synth.make_prompts(TINY, seed=8)[0][:21]], chunk=8)
    for s in range(2):
        ls.step()
    assert ls.max_logit_err <= 1e-4


def test_mha_shape_bf16():
    """Structure of the Vicuna-7B-shaped workload: one query head per KV head, RoPE base 1e4."""
    _torch()
    shape = synth.scaled(synth.CONFIGS[2], name="mini-mha", n_layers=2, hidden=512, n_q_heads=4, n_kv_heads=4,
                         ffn=1280, vocab=4096, tree_k=(4, 3, 2, 2), tree_nodes=24, seed=17)
    ls = _lockstep(shape, gain_jitter=0.1, max_seq=384)
    ls.prefill([synth.make_prompts(shape)[0][:131]], chunk=24)
    for s in range(3):
        ms = ls.step()
        say(f"  step {s}: m={ms} max|dlogit|={ls.max_logit_err:.2e} ties={ls.tie_events}")
    assert ls.max_logit_err <= 3e-2


@pytest.mark.parametrize("bf16", [False, True], ids=["fp32", "bf16"])
def test_single_node_tree_is_plain_decoding(bf16):
    """Degenerate tree: the root alone.  Every step verifies one row, accepts it and emits the target's next token,
    i.e. plain greedy decoding through the same three calls (the draft head still has to advance its own cache)."""
    _torch()
    shape = MINI if bf16 else TINY
    parent, rank = np.array([-1]), np.array([0])
    ls = _lockstep(shape, gain_jitter=0.1, tree=(parent, rank), max_seq=128, max_nodes=16)
    ls.prefill([synth.make_prompts(shape, seed=5)[0][:19]], chunk=8)
    for s in range(5):
        ms = ls.step()
        assert ms == [1]
    assert ls.max_logit_err <= (3e-2 if bf16 else 1e-4)
    assert ls.gpu.seq_len()[0] == 19 + 5


@pytest.mark.parametrize("bf16", [False, True], ids=["fp32", "bf16"])
def test_paper_size_head_two_aug_layers_five_depths(bf16):
    """The draft head at the paper's size (Sec. 3.3, 4.1): two augmenting layers, five depths (FC_1..FC_4)."""
    _torch()
    shape = synth.scaled(MINI if bf16 else TINY, name="paper-head", aug_layers=2, draft_depths=5,
                         tree_k=(3, 2, 2, 2, 1), tree_nodes=20, seed=23)
    ls = _lockstep(shape, gain_jitter=0.1, max_seq=256)
    ls.prefill([synth.make_prompts(shape)[0][:47]], chunk=20)
    for s in range(4):
        ms = ls.step()
        say(f"  step {s}: m={ms} max|dlogit|={ls.max_logit_err:.2e} ties={ls.tie_events}")
    assert ls.max_logit_err <= (3e-2 if bf16 else 1e-4)


def test_batch8_ragged_32_node_tree():
    """Structure of the batch-8 workload: 8 ragged sequences x 32-node tree = 256 rows per GEMM."""
    _torch()
    shape = synth.scaled(synth.CONFIGS[4], name="mini-b8", n_layers=2, hidden=512, n_q_heads=4, n_kv_heads=2,
                         ffn=1536, vocab=8192, prompt_len=(16, 200), seed=19)
    ls = _lockstep(shape, gain_jitter=0.1, batch=8, max_seq=384)
    prompts = synth.make_prompts(shape)
    say("batch 8 prompt lengths", [len(p) for p in prompts])
    ls.prefill(prompts, chunk=32)
    for s in range(3):
        ms = ls.step()
        say(f"  step {s}: m={ms} max|dlogit|={ls.max_logit_err:.2e} ties={ls.tie_events}")
    assert ls.max_logit_err <= 3e-2


def test_batch12_384_rows():
    """More than 8 sequences and more than 256 rows per pass (12 ragged sequences x 32-node tree = 384 rows): the GEMMs
    run as several row batches, attention and acceptance per sequence."""
    _torch()
    shape = synth.scaled(synth.CONFIGS[4], name="mini-b12", n_layers=2, hidden=512, n_q_heads=4, n_kv_heads=2,
                         ffn=1536, vocab=8192, batch=12, prompt_len=(10, 120), seed=43)
    ls = _lockstep(shape, gain_jitter=0.1, batch=12, max_seq=256)
    prompts = synth.make_prompts(shape)
    say("batch 12 prompt lengths", [len(p) for p in prompts])
    ls.prefill(prompts, chunk=32)
    for s in range(2):
        ms = ls.step()
        say(f"  step {s}: m={ms} max|dlogit|={ls.max_logit_err:.2e} ties={ls.tie_events}")
    assert ls.max_logit_err <= 3e-2


def test_long_context_96_node_tree():
    """Structure of the long-context workload: 96-node tree, draft depth 5, >1000 cached keys (many key
    tiles and several key splits per attention launch)."""
    _torch()
    from tests.parity import truth_hook_factory
    shape = synth.scaled(synth.CONFIGS[5], name="mini-long", n_layers=2, hidden=512, n_q_heads=4, n_kv_heads=2,
                         ffn=1536, vocab=8192, prompt_len=(1100, 1100), seed=23)
    ls = _lockstep(shape, gain_jitter=0.1, max_seq=1536)
    ls.prefill(synth.make_prompts(shape), chunk=96)
    want = [6, 2]
    hook = truth_hook_factory(ls, want)
    for s in range(len(want)):
        ties = ls.tie_events
        ms = ls.step(tree_hook=hook)
        say(f"  step {s}: want {want[s]} got {ms} max|dlogit|={ls.max_logit_err:.2e} ties={ls.tie_events}")
        if ls.tie_events == ties:
            assert ms == [want[s]]
    ms = ls.step()
    say(f"  free step: m={ms} max|dlogit|={ls.max_logit_err:.2e}")
    assert ls.max_logit_err <= 3e-2


# ------------------------------------------------------------------------------------------
# paged KV caches: any permutation of the pages gives the same results
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("case", ["fp32_generic", "bf16_mfma_batch3", "bf16_mfma_prefill_call"])
def test_paged_kv_shuffled_page_table(case):
    """The caches are pools of 32-position pages; with a random permutation as page table (pages of one sequence
    scattered between those of the others) every cache row read back, every logit and every accepted token must be
    what the oracle computes: writes (RoPE/KV kernel, cache-row upload), reads (both attention kernels, the read-back)
    and moves (compaction across a page boundary) all go through the table."""
    _torch()
    from tests.parity import truth_hook_factory
    bf16 = case.startswith("bf16")
    batch = 3 if "batch3" in case else (2 if "prefill_call" in case else 1)
    if bf16:
        shape = synth.scaled(MINI, batch=batch, prompt_len=(28, 95), seed=67)
    else:
        shape = TINY
    max_seq = 256
    ls = _lockstep(shape, flags=0 if bf16 else 0, gain_jitter=0.1, batch=batch, max_seq=max_seq,
                   prefill_rows=64 if "prefill_call" in case else 0)
    perm = np.random.default_rng(77).permutation(batch * (max_seq // 32)).astype(np.int32)
    ls.gpu.set_page_table(perm)
    prompts = synth.make_prompts(shape, seed=15) if batch > 1 else [synth.make_prompts(shape, seed=15)[0][:61]]
    say(f"paged KV {case}: prompts {[len(p) for p in prompts]}, page table {perm[:8].tolist()}...")
    if "prefill_call" in case:
        ls.prefill_prompts(prompts, oracle_chunk=32)
    else:
        ls.prefill(prompts, chunk=16)
    want = [3, 1, 4, 2]
    hook = truth_hook_factory(ls, want)
    for s in range(len(want)):
        ms = ls.step(tree_hook=hook)
        say(f"  step {s}: want {want[s]} got {ms} max|dlogit|={ls.max_logit_err:.2e} max|dKV|={ls.max_kv_err:.2e}")
    for s in range(2):
        ls.step()
    assert ls.max_logit_err <= (3e-2 if bf16 else 1e-4)
    with pytest.raises(clover.CloverError) as e:
        ls.gpu.set_page_table(np.zeros(batch * (max_seq // 32), np.int32))     # not a permutation
    assert e.value.code == clover.E_SHAPE


# ------------------------------------------------------------------------------------------
# linear-size tree mask (Appendix A.1): interval labels instead of one bit set per node
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("case", ["fp32_generic", "bf16_mfma", "bf16_generic", "bf16_dynamic_batch2"])
def test_interval_mask(case):
    """The same lock-step runs as with the bit-set mask, with CLOVER_FLAG_INTERVAL_MASK: random topologies (the mask
    is the only thing that tells siblings apart), injected accept lengths, a dynamic tree whose labels the selection
    kernel writes per sequence."""
    _torch()
    from tests.parity import bfs_tree_random, truth_hook_factory
    bf16 = case.startswith("bf16")
    flags = clover.FLAG_INTERVAL_MASK | (clover.FLAG_GENERIC if "generic" in case else 0)
    rng = np.random.default_rng(29)
    if "dynamic" in case:
        shape = synth.scaled(MINI, batch=2, prompt_len=(20, 40), seed=63)
        ls = _lockstep(shape, flags=flags, gain_jitter=0.1, batch=2, max_seq=384, max_nodes=32, dynamic=(24, 4, 4))
        ls.prefill(synth.make_prompts(shape, seed=35), chunk=16)
        hook = None
    else:
        shape = MINI if bf16 else TINY
        parent, rank = bfs_tree_random(rng, 24 if bf16 else 16, 4 if bf16 else 3)
        say(f"interval mask {case}: random tree parents", parent.tolist())
        ls = _lockstep(shape, flags=flags, gain_jitter=0.1, tree=(parent, rank), max_seq=256, max_nodes=len(parent))
        ls.prefill([synth.make_prompts(shape, seed=9)[0][:37]], chunk=8)
        hook = None
    assert ls.gpu.path_info() == (0 if "generic" in case or not bf16 else 3)
    for s in range(4):
        ms = ls.step(tree_hook=hook)
        say(f"  step {s}: m={ms} max|dlogit|={ls.max_logit_err:.2e} ties={ls.tie_events}")
    assert ls.max_logit_err <= (3e-2 if bf16 else 1e-4)


def test_interval_mask_160_node_tree():
    """A static tree of 160 nodes (beyond the 128 of the bit-set mask): five node groups per KV head in the attention,
    160 rows per pass through the many-row GEMM; injected accept lengths up to the full depth."""
    _torch()
    from tests.parity import truth_hook_factory
    shape = synth.scaled(MINI, name="mini-160", tree_k=(8, 6, 4, 3), tree_nodes=160, seed=65)
    ls = _lockstep(shape, flags=clover.FLAG_INTERVAL_MASK, gain_jitter=0.1, max_seq=768)
    assert len(ls.parent) == 160
    ls.prefill([synth.make_prompts(shape, seed=5)[0][:70]], chunk=64)
    want = [5, 2, 1]
    hook = truth_hook_factory(ls, want)
    for s in range(len(want)):
        ties = ls.tie_events
        ms = ls.step(tree_hook=hook)
        say(f"  step {s}: want {want[s]} got {ms} max|dlogit|={ls.max_logit_err:.2e} ties={ls.tie_events}")
        if ls.tie_events == ties:
            assert ms == [want[s]]
    ms = ls.step()
    say(f"  free step: m={ms} max|dlogit|={ls.max_logit_err:.2e}")
    assert ls.max_logit_err <= 3e-2
    with pytest.raises(clover.CloverError) as e:      # without the flag the bit sets bound the tree at 128 nodes
        clover.Clover(shape, ls.dev_w, ls.parent, ls.rank, 1, 768, 160)
    assert e.value.code == clover.E_CONFIG


# ------------------------------------------------------------------------------------------
# dynamic (score-pruned) tree: a new topology per sequence and step (Sec. 4.1)
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("case", ["fp32", "fp32_generic_batch2", "bf16", "bf16_generic"])
def test_dynamic_tree(case):
    _torch()
    from tests.parity import truth_hook_factory
    bf16 = case.startswith("bf16")
    shape = MINI if bf16 else TINY
    batch = 2 if "batch2" in case else 1
    if batch > 1:
        shape = synth.scaled(shape, batch=batch, prompt_len=(20, 40), seed=61)
    flags = clover.FLAG_GENERIC if "generic" in case else 0
    dyn = (24, 4, 4) if bf16 else (16, 4, 3)          # (tree nodes, children per expansion, expansions per depth)
    ls = _lockstep(shape, flags=flags, gain_jitter=0.1, batch=batch, max_seq=384, max_nodes=32, dynamic=dyn)
    prompts = synth.make_prompts(shape, seed=33) if batch > 1 else [synth.make_prompts(shape, seed=33)[0][:45]]
    say(f"dynamic tree {case}: {dyn}, prompts {[len(p) for p in prompts]}")
    ls.prefill(prompts, chunk=16)
    want = [3, 1, 2, 4] if bf16 else [3, 1, 2]
    hook = truth_hook_factory(ls, want)
    for s in range(len(want)):
        ties = ls.tie_events
        ms = ls.step(tree_hook=hook)
        say(f"  step {s}: want {want[s]} got {ms} parents {ls.parents[0].tolist()} max|dlogit|={ls.max_logit_err:.2e} "
            f"max|dscore|={ls.max_score_err:.2e} ties={ls.tie_events}")
        if ls.tie_events == ties:
            assert all(mb <= want[s] for mb in ms) and max(ms) >= 1   # the tree of a step may be shallower than asked
    for s in range(3):
        ms = ls.step()
        say(f"  free step {s}: m={ms} max|dlogit|={ls.max_logit_err:.2e} max|ddraft|={ls.max_draft_logit_err:.2e}")
    assert ls.max_logit_err <= (3e-2 if bf16 else 1e-4)


def test_dynamic_tree_full_width():
    """The LLaMA3-8B-shaped workload's widths (2 layers) with a 64-node dynamic tree: 8 children per expansion,
    8 expansions per depth, 201 candidates per step."""
    _torch()
    O = __import__("oracle.clover2_oracle", fromlist=["x"])
    shape = synth.scaled(synth.CONFIGS[3], name="wide-dynamic", n_layers=2, prompt_len=(100, 100), seed=71)
    ls = _lockstep(shape, max_seq=512, dynamic=(64, 8, 8))
    ls.ocfg.dtype = np.float32
    ls.W = O.Weights(ls.store.get_f32, np.float32)
    ls.seqs = [O.SeqState(ls.ocfg)]
    ls.prefill(synth.make_prompts(shape), chunk=64)
    for s in range(2):
        ms = ls.step()
        say(f"  step {s}: m={ms} depth of tree {int(__import__('oracle.clover2_oracle', fromlist=['x']).tree_depths(ls.parents[0]).max())} "
            f"max|dlogit|={ls.max_logit_err:.2e} max|dscore|={ls.max_score_err:.2e} ties={ls.tie_events}")
    # and verification at a temperature over the full vocabulary (the draw inverts a 128256-entry cumulative sum)
    for s, temp in enumerate([1.0, 0.05, 1.0]):
        ms = ls.step(sampled=(temp, 300 + s))
        say(f"  sampled step T={temp}: m={ms} ties={ls.tie_events}")
    assert ls.max_logit_err <= 3e-2


def test_dynamic_tree_argument_errors():
    _torch()
    ls = _lockstep(TINY, max_seq=128, max_nodes=32)
    g = ls.gpu
    for args, code in [((33, 4, 3), clover.E_TREE), ((16, 17, 3), clover.E_TREE), ((16, 4, 65), clover.E_TREE),
                       ((16, 16, 16), clover.E_TREE),      # 1 + 16 + 2 * 16 * 16 candidates > 256
                       ((32, 2, 1), clover.E_TREE)]:       # 1 + 2 + 2 * 2 = 7 candidates < 32 nodes
        with pytest.raises(clover.CloverError) as e:
            g.set_dynamic_tree(*args)
        assert e.value.code == code, args
    g.set_dynamic_tree(16, 4, 3)
    with pytest.raises(clover.CloverError):
        g.accept_forced(1)                                  # prompt chunks need the chain tree


# ------------------------------------------------------------------------------------------
# verification at a temperature > 0 (Table 1, temperature 1 rows)
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("case", ["fp32", "bf16", "bf16_dynamic_tree"])
def test_sampled_verification(case):
    """Same seeded uniforms on both sides: identical walks and draws (threshold cases within tolerance), the
    compaction and the hand-off that follow, over several steps; a low temperature makes acceptances frequent
    when the tree carries the target's favourite continuation, temperature 1 exercises the draw from the rest."""
    _torch()
    from tests.parity import truth_hook_factory
    bf16 = case.startswith("bf16")
    shape = MINI if bf16 else TINY
    dyn = (24, 4, 4) if case.endswith("dynamic_tree") else None
    ls = _lockstep(shape, gain_jitter=0.1, max_seq=384, max_nodes=32, dynamic=dyn)
    ls.prefill([synth.make_prompts(shape, seed=52)[0][:41]], chunk=16)
    want = [4, 3, 2, 4, 3, 4]
    hook = truth_hook_factory(ls, want)
    seen = []
    for s, temp in enumerate([0.02, 0.05, 1.0, 0.02, 0.3, 1.0]):
        ms = ls.step(tree_hook=hook, sampled=(temp, 100 + s))
        say(f"  step {s}: T={temp} planted {want[s]} accepted {ms} ties={ls.tie_events}")
        seen.append(ms[0])
    assert max(seen) >= 2 and min(seen) == 1            # both outcomes occurred
    for s in range(4):
        ms = ls.step(sampled=(1.0, 200 + s))
    assert ls.max_logit_err <= (3e-2 if bf16 else 1e-4)


def test_sampled_verification_crafted():
    """Crafted logits through the C ABI: probabilities 0.5 / 0.25 / 0.25 over three tokens at the root, two of them
    offered as children; the uniforms decide exactly which branch is taken."""
    torch = _torch()
    shape = TINY
    parent = np.asarray([-1, 0, 0, 1], np.int32)
    rank = np.asarray([0, 0, 1, 0], np.int32)
    ls = _lockstep(shape, tree=(parent, rank), max_seq=128, max_nodes=16)
    g = ls.gpu
    ls.prefill([synth.make_prompts(shape, seed=77)[0][:17]], chunk=8)
    toks = np.zeros((1, g.R), np.int32)
    toks[0, :4] = [int(g.tree_tokens[0, 0].item()), 11, 22, 33]
    base = np.full((4, shape.vocab), -1e4, np.float32)
    base[0, [11, 22, 44]] = np.log([0.5, 0.25, 0.25])       # root: child tokens 11 (p .5), 22 (p .25); 44 not offered
    base[1, [33, 55]] = np.log([0.5, 0.5])                  # node 1: child token 33 (p .5)
    base[2, 66] = 0.0                                       # node 2 (leaf): 66 with certainty
    base[3, [70, 71]] = np.log([0.25, 0.75])                # node 3 (leaf)
    cases = [  # uniforms at (node, slot) -> expected path, next token
        ({(0, 0): 0.49, (1, 0): 0.49, (3, 16): 0.24}, [0, 1, 3], 70),
        ({(0, 0): 0.49, (1, 0): 0.49, (3, 16): 0.26}, [0, 1, 3], 71),
        ({(0, 0): 0.49, (1, 0): 0.51, (1, 16): 0.9}, [0, 1], 55),
        ({(0, 0): 0.51, (0, 1): 0.49, (2, 16): 0.3}, [0, 2], 66),     # 22 accepted with 0.25 / (1 - 0.5) = 0.5
        ({(0, 0): 0.51, (0, 1): 0.51, (0, 16): 0.7}, [0], 44),        # both refused: only 44 is left
    ]
    for uni_set, want_path, want_tok in cases:
        g.tree_tokens.copy_(torch.from_numpy(toks))
        g.verify_tree(1)                                     # K/V rows for the compaction that follows
        g.logits[0, :4].copy_(torch.from_numpy(base))
        uni = np.full((1, g.R, 17), 0.999, np.float32)
        for (node, slot), v in uni_set.items():
            uni[0, node, slot] = v
        L = int(g.seq_len()[0])
        g.accept_and_compact_sampled(1, 1.0, torch.from_numpy(uni).to(g.dev))
        torch.cuda.synchronize()
        m = int(g.m[0].item())
        assert g.acc_idx[0, :m].cpu().tolist() == want_path, (uni_set, g.acc_idx[0, :m].cpu().tolist())
        assert int(g.new_tokens[0, m - 1].item()) == want_tok
        assert g.new_tokens[0, :m - 1].cpu().tolist() == [int(toks[0, u]) for u in want_path[1:]]
        assert int(g.seq_len()[0]) == L + m
        # the same decisions from the oracle's procedure on the same numbers
        O = __import__("oracle.clover2_oracle", fromlist=["x"])
        path, bonus, _ = O.accept_sampled(toks[0, :4], base.astype(np.float64), parent, 1.0, uni[0].astype(np.float64))
        assert (path, bonus) == (want_path, want_tok)
        # keep the draft head's cache in step with the target's
        g.draft_tree(1)
    with pytest.raises(clover.CloverError) as e:
        g.accept_and_compact_sampled(1, 0.0, torch.from_numpy(uni).to(g.dev))
    assert e.value.code == clover.E_SHAPE


# ------------------------------------------------------------------------------------------
# acceptance and compaction on crafted logits: overlapping moves, a sibling search, a late child
# ------------------------------------------------------------------------------------------
CRAFTED = [
    # parent array, accepted path it must produce
    ([-1, 0, 1, 2], [0, 1, 2, 3]),                  # chain accepted whole: every move is the identity, m = D + 1
    ([-1, 0, 0, 1, 1, 2, 2], [0, 2, 5]),            # slot L+1 <- L+2, slot L+2 <- L+5: a destination is an earlier source
    ([-1, 0, 0, 0, 0, 1], [0, 4]),                  # the last of four siblings
    ([-1, 0, 0, 1, 2, 2, 4, 5, 5], [0, 2, 5, 8]),   # moves 2->1, 5->2, 8->3
]


@pytest.mark.parametrize("bf16", [False, True], ids=["fp32", "bf16"])
@pytest.mark.parametrize("case", range(len(CRAFTED)))
def test_accept_and_compact_crafted_paths(bf16, case):
    torch = _torch()
    O = __import__("oracle.clover2_oracle", fromlist=["x"])
    shape = MINI if bf16 else TINY
    parent, want_path = CRAFTED[case]
    parent = np.asarray(parent, np.int32)
    n = len(parent)
    kids = O.children_of(parent)
    rank = np.zeros(n, np.int32)
    for u in range(n):
        for i, c in enumerate(kids[u]):
            rank[c] = i
    say(f"crafted accept: parent {parent.tolist()} path {want_path} bf16={bf16}")
    ls = _lockstep(shape, gain_jitter=0.1, tree=(parent, rank), max_seq=128, max_nodes=16)
    g = ls.gpu
    ls.prefill([synth.make_prompts(shape, seed=40 + case)[0][:23]], chunk=8)
    L = int(g.seq_len()[0])
    tokens = np.zeros((1, g.R), np.int32)
    tokens[0, :n] = 100 + 7 * np.arange(n)                      # distinct ids
    tokens[0, 0] = int(g.tree_tokens[0, 0].item())              # the root stays the hand-off token
    g.tree_tokens.copy_(torch.from_numpy(tokens))
    g.verify_tree(1)
    torch.cuda.synchronize()
    seq = ls.seqs[0]
    o_hidden, o_logits = O.verify_tree(ls.W, ls.ocfg, seq, tokens[0, :n], parent)     # fills the oracle's tree rows
    pre = [g.read_kv(0, l, 0, L, n) for l in range(shape.n_layers)]
    hidden = g.hidden.cpu().numpy()
    # one-hot logits that walk exactly want_path and then emit `bonus`
    bonus = 77
    logits = np.zeros((n, shape.vocab), np.float32)
    logits[:, 3] = 1.0                                          # off-path nodes point at a token nobody carries
    for i, u in enumerate(want_path):
        logits[u, 3] = 0.0
        logits[u, tokens[0, want_path[i + 1]] if i + 1 < len(want_path) else bonus] = 5.0
    g.logits[0, :n].copy_(torch.from_numpy(logits))
    g.accept_and_compact(1)
    torch.cuda.synchronize()
    m = int(g.m[0].item())
    acc = O.accept_and_compact(ls.ocfg, seq, tokens[0, :n], logits.astype(np.float64), o_hidden, parent)
    assert acc["path"] == want_path                             # the crafted case means what it says
    assert m == len(want_path)
    assert g.acc_idx[0, :m].cpu().tolist() == want_path
    assert g.new_tokens[0, :m].cpu().tolist() == acc["new_tokens"] == [int(tokens[0, u]) for u in want_path[1:]] + [bonus]
    assert g.next_tok[0, :m].cpu().tolist() == acc["next_tok"]
    assert int(g.seq_len()[0]) == L + m == seq.L
    np.testing.assert_array_equal(g.hid_acc[0, :m].cpu().numpy(), hidden[0, want_path])
    for l in range(shape.n_layers):
        k2, v2 = g.read_kv(0, l, 0, L, m)
        np.testing.assert_array_equal(k2, pre[l][0][want_path])  # the moves carry bits, in an order that keeps sources intact
        np.testing.assert_array_equal(v2, pre[l][1][want_path])
    ls.compare_kv(0, L, L + m, stacks=(0,))                      # and the compacted rows are the oracle's


# ------------------------------------------------------------------------------------------
# error paths reachable without touching the kernels
# ------------------------------------------------------------------------------------------
def test_capacity_and_shape_errors():
    _torch()
    ls = _lockstep(TINY, max_seq=64)
    g = ls.gpu
    with pytest.raises(clover.CloverError) as e:
        g.verify_tree(2)
    assert e.value.code == clover.E_SHAPE
    ls.prefill([synth.make_prompts(TINY, seed=2)[0][:16]], chunk=16)
    g.verify_tree(1)
    g.accept_and_compact(1)
    with pytest.raises(clover.CloverError) as e:      # the host-side length bound grows by D+1 per step
        for _ in range(12):
            g.draft_tree(1); g.verify_tree(1); g.accept_and_compact(1)
    assert e.value.code == clover.E_CAPACITY
    assert g.seq_len()[0] <= 64


# ------------------------------------------------------------------------------------------
# full size: the LLaMA3-8B-shaped batch-1 workload exactly as bench.py runs it
# ------------------------------------------------------------------------------------------
def test_config3_full_size_step():
    """All 32 layers, vocab 128256, 64-node tree over a 1024-token prompt: every logit of the
    verify pass, the tree KV rows, acceptance, compaction and the next draft tree against the
    oracle (fp32 NumPy on the host cores, same bf16-rounded weights)."""
    _torch()
    from tests.parity import truth_hook_factory
    shape = synth.CONFIGS[3]
    say("config 3 full size: generating weights, prefilling 1024 tokens on both sides")
    ls = _lockstep(shape, max_seq=1024 + 3 * 64 + 64)
    assert ls.gpu.path_info() & 3 == 3   # MFMA GEMMs and MFMA attention, as bench.py runs it
    ls.ocfg.dtype = np.float32
    ls.W = __import__("oracle.clover2_oracle", fromlist=["x"]).Weights(ls.store.get_f32, np.float32)
    ls.seqs = [__import__("oracle.clover2_oracle", fromlist=["x"]).SeqState(ls.ocfg)]
    ls.prefill(synth.make_prompts(shape), chunk=64)
    say(f"  prefill ok, tie events {ls.tie_events}")
    want = [3, 1]
    hook = truth_hook_factory(ls, want)
    for s in range(len(want)):
        ties = ls.tie_events
        ms = ls.step(tree_hook=hook)
        say(f"  step {s}: want {want[s]} got {ms} max|dlogit|={ls.max_logit_err:.3e} "
            f"max|dhidden|={ls.max_hidden_err:.3e} ties={ls.tie_events}")
        if ls.tie_events == ties:
            assert ms == [want[s]]
    assert ls.max_logit_err <= 3e-2


def test_config2_full_size_step():
    """The Vicuna-7B-shaped workload at full size (32 layers, 32 MHA heads, FFN 11008, vocab 32000, RoPE base 1e4,
    64-node tree over a 512-token prompt): its shapes take other launch routes than the LLaMA3 one (K = 11008 ends
    in a 256-column slice, 688 gate/up column blocks, one query head per KV head)."""
    _torch()
    from tests.parity import truth_hook_factory
    O = __import__("oracle.clover2_oracle", fromlist=["x"])
    shape = synth.CONFIGS[2]
    say("config 2 full size: generating weights, prefilling 512 tokens on both sides")
    ls = _lockstep(shape, max_seq=512 + 3 * 64 + 64)
    assert ls.gpu.path_info() & 3 == 3
    ls.ocfg.dtype = np.float32
    ls.W = O.Weights(ls.store.get_f32, np.float32)
    ls.seqs = [O.SeqState(ls.ocfg)]
    ls.prefill(synth.make_prompts(shape), chunk=64)
    say(f"  prefill ok, tie events {ls.tie_events}")
    want = [2, 1]
    hook = truth_hook_factory(ls, want)
    for s in range(len(want)):
        ties = ls.tie_events
        ms = ls.step(tree_hook=hook)
        say(f"  step {s}: want {want[s]} got {ms} max|dlogit|={ls.max_logit_err:.3e} "
            f"max|dhidden|={ls.max_hidden_err:.3e} ties={ls.tie_events}")
        if ls.tie_events == ties:
            assert ms == [want[s]]
    assert ls.max_logit_err <= 3e-2


@pytest.mark.parametrize("cfg,batch", [(4, 8), (4, 5), (5, 1)], ids=["batch8_256_rows", "batch5_160_rows", "tree96_depth5"])
def test_full_width_two_layers(cfg, batch):
    """Configs 4 and 5 at their real widths (H 4096, FFN 14336, vocab 128256, 32/8 heads) with two layers and short
    prompts, so that the oracle stays quick: passes of 96 and 256 rows take the 128-row routes of the real shapes
    (QKV, Wo and down over K ranges of the panel kernel, gate+up and LM head full-K), which the small models above
    are too narrow for."""
    _torch()
    O = __import__("oracle.clover2_oracle", fromlist=["x"])
    base = synth.CONFIGS[cfg]
    # (160 rows: a full 128-row batch followed by a short one)
    shape = synth.scaled(base, name=f"wide-{cfg}-{batch}", n_layers=2, batch=batch,
                         prompt_len=(24, 90) if cfg == 4 else (150, 150), seed=31 + cfg + batch)
    ls = _lockstep(shape, batch=shape.batch, max_seq=384)
    assert ls.gpu.path_info() & 3 == 3
    ls.ocfg.dtype = np.float32
    ls.W = O.Weights(ls.store.get_f32, np.float32)
    ls.seqs = [O.SeqState(ls.ocfg) for _ in range(shape.batch)]
    prompts = synth.make_prompts(shape)
    say(f"config {cfg} widths, 2 layers: prompt lengths {[len(p) for p in prompts]}")
    ls.prefill(prompts, chunk=len(synth.tree_for(shape)[0]))
    for s in range(2):
        ms = ls.step()
        say(f"  step {s}: m={ms} max|dlogit|={ls.max_logit_err:.3e} ties={ls.tie_events}")
    assert ls.max_logit_err <= 3e-2


# ------------------------------------------------------------------------------------------
# the prefill call: many-row passes with causal attention, LM head on the last row only (Sec. 1, 3.1, 3.3)
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("flags,prefill_rows,lengths", [
    (0, 128, [300, 77]),                       # 128 + 128 + 44 rows; a prompt shorter than one pass
    (0, 256, [600, 1]),                        # 256 + 256 + 88 rows; a one-token prompt (no draft-side row)
    (0, 0, [50, 24]),                          # no extra capacity: passes of max_batch * max_nodes = 48 rows
    (clover.FLAG_GENERIC, 96, [200, 96]),      # the plain fp32 kernels; a prompt of exactly one pass
], ids=["mfma_128", "mfma_256", "mfma_default_rows", "generic_96"])
def test_prefill_call_mini_bf16(flags, prefill_rows, lengths):
    _torch()
    shape = synth.scaled(MINI, batch=2, seed=41)
    ls = _lockstep(shape, flags=flags, gain_jitter=0.1, batch=2, max_seq=768, prefill_rows=prefill_rows)
    rng = np.random.default_rng(7)
    prompts = [rng.integers(0, shape.vocab, size=n).astype(np.int32) for n in lengths]
    say(f"prefill call, flags={flags}, rows per pass {prefill_rows or 48}: prompts {lengths}")
    ls.prefill_prompts(prompts, oracle_chunk=64)
    say(f"  after prefill: max|dlogit|={ls.max_logit_err:.2e} max|dKV|={ls.max_kv_err:.2e} max|dhid|={ls.max_hidden_err:.2e}")
    for s in range(3):
        ms = ls.step()
        say(f"  step {s}: m={ms} max|dlogit|={ls.max_logit_err:.2e} ties={ls.tie_events}")
    assert ls.max_logit_err <= 3e-2


def test_prefill_call_config1_fp32():
    _torch()
    ls = _lockstep(TINY, max_seq=256, prefill_rows=40)
    prompts = synth.make_prompts(TINY)
    say("config 1: prefill call, 64 tokens in passes of 40 rows")
    ls.prefill_prompts(prompts, oracle_chunk=16)
    for s in range(4):
        ms = ls.step()
        say(f"  step {s}: m={ms} max|dlogit|={ls.max_logit_err:.2e}")
    assert ls.max_logit_err <= 1e-4


def test_prefill_call_full_width_two_layers():
    """The prefill call at the LLaMA3-8B widths (two layers): a 600-token prompt in passes of 256 rows through the
    many-row GEMM, causal attention over eight node groups, then two speculative steps on top."""
    _torch()
    O = __import__("oracle.clover2_oracle", fromlist=["x"])
    shape = synth.scaled(synth.CONFIGS[3], name="wide-3-prefill", n_layers=2, seed=43)
    ls = _lockstep(shape, max_seq=768, prefill_rows=256)
    assert ls.gpu.path_info() & 3 == 3
    ls.ocfg.dtype = np.float32
    ls.W = O.Weights(ls.store.get_f32, np.float32)
    ls.seqs = [O.SeqState(ls.ocfg)]
    rng = np.random.default_rng(9)
    prompts = [rng.integers(0, shape.vocab, size=600).astype(np.int32)]
    ls.prefill_prompts(prompts, oracle_chunk=128)
    say(f"  after prefill: max|dlogit|={ls.max_logit_err:.2e} max|dKV|={ls.max_kv_err:.2e} max|dhid|={ls.max_hidden_err:.2e}")
    for s in range(2):
        ms = ls.step()
        say(f"  step {s}: m={ms} max|dlogit|={ls.max_logit_err:.3e} ties={ls.tie_events}")
    assert ls.max_logit_err <= 3e-2


def test_prefill_call_argument_errors():
    _torch()
    torch = _torch()
    ls = _lockstep(MINI, max_seq=128, prefill_rows=64)
    g = ls.gpu
    toks = torch.zeros(200, dtype=torch.int32, device=g.dev)
    out = [C.c_void_p(t.data_ptr()) for t in (g.logits[0, 0], g.hid_acc[0, 0], g.next_tok[0, 0])]
    assert g.lib.clover_prefill(g.ctx, 1, C.c_void_p(toks.data_ptr()), 10, *out) == clover.E_SHAPE      # sequence 1 of 1
    assert g.lib.clover_prefill(g.ctx, 0, None, 10, *out) == clover.E_NULL
    assert g.lib.clover_prefill(g.ctx, 0, C.c_void_p(toks.data_ptr()), 0, *out) == clover.E_SHAPE       # empty prompt
    with pytest.raises(clover.CloverError) as e:
        g.prefill_prompt(0, toks[:129])
    assert e.value.code == clover.E_CAPACITY
    with pytest.raises(clover.CloverError) as e:
        clover.Clover(MINI, ls.dev_w, ls.parent, ls.rank, 1, 128, 24, prefill_rows=257)
    assert e.value.code == clover.E_CONFIG


# ------------------------------------------------------------------------------------------
# the long-context and the ragged batch-8 workloads at their real widths AND their real cache lengths
# ------------------------------------------------------------------------------------------
def _seeded(cfg, lengths, seed, max_seq, n_layers=2):
    O = __import__("oracle.clover2_oracle", fromlist=["x"])
    base = synth.CONFIGS[cfg]
    shape = synth.scaled(base, name=f"wide-{cfg}-seeded", n_layers=n_layers, batch=len(lengths), seed=seed)
    ls = _lockstep(shape, batch=len(lengths), max_seq=max_seq)
    assert ls.gpu.path_info() & 3 == 3
    ls.ocfg.dtype = np.float32
    ls.W = O.Weights(ls.store.get_f32, np.float32)
    ls.seqs = [O.SeqState(ls.ocfg) for _ in lengths]
    ls.seed_cache(lengths, seed)
    return ls


def test_config5_8192_cached_keys_96_node_tree():
    """The long-context workload at its real size except for the layer count: H 4096, 32/8 heads, vocab 128256,
    8192 cached keys (seeded rows written straight into both caches), 96-node tree of depth 5: the attention runs
    its full split arithmetic (several hundred key tiles over the key splits, three node groups), every logit,
    tree K/V row and draft logit is compared with the oracle, and two steps accept 4 and 2 nodes."""
    _torch()
    from tests.parity import truth_hook_factory
    say("config 5 widths, 2 layers, 8192 seeded cache rows")
    ls = _seeded(5, [8192], seed=51, max_seq=8192 + 4 * 96)
    want = [4, 2]
    hook = truth_hook_factory(ls, want)
    for s in range(len(want)):
        ties = ls.tie_events
        ms = ls.step(tree_hook=hook)
        say(f"  step {s}: want {want[s]} got {ms} max|dlogit|={ls.max_logit_err:.3e} max|dhidden|={ls.max_hidden_err:.3e} "
            f"max|dKV|={ls.max_kv_err:.3e} max|ddraft|={ls.max_draft_logit_err:.3e} ties={ls.tie_events}")
        if ls.tie_events == ties:
            assert ms == [want[s]]
    assert ls.max_logit_err <= 3e-2


def test_long_key_splits_with_shuffled_pages():
    """Batch 8 over caches of up to 8400 keys: 64 (sequence, KV head) pairs leave four key splits of 66 tiles each, more
    than the 64 page numbers one register of the attention kernel holds per split, and the page table is a random
    permutation, so the tiles past the 64th of a split are fetched through the second page-number register from
    scattered pages.  Ragged lengths: short sequences end inside the first split."""
    _torch()
    from tests.parity import truth_hook_factory
    lengths = [8400, 300, 8211, 1500, 64, 8388, 4000, 700]
    max_seq = 8576
    O = __import__("oracle.clover2_oracle", fromlist=["x"])
    shape = synth.scaled(synth.CONFIGS[4], name="wide-4-long-splits", n_layers=2, batch=len(lengths), seed=43)
    ls = _lockstep(shape, batch=len(lengths), max_seq=max_seq)
    assert ls.gpu.path_info() & 3 == 3
    perm = np.random.default_rng(78).permutation(len(lengths) * (max_seq // 32)).astype(np.int32)
    ls.gpu.set_page_table(perm)
    ls.ocfg.dtype = np.float32
    ls.W = O.Weights(ls.store.get_f32, np.float32)
    ls.seqs = [O.SeqState(ls.ocfg) for _ in lengths]
    ls.seed_cache(lengths, 43)
    say(f"long key splits: lengths {lengths}, shuffled page table {perm[:6].tolist()}...")
    want = [2, 3]
    hook = truth_hook_factory(ls, want)
    for s in range(len(want)):
        ms = ls.step(tree_hook=hook)
        say(f"  step {s}: want {want[s]} got {ms} max|dlogit|={ls.max_logit_err:.3e} max|dhidden|={ls.max_hidden_err:.3e} "
            f"max|dKV|={ls.max_kv_err:.3e} ties={ls.tie_events}")
    assert ls.max_logit_err <= 3e-2


def test_config4_ragged_256_to_2048_cached_keys():
    """The batch-8 workload at its real widths and cache lengths (the recipe's eight lengths, uniform in
    [256, 2048]), 32-node trees, 256 rows per pass, 2 layers."""
    _torch()
    from tests.parity import truth_hook_factory
    lengths = [len(p) for p in synth.make_prompts(synth.CONFIGS[4])]
    assert len(lengths) == 8 and min(lengths) >= 256 and max(lengths) <= 2048
    say(f"config 4 widths, 2 layers, seeded cache rows, lengths {lengths}")
    ls = _seeded(4, lengths, seed=41, max_seq=2048 + 4 * 32)
    want = [3, 1]
    hook = truth_hook_factory(ls, want)
    for s in range(len(want)):
        ms = ls.step(tree_hook=hook)
        say(f"  step {s}: want {want[s]} got {ms} max|dlogit|={ls.max_logit_err:.3e} max|dhidden|={ls.max_hidden_err:.3e} "
            f"max|dKV|={ls.max_kv_err:.3e} max|ddraft|={ls.max_draft_logit_err:.3e} ties={ls.tie_events}")
    assert ls.max_logit_err <= 3e-2
