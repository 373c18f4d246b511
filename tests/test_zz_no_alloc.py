"""The entry point that allocates nothing (varlen_attn_fwd_noalloc: tile table built on the device in a fixed device
array) against varlen_attn_fwd, through the C ABI: same kernel, same tiles, so O and LSE must agree bit for bit. Two
calls in a row share the one table; the second is a smaller batch, so stale records of the first sit behind its own."""
import numpy as np
import pytest
import torch

from paper_2509_21841_amd import binding as B, synth

pytestmark = pytest.mark.gpu


def _run_both(lengths, Hq, Hkv, d, seed, skip=None):
    dev = "cuda:0"
    T = int(sum(lengths))
    q, k, v = synth.make_qkv(T, Hq, Hkv, d, seed, dev)
    cu = synth.cu_seqlens(lengths)
    o_ref, lse_ref = B.varlen_attn_fwd(q, k, v, cu, seq_skip=skip)
    # poison the outputs so that rows the call does not write cannot pass by accident
    o = torch.full_like(q, 7.0)
    lse = torch.full((Hq, T), 7.0, dtype=torch.float32, device=dev)
    if skip is not None:   # flagged sequences are not written by either entry point: start both from the same bytes
        o_ref2 = torch.full_like(q, 7.0); lse_ref2 = torch.full_like(lse, 7.0)
        o_ref, lse_ref = B.varlen_attn_fwd(q, k, v, cu, o=o_ref2, lse=lse_ref2, seq_skip=skip)
    B.varlen_attn_fwd_noalloc(q, k, v, cu, o, lse, seq_skip=skip)
    torch.cuda.synchronize()
    assert np.array_equal(synth.bf16_bits(o), synth.bf16_bits(o_ref)), "O differs from varlen_attn_fwd"
    assert np.array_equal(lse.cpu().numpy().view(np.uint32), lse_ref.cpu().numpy().view(np.uint32)), "LSE differs"


def test_noalloc_forward_equals_forward_on_two_calls_in_a_row():
    # ragged lengths over several tiles with tails, zero-length and one-token sequences, equal costs across sequences
    big = [700, 129, 0, 1, 128, 2049, 64, 300, 256, 513, 127]
    _run_both(big, 8, 2, 128, 2101)
    small = [130, 5, 0, 384]
    _run_both(small, 8, 2, 128, 2102)
    # head dimension 64, MHA, and a flagged sequence, again on the same table
    skip = np.zeros(len(big), np.uint8); skip[5] = 1
    _run_both(big, 4, 4, 64, 2103, skip=skip)
    _run_both([64], 4, 4, 64, 2104)


def test_noalloc_at_its_limits():
    # exactly the largest tile table (8192 blocks of 128 rows, a million tokens), then exactly the most sequences
    assert B.NOALLOC_MAX_TILES % 16 == 0
    _run_both([2048] * (B.NOALLOC_MAX_TILES // 16), 1, 1, 64, 2105)
    rng = np.random.default_rng(2106)
    _run_both([int(x) for x in rng.integers(0, 300, size=B.NOALLOC_MAX_SEQS)], 2, 1, 64, 2106)


def test_noalloc_limits_are_errors():
    dev = "cuda:0"
    lengths = [1] * (B.NOALLOC_MAX_SEQS + 1)
    T = sum(lengths)
    q, k, v = synth.make_qkv(T, 2, 2, 64, 5, dev)
    o = torch.empty_like(q); lse = torch.empty((2, T), dtype=torch.float32, device=dev)
    with pytest.raises(B.ZpError) as e:
        B.varlen_attn_fwd_noalloc(q, k, v, synth.cu_seqlens(lengths), o, lse)
    assert e.value.code == -5


def test_noalloc_forward_replays_from_a_captured_graph():
    """What the entry point is for: one call recorded into a HIP graph (nothing in it allocates, uploads or clears
    memory with a memset node), replayed on new contents of the same buffers, each replay against an eager
    varlen_attn_fwd of the same inputs, with the program's own eager work and synchronisations in between."""
    dev = "cuda:0"
    lengths = [900, 129, 0, 1, 2049, 64, 300]
    Hq, Hkv, d = 8, 2, 128
    T = int(sum(lengths))
    cu = np.asarray(synth.cu_seqlens(lengths))
    q, k, v = synth.make_qkv(T, Hq, Hkv, d, 2201, dev)
    o = torch.full_like(q, 7.0)
    lse = torch.full((Hq, T), 7.0, dtype=torch.float32, device=dev)
    B.varlen_attn_fwd_noalloc(q, k, v, cu, o, lse)      # first call on the device: looks up the array's address
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        B.varlen_attn_fwd_noalloc(q, k, v, cu, o, lse)  # on the capture stream (torch's current stream here)
    for rep in range(3):
        q2, k2, v2 = synth.make_qkv(T, Hq, Hkv, d, 2300 + rep, dev)
        q.copy_(q2); k.copy_(k2); v.copy_(v2)
        o_ref, lse_ref = B.varlen_attn_fwd(q, k, v, cu)
        o.fill_(7.0); lse.fill_(7.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(synth.bf16_bits(o), synth.bf16_bits(o_ref)), f"replay {rep}: O differs"
        assert np.array_equal(lse.cpu().numpy().view(np.uint32), lse_ref.cpu().numpy().view(np.uint32)), f"replay {rep}: LSE differs"
