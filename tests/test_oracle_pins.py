"""Pins for the CPU oracle: each check compares it with something that is not itself.

The dense reference below is written independently, element by element with math.exp, over
contiguous (non-paged) K/V and an explicit mask matrix.  The paper prints no worked numeric
example of attention, so the pins are brute force, closed forms and invariants, plus the two
figures the paper does fix: 192 KB of KVCache per token for a 48-layer GQA model with 8 KV heads
of 128 dims in bf16 (Section 2.2), and p*c + (c^2+c)/2 attended pairs per chunk (Eq. 1).
"""
import math

import numpy as np
import pytest
import torch

from oracle import paged_attention as O
from paper_2412_18169_amd import synth


# ------------------------------------------------------------------------------------------
# independent dense reference (pure Python loops; tiny inputs only)
# ------------------------------------------------------------------------------------------

def dense_attention(q, K, V, scale, mask):
    """q [R][d], K,V [L][d] as nested lists of floats; mask[R][L] of bools (True = visible)."""
    out = []
    for i, qi in enumerate(q):
        z = []
        for t, kt in enumerate(K):
            if mask[i][t]:
                z.append((t, scale * math.fsum(a * b for a, b in zip(qi, kt))))
        m = max(v for _, v in z)
        w = [(t, math.exp(v - m)) for t, v in z]
        den = math.fsum(x for _, x in w)
        out.append([math.fsum(x * V[t][j] for t, x in w) / den for j in range(len(V[0]))])
    return out


def make_pool(w, poison=True):
    ranges = synth.alloc_ranges(w, "cpu", poison=poison)
    synth.fill_pool(w, ranges)
    sh = w.shape
    pool = O.OraclePool([synth.to_host_bits(r).reshape(-1) for r in ranges], sh.Hkv, sh.d, sh.B,
                        sh.dtype)
    return ranges, pool


def tiny_shape(dtype="f32", Hq=4, Hkv=2, d=8, B=4):
    return synth.LayerShape(Hq=Hq, Hkv=Hkv, d=d, B=B, dtype=dtype)


def logical(w, seq, dtype64=True):
    L = int(w.seq_lens[seq])
    k, v = synth.kv_logical(w, seq, 0, L)
    return k.double().numpy(), v.double().numpy()


# ------------------------------------------------------------------------------------------
# check 1: brute force against dense, non-paged attention
# ------------------------------------------------------------------------------------------

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_decode_matches_dense_brute_force(dtype):
    sh = tiny_shape(dtype)
    w = synth.custom_workload("t", sh, [1, 3, 4, 5, 13], extra_blocks=3, range_fracs=(0.5, 0.5))
    _, pool = make_pool(w)
    q = synth.q_decode(w)
    out = O.paged_decode(pool, synth.to_host_bits(q), w.table_array(range(w.S)), w.decode_lens,
                         sh.Hq, sh.scale)
    for s in range(w.S):
        K, V = logical(w, s)
        L = K.shape[0]
        for h in range(sh.Hq):
            kvh = h // sh.G
            ref = dense_attention([q[s, h].double().tolist()], K[:, kvh].tolist(),
                                  V[:, kvh].tolist(), float(np.float32(sh.scale)),
                                  [[True] * L])
            np.testing.assert_allclose(out[s, h], ref[0], rtol=0, atol=1e-13)


@pytest.mark.parametrize("p,c", [(0, 6), (5, 7), (8, 1)])
def test_prefill_chunk_matches_dense_causal_brute_force(p, c):
    sh = tiny_shape("bf16")
    w = synth.custom_workload("t", sh, [3], chunks=[(p, c)], extra_blocks=2)
    _, pool = make_pool(w)
    seq = w.S
    q = synth.q_chunk(w, 0)
    out, pairs = O.paged_prefill_chunk(pool, synth.to_host_bits(q), w.block_tables[seq], p, c,
                                       sh.Hq, sh.scale)
    assert pairs == p * c + (c * c + c) // 2            # Eq. 1 attention term
    K, V = logical(w, seq)
    L = p + c
    mask = [[t <= p + r for t in range(L)] for r in range(c)]     # explicit c x L mask matrix
    assert sum(sum(row) for row in mask) == pairs
    for h in range(sh.Hq):
        kvh = h // sh.G
        ref = dense_attention(q[:, h].double().tolist(), K[:, kvh].tolist(), V[:, kvh].tolist(),
                              float(np.float32(sh.scale)), mask)
        np.testing.assert_allclose(out[:, h], np.array(ref), rtol=0, atol=1e-13)


def test_mha_reduces_to_plain_attention_via_library_softmax():
    # Hkv == Hq: no head sharing; compare with torch's own softmax on contiguous tensors.
    sh = synth.LayerShape(Hq=3, Hkv=3, d=16, B=4, dtype="f32")
    w = synth.custom_workload("t", sh, [9, 21])
    _, pool = make_pool(w)
    q = synth.q_decode(w)
    out = O.paged_decode(pool, synth.to_host_bits(q), w.table_array(range(w.S)), w.decode_lens,
                         sh.Hq, sh.scale)
    for s in range(w.S):
        k, v = synth.kv_logical(w, s, 0, int(w.decode_lens[s]))
        z = torch.einsum("hd,thd->ht", q[s].double(), k.double()) * float(np.float32(sh.scale))
        ref = torch.einsum("ht,thd->hd", torch.softmax(z, dim=1), v.double())
        np.testing.assert_allclose(out[s], ref.numpy(), rtol=0, atol=1e-13)


# ------------------------------------------------------------------------------------------
# check 2: invariance to the physical placement of blocks (also across ranges)
# ------------------------------------------------------------------------------------------

def test_invariant_under_block_permutation_and_range_moves():
    sh = tiny_shape("bf16", Hq=4, Hkv=2, d=8, B=4)
    lens = [2, 9, 16, 23]
    outs = []
    for seed, fracs in [(1, (1.0,)), (2, (1.0,)), (3, (0.3, 0.3, 0.4)), (4, (0.1, 0.9))]:
        w = synth.custom_workload("t", sh, lens, chunks=[(5, 6)], seed=99, extra_blocks=5,
                                  range_fracs=fracs)
        # same logical data (seed 99), different placement
        w2 = synth.Workload(w.name, 0, 99, sh, w.decode_lens, w.chunks, w.range_blocks)
        w2.seed = 99
        rng = np.random.default_rng(seed)
        ids = rng.permutation(w.num_blocks)
        need = synth.blocks_needed(w.seq_lens, sh.B)
        o = 0
        for n in need:
            w2.block_tables.append(ids[o:o + int(n)].astype(np.int32))
            o += int(n)
        _, pool = make_pool(w2)
        q = synth.q_decode(w2)
        dec = O.paged_decode(pool, synth.to_host_bits(q), w2.table_array(range(w2.S)),
                             w2.decode_lens, sh.Hq, sh.scale)
        pre, _ = O.paged_prefill_chunk(pool, synth.to_host_bits(synth.q_chunk(w2, 0)),
                                       w2.block_tables[w2.S], 5, 6, sh.Hq, sh.scale)
        outs.append((dec, pre))
    for dec, pre in outs[1:]:
        assert np.array_equal(dec, outs[0][0])          # bit-identical
        assert np.array_equal(pre, outs[0][1])


# ------------------------------------------------------------------------------------------
# check 3: softmax rows sum to 1;  check 4: length-1 context returns V exactly
# ------------------------------------------------------------------------------------------

def test_softmax_rows_sum_to_one():
    rng = np.random.default_rng(0)
    q = rng.standard_normal((7, 16)) * 3
    K = rng.standard_normal((50, 16)) * 3
    V = rng.standard_normal((50, 16))
    vis = [1, 2, 10, 33, 49, 50, 50]
    _, wts = O.attention_rows(q, K, V, 0.25, vis)
    for i, n in enumerate(vis):
        assert abs(wts[i].sum() - 1.0) < 1e-12
        assert np.all(wts[i][n:] == 0.0) and np.all(wts[i][:n] > 0.0)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_length_one_context_returns_v_exactly(dtype):
    sh = tiny_shape(dtype)
    w = synth.custom_workload("t", sh, [1, 1], chunks=[(0, 3)], extra_blocks=1)
    _, pool = make_pool(w)
    q = synth.q_decode(w)
    out = O.paged_decode(pool, synth.to_host_bits(q), w.table_array(range(w.S)), w.decode_lens,
                         sh.Hq, sh.scale)
    for s in range(2):
        _, v = synth.kv_logical(w, s, 0, 1)
        for h in range(sh.Hq):
            assert np.array_equal(out[s, h], v[0, h // sh.G].double().numpy())
    # first row of a chunk with no prior tokens sees only itself
    pre, _ = O.paged_prefill_chunk(pool, synth.to_host_bits(synth.q_chunk(w, 0)),
                                   w.block_tables[2], 0, 3, sh.Hq, sh.scale)
    _, v = synth.kv_logical(w, 2, 0, 1)
    for h in range(sh.Hq):
        assert np.array_equal(pre[0, h], v[0, h // sh.G].double().numpy())


# ------------------------------------------------------------------------------------------
# closed forms
# ------------------------------------------------------------------------------------------

def test_closed_forms():
    rng = np.random.default_rng(1)
    K = rng.standard_normal((20, 8))
    V = rng.standard_normal((20, 8))
    # q = 0: uniform weights -> mean of the visible values
    o, _ = O.attention_rows(np.zeros((2, 8)), K, V, 0.3, [20, 7])
    np.testing.assert_allclose(o[0], V.mean(axis=0), atol=1e-14)
    np.testing.assert_allclose(o[1], V[:7].mean(axis=0), atol=1e-14)
    # identical keys: same
    o, _ = O.attention_rows(rng.standard_normal((1, 8)), np.tile(K[:1], (20, 1)), V, 0.3, [20])
    np.testing.assert_allclose(o[0], V.mean(axis=0), atol=1e-13)
    # identical values: output is that value
    o, _ = O.attention_rows(rng.standard_normal((3, 8)), K, np.tile(V[:1], (20, 1)), 0.3,
                            [20, 3, 11])
    np.testing.assert_allclose(o, np.tile(V[:1], (3, 1)), atol=1e-14)
    # one dominant key (z larger by >= 50): output is its value
    q = np.zeros((1, 8)); q[0, 0] = 1.0
    Kd = np.zeros((20, 8)); Kd[13, 0] = 60.0
    o, _ = O.attention_rows(q, Kd, V, 1.0, [20])
    np.testing.assert_allclose(o[0], V[13], atol=1e-12)
    # two keys with z = ln 3 and 0: weights 3/4 and 1/4
    Kd = np.zeros((2, 8)); Kd[0, 0] = math.log(3.0)
    o, wts = O.attention_rows(q, Kd, V[:2], 1.0, [2])
    np.testing.assert_allclose(wts[0], [0.75, 0.25], atol=1e-15)
    np.testing.assert_allclose(o[0], 0.75 * V[0] + 0.25 * V[1], atol=1e-15)
    # sign of the exponent / the scale: a negative score must lose
    Kd = np.zeros((2, 8)); Kd[0, 0] = -2.0
    _, wts = O.attention_rows(q, Kd, V[:2], 0.5, [2])
    np.testing.assert_allclose(wts[0], [1 / (1 + math.e), math.e / (1 + math.e)], atol=1e-15)


def test_gqa_heads_of_a_group_share_kv():
    sh = tiny_shape("f32", Hq=6, Hkv=2, d=8, B=4)
    w = synth.custom_workload("t", sh, [11])
    _, pool = make_pool(w)
    q = synth.q_decode(w)
    q[0, 1] = q[0, 0]; q[0, 2] = q[0, 0]        # group 0 all equal
    q[0, 3] = q[0, 0]                           # head of group 1 with the same query
    out = O.paged_decode(pool, synth.to_host_bits(q), w.table_array([0]), w.decode_lens, sh.Hq,
                         sh.scale)
    assert np.array_equal(out[0, 0], out[0, 1]) and np.array_equal(out[0, 0], out[0, 2])
    assert not np.allclose(out[0, 0], out[0, 3])   # other KV head: different keys


# ------------------------------------------------------------------------------------------
# chunking equivalence (a later chunk also attends to the earlier ones, Section 4.3)
# ------------------------------------------------------------------------------------------

def test_chunk_rows_equal_unchunked_prefill_and_decode_is_a_one_token_chunk():
    sh = tiny_shape("bf16")
    L = 19
    w = synth.custom_workload("t", sh, [L], chunks=[(0, L)], extra_blocks=0)
    # make the chunk sequence hold the same logical data as the decode sequence
    ranges = synth.alloc_ranges(w, "cpu")
    k, v = synth.kv_logical(w, 0, 0, L)
    synth.write_pages(w, ranges, 0, 0, L, k, v)
    synth.write_pages(w, ranges, 1, 0, L, k, v)
    pool = O.OraclePool([synth.to_host_bits(r).reshape(-1) for r in ranges], sh.Hkv, sh.d, sh.B,
                        sh.dtype)
    qfull = synth.normal_values(5, synth.TENSOR_Q, 0, 0, L * sh.Hq * sh.d,
                                torch.bfloat16).view(L, sh.Hq, sh.d)
    qb = synth.to_host_bits(qfull)
    full, _ = O.paged_prefill_chunk(pool, qb, w.block_tables[1], 0, L, sh.Hq, sh.scale)
    for p, c in [(0, 5), (5, 9), (14, 5)]:
        part, pairs = O.paged_prefill_chunk(pool, qb[p:p + c], w.block_tables[1], p, c, sh.Hq,
                                            sh.scale)
        assert pairs == p * c + (c * c + c) // 2
        np.testing.assert_allclose(part, full[p:p + c], rtol=0, atol=1e-14)
    # decode(L) == chunk(p = L-1, c = 1)
    dec = O.paged_decode(pool, qb[L - 1:L], w.table_array([0]), [L], sh.Hq, sh.scale)
    np.testing.assert_allclose(dec[0], full[L - 1], rtol=0, atol=1e-14)


def test_merge_of_any_two_way_split_equals_unsplit():
    rng = np.random.default_rng(3)
    q = rng.standard_normal((1, 8)) * 4
    K = rng.standard_normal((40, 8)) * 4
    V = rng.standard_normal((40, 8))
    whole, _ = O.attention_rows(q, K, V, 0.5, [40])
    for cut in [1, 7, 20, 39]:
        parts = []
        for lo, hi in [(0, cut), (cut, 40)]:
            z = 0.5 * (K[lo:hi] @ q[0])
            m = z.max()
            e = np.exp(z - m)
            parts.append((m, e.sum(), e @ V[lo:hi]))
        merged = O.merge_partials(np.array([x[0] for x in parts]),
                                  np.array([x[1] for x in parts]),
                                  np.stack([x[2] for x in parts]))
        np.testing.assert_allclose(merged, whole[0], rtol=0, atol=1e-12)


# ------------------------------------------------------------------------------------------
# garbage immunity, indexing, bytes
# ------------------------------------------------------------------------------------------

def test_nan_in_unused_slots_and_blocks_is_ignored():
    sh = tiny_shape("f32")
    w = synth.custom_workload("t", sh, [5, 10], extra_blocks=4)
    outs = []
    for poison in (True, False):
        ranges = synth.alloc_ranges(w, "cpu", poison=True)
        if not poison:
            for r in ranges:
                r.zero_()
        synth.fill_pool(w, ranges)
        pool = O.OraclePool([synth.to_host_bits(r).reshape(-1) for r in ranges], sh.Hkv, sh.d,
                            sh.B, sh.dtype)
        tab = w.table_array(range(w.S), pad=-1)
        outs.append(O.paged_decode(pool, synth.to_host_bits(synth.q_decode(w)), tab,
                                   w.decode_lens, sh.Hq, sh.scale))
    assert np.isfinite(outs[0]).all() and np.array_equal(outs[0], outs[1])


def test_resolve_block_and_slots_brute_force():
    rb = [5, 1, 7, 3]
    flat = [(r, i) for r, n in enumerate(rb) for i in range(n)]     # enumerate every block
    for blk, expect in enumerate(flat):
        assert O.resolve_block(rb, blk) == expect
        assert O.block_byte_offset(rb, blk, 4096) == (expect[0], expect[1] * 4096)
    for bad in (-1, 16, 100):
        with pytest.raises(IndexError):
            O.resolve_block(rb, bad)
    row = [9, 4, 11]
    assert [O.token_slot(row, t, 4) for t in (0, 3, 4, 11)] == [(9, 0), (9, 3), (4, 0), (11, 3)]
    assert O.usable_blocks(65536 * 3 + 100, 65536) == 3 and O.usable_blocks(65535, 65536) == 0


def test_kv_bytes_match_papers_per_token_figure():
    # Section 2.2: 192 KB per token for a 48-layer model with 8 KV heads x 128 dims in bf16.
    pool = O.OraclePool([np.zeros(0, np.uint16)], Hkv=8, d=128, B=16, dtype="bf16")
    per_token_per_layer = pool.block_bytes // pool.B
    assert per_token_per_layer == 4096
    assert per_token_per_layer * 48 == 192 * 1024
    assert synth.SHAPE_8B.block_bytes == 65536 and synth.SHAPE_TINY.block_bytes == 16384


@pytest.mark.parametrize("B,lens", [(4, [6, 3]), (16, [40, 16, 1]), (64, [150, 64, 65, 3])])
def test_kv_append_slot_map_and_layout(B, lens):
    sh = tiny_shape("f32", Hq=2, Hkv=2, d=4, B=B)
    w = synth.custom_workload("t", sh, lens, extra_blocks=2, range_fracs=(0.5, 0.5))
    ranges = synth.alloc_ranges(w, "cpu")
    pool = O.OraclePool([synth.to_host_bits(r).reshape(-1) for r in ranges], sh.Hkv, sh.d, sh.B,
                        sh.dtype)
    seqs, poss, ks, vs = [], [], [], []
    for s in range(len(lens)):
        L = int(w.decode_lens[s])
        k, v = synth.kv_logical(w, s, 0, L)
        ks.append(k); vs.append(v)
        seqs += [s] * L; poss += list(range(L))
    tab = w.table_array(range(len(lens)))
    slots = O.kv_append(pool, torch.cat(ks).numpy(), torch.cat(vs).numpy(), seqs, poss, tab)
    # expected slot map by direct enumeration
    firsts = np.concatenate([[0], np.cumsum(w.range_blocks)])
    for (r, local, slot), s, t in zip(slots, seqs, poss):
        blk = int(w.block_tables[s][t // sh.B])
        assert firsts[r] + local == blk and slot == t % sh.B
    # the appended pages read back as the logical K/V, and agree with the generator's own writer
    for s in range(len(lens)):
        for kvh in range(sh.Hkv):
            K, V = O.gather_kv(pool, tab[s], int(w.decode_lens[s]), kvh)
            assert np.array_equal(K, ks[s][:, kvh].double().numpy())
            assert np.array_equal(V, vs[s][:, kvh].double().numpy())
    ranges2 = synth.alloc_ranges(w, "cpu")
    synth.fill_pool(w, ranges2)
    for a, b in zip(ranges, ranges2):
        assert np.array_equal(synth.to_host_bits(a), synth.to_host_bits(b), equal_nan=True)


def test_page_of_64_tokens_is_four_pages_of_16_tokens_in_a_row():
    # the layout inside a block (this library's ABI): tiles of 16 tokens.  With one KV head a block of
    # 64 tokens must be byte-identical to blocks 0..3 of a pool of 16-token blocks holding the same
    # tokens; two offsets worked out by hand pin the page and tile strides with two KV heads.
    rng = np.random.default_rng(5)
    d, L = 8, 150
    k = rng.standard_normal((L, 1, d)).astype(np.float32)
    v = rng.standard_normal((L, 1, d)).astype(np.float32)
    seqs, poss = [0] * L, list(range(L))
    p64 = O.OraclePool([np.zeros(3 * 2 * 64 * d, np.float32)], 1, d, 64, "f32")
    p16 = O.OraclePool([np.zeros(12 * 2 * 16 * d, np.float32)], 1, d, 16, "f32")
    O.kv_append(p64, k, v, seqs, poss, np.array([[0, 1, 2]]))
    O.kv_append(p16, k, v, seqs, poss, np.arange(12)[None, :])
    assert np.array_equal(p64.ranges[0], p16.ranges[0])
    K, V = O.gather_kv(p64, [0, 1, 2], L, 0)
    assert np.array_equal(K, k[:, 0].astype(np.float64)) and np.array_equal(V, v[:, 0].astype(np.float64))
    # two KV heads, d = 8: block 1, head 1 starts at (1*2+1) * 2*64*8 = 3072; slot 37 is slot 5 of tile 2,
    # tiles are 2*16*8 = 256 elements: K[37][3] at 3072 + 512 + 5*8 + 3, V[37][3] at 3072 + 512 + 128 + 3*16 + 5
    p2 = O.OraclePool([np.zeros(2 * 2 * 2 * 64 * d, np.float32)], 2, d, 64, "f32")
    assert O.k_elem_offset(p2, 1, 1, 37) + 3 == 3627
    assert O.v_elem_offset(p2, 1, 1, 37, 3) == 3765
    # blocks of at most 16 tokens are one tile: K rows, then V columns
    p4 = O.OraclePool([np.zeros(2 * 2 * 4 * d, np.float32)], 2, d, 4, "f32")
    assert O.k_elem_offset(p4, 0, 1, 3) == 64 + 24 and O.v_elem_offset(p4, 0, 1, 3, 2) == 64 + 32 + 2 * 4 + 3


# ------------------------------------------------------------------------------------------
# the generator itself
# ------------------------------------------------------------------------------------------

def test_hash_matches_uint64_reference_and_values_are_standard_normal():
    idx = torch.arange(0, 200000, dtype=torch.int64) * 7919 + 3
    key = synth.stream_key(1002, synth.TENSOR_K, 5)
    a = synth.hash_u16(key, idx).numpy()
    b = synth.hash_u16_numpy(key, idx.numpy())
    assert np.array_equal(a, b)
    assert a.min() >= 0 and a.max() < 65536
    x = synth.normal_values(1, synth.TENSOR_V, 0, 0, 400000, torch.float32).double().numpy()
    assert abs(x.mean()) < 0.01 and abs(x.std() - 1.0) < 0.01
    assert abs(np.mean(x ** 4) - 3.0) < 0.1
    # keyed by logical coordinates: a sub-range reproduces the same values
    y = synth.normal_values(1, synth.TENSOR_V, 0, 1000, 50, torch.float32).double().numpy()
    assert np.array_equal(y, x[1000:1050])


def test_config_shapes():
    w1 = synth.config(1)
    assert list(w1.decode_lens) == [17, 64, 200, 513] and w1.num_blocks == 64
    assert sum(len(b) for b in w1.block_tables) == 52 and w1.decode_kv_tokens == 794
    w2 = synth.config(2)
    assert w2.S == 64 and w2.decode_lens.min() >= 512 and w2.decode_lens.max() <= 4096
    w3 = synth.config(3)
    assert w3.S == 512 and len(w3.range_blocks) == 3 and w3.phase_resident[-1] == 512
    used = np.concatenate(w3.block_tables)
    assert len(np.unique(used)) == len(used) == w3.num_blocks
    r, _ = synth.range_of_blocks(w3.range_blocks, used.astype(np.int64))
    assert set(np.unique(r)) == {0, 1, 2}
    # sequences admitted in phase 0 only use range 0
    first = np.concatenate(w3.block_tables[:w3.phase_resident[0]])
    assert first.max() < w3.range_blocks[0]
    w4 = synth.config(4)
    assert w4.n_chunks == 8 and all(c == 512 and 0 <= p <= 3584 for p, c in w4.chunks)
    assert w4.prefill_pairs == sum(p * 512 + 512 * 513 // 2 for p, _ in w4.chunks)
    w5 = synth.config(5)
    assert w5.num_blocks * w5.shape.block_bytes >= 149 * 10**9 and len(w5.range_blocks) == 5
    used = np.concatenate(w5.block_tables)
    assert len(np.unique(used)) == len(used)


# ------------------------------------------------------------------------------------------
# FP8 (E4M3) pages: the lossy KV representation Section 7 names as the alternative under memory
# pressure.  The oracle widens the page bytes exactly; these pins fix what "exactly" means.
# ------------------------------------------------------------------------------------------

def test_fp8_e4m3_codes_widen_to_the_values_the_format_defines():
    codes = np.arange(256, dtype=np.uint8)
    got = O.widen(codes, "fp8")
    # (a) values typed in by hand from the format's definition (1 sign, 4 exponent bits, bias 7, 3
    #     mantissa bits, subnormals at exponent 0, no infinities, S.1111.111 is the only NaN)
    by_hand = {0x00: 0.0, 0x01: 2.0 ** -9, 0x02: 2.0 ** -8, 0x07: 7 * 2.0 ** -9, 0x08: 2.0 ** -6, 0x09: 1.125 * 2.0 ** -6,
               0x30: 0.5, 0x38: 1.0, 0x39: 1.125, 0x3F: 1.875, 0x40: 2.0, 0x44: 3.0, 0x48: 4.0, 0x77: 240.0, 0x78: 256.0,
               0x7E: 448.0, 0x81: -2.0 ** -9, 0xB8: -1.0, 0xC0: -2.0, 0xFE: -448.0}
    for c, v in by_hand.items():
        assert got[c] == v, (hex(c), got[c], v)
    assert np.isnan(got[0x7F]) and np.isnan(got[0xFF]) and np.isfinite(np.delete(got, [0x7F, 0xFF])).all()
    assert got[0x80] == 0.0 and np.signbit(got[0x80]) and not np.signbit(got[0x00])
    # (b) structure: the 127 non-negative finite codes increase strictly; inside a binade the step is
    #     constant and doubles from one binade to the next; the negative half mirrors the positive one
    pos = got[:0x7F]
    assert (np.diff(pos) > 0).all()
    steps = np.diff(pos)
    assert (steps[:15] == 2.0 ** -9).all()                              # subnormals and the first binade
    for e in range(2, 16):
        assert (steps[8 * e:8 * e + 7] == 2.0 ** (e - 10)).all()
    assert np.array_equal(got[0x80:0xFF], -pos)
    # (c) a library's conversion of the same codes (torch's float8_e4m3fn), all 256
    lib = torch.from_numpy(codes.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.array_equal(got, lib, equal_nan=True)


def test_fp8_pages_decode_and_prefill_match_dense_brute_force():
    # K/V pages hold E4M3 codes, queries are bf16; the dense reference decodes the codes with the
    # library conversion and never sees pages, tiles or block tables
    sh = synth.LayerShape(Hq=4, Hkv=2, d=8, B=4, dtype="fp8")
    w = synth.custom_workload("fp8-tiny", sh, [1, 3, 4, 9], chunks=[(2, 5)], extra_blocks=2, range_fracs=(0.5, 0.5))
    ranges, pool = make_pool(w)
    assert pool.elt == 1 and pool.q_dtype == "bf16" and pool.block_bytes == 2 * 2 * 4 * 8
    q = synth.q_decode(w)
    got = O.paged_decode(pool, synth.to_host_bits(q), w.table_array(range(w.S)), w.decode_lens, sh.Hq, sh.scale)

    def dense_kv(seq, L):
        k, v = synth.kv_logical(w, seq, 0, L)
        assert k.dtype == torch.uint8
        return (k.view(torch.float8_e4m3fn).to(torch.float64).numpy(), v.view(torch.float8_e4m3fn).to(torch.float64).numpy())

    scale = float(np.float32(sh.scale))
    for s in range(w.S):
        L = int(w.decode_lens[s])
        k, v = dense_kv(s, L)
        for h in range(sh.Hq):
            kvh = h // sh.G
            ref = dense_attention([q[s, h].double().tolist()], k[:, kvh].tolist(), v[:, kvh].tolist(), scale,
                                  [[True] * L])
            assert np.allclose(got[s, h], ref[0], rtol=0, atol=1e-12)
    p, c = w.chunks[0]
    qc = synth.q_chunk(w, 0)
    gotc, pairs = O.paged_prefill_chunk(pool, synth.to_host_bits(qc), w.block_tables[w.S], p, c, sh.Hq, sh.scale)
    assert pairs == p * c + (c * c + c) // 2
    k, v = dense_kv(w.S, p + c)
    for h in range(sh.Hq):
        kvh = h // sh.G
        mask = [[t <= p + r for t in range(p + c)] for r in range(c)]
        ref = dense_attention(qc[:, h].double().tolist(), k[:, kvh].tolist(), v[:, kvh].tolist(), scale, mask)
        assert np.allclose(gotc[:, h], np.asarray(ref), rtol=0, atol=1e-12)
    # unused slots hold the NaN code and never reach an output
    assert np.isfinite(got).all() and np.isfinite(gotc).all()
    assert any((synth.to_host_bits(r) == 0x7F).any() for r in ranges)


def test_fp8_values_of_the_generator_are_the_nearest_e4m3_codes():
    # the input generator rounds its N(0,1) quantiles to E4M3 with torch; the oracle's widening of those
    # codes must land within half a step of the quantile (round to nearest), so the two agree on the format
    tab = synth.normal_table(synth.FP8)
    from scipy.special import ndtri
    want = ndtri((np.arange(65536, dtype=np.float64) + 0.5) / 65536.0)
    got = O.widen(tab.numpy(), "fp8")
    step = np.maximum(2.0 ** (np.floor(np.log2(np.maximum(np.abs(want), 2.0 ** -6))) - 3), 2.0 ** -9)
    # (the generator goes through fp32 first, which can turn a near tie into a tie: half a step plus an fp32 ulp)
    assert (np.abs(got - want) <= step / 2 * (1 + 2.0 ** -20)).all()
    assert abs(got.mean()) < 1e-3 and abs(got.std() - 1.0) < 2e-2
