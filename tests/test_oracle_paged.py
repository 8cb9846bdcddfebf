"""Pins of the paged oracle.  Paging is a pure relocation of 128-token blocks, so the paged cache
is pinned against the contiguous IntCache (itself pinned in test_oracle_quant / _attention):
same bytes per block wherever the block lives, same attention output whatever the page order,
ragged lengths equal to independent single-sequence caches."""
import numpy as np
import pytest

from oracle import bitdecode_oracle as O
from paper_2503_18773_amd import workloads as W


def _kv(seed, H, L):
    w = W.scaled(W.CONFIGS["cfg1"], batch=1, n_q_heads=H, n_kv_heads=H, context=max(L, 1), seed=seed)
    K, V = W.make_kv(w)
    return K[0, :, :L], V[0, :, :L]


def _table(rng, B, max_pages, P):
    """Distinct pages for every (sequence, block), scattered over the pool."""
    perm = rng.permutation(P)[:B * max_pages]
    return perm.reshape(B, max_pages).astype(np.int32)


@pytest.mark.parametrize("bits", [4, 2])
def test_identity_table_holds_the_contiguous_bytes(bits):
    B, H, L = 2, 2, 3 * 128 + 17
    c = O.IntCache(B, H, bits, 4 * 128)
    KV = [_kv(10 + b, H, L) for b in range(B)]
    c.quant_pack_kv(np.stack([k for k, _ in KV]), np.stack([v for _, v in KV]))
    table = np.arange(B * 4, dtype=np.int32).reshape(B, 4)          # page = b * 4 + n
    p = O.PagedIntCache(B, H, bits, B * 4, 4, table)
    for b in range(B):
        p.quant_pack_kv(b, *KV[b])
    for name in ("k_codes", "v_codes", "k_params", "v_params"):
        got = getattr(p, name).reshape(B, 4, H, *getattr(p, name).shape[2:]).swapaxes(1, 2)
        assert np.array_equal(got, getattr(c, name)), name
    assert np.array_equal(p.k_res, c.k_res) and np.array_equal(p.v_res, c.v_res)
    assert list(p.seq_lens) == [L, L]


@pytest.mark.parametrize("bits,group", [(4, 128), (2, 128), (4, 32), (2, 64)])
def test_ragged_scattered_pages_equal_independent_caches(bits, group):
    rng = np.random.default_rng(5)
    B, H, Hq = 4, 2, 4
    lens = [300, 0, 128, 517]
    table = _table(rng, B, 6, 40)
    p = O.PagedIntCache(B, H, bits, 40, 6, table, group=group)
    singles = []
    for b, L in enumerate(lens):
        K, V = _kv(20 + b, H, L)
        p.quant_pack_kv(b, K, V)
        c = O.IntCache(1, H, bits, 6 * 128, group=group)
        c.quant_pack_kv(K[None], V[None])
        singles.append(c)
    # three decode steps: sequence 2 (128 tokens) stays aligned, sequence 3 crosses nothing, then
    # run sequence 0 over a flush by appending until 384
    q = np.random.default_rng(6).standard_normal((B, Hq, 128)).astype(np.float16)
    for step in range(90):
        kn = rng.standard_normal((B, H, 128)).astype(np.float16)
        vn = rng.standard_normal((B, H, 128)).astype(np.float16)
        p.append_kv(kn, vn)
        for b in range(B):
            singles[b].append_kv(kn[b:b + 1], vn[b:b + 1])
    assert [int(x) for x in p.seq_lens] == [L + 90 for L in lens]
    out = O.decode_attn(p, q, 0.09)
    for b in range(B):
        ref = O.decode_attn(singles[b], q[b:b + 1], 0.09)
        assert np.array_equal(out[b], ref[0]), b
        # every block of the sequence holds the single cache's bytes, in its own page
        for n in range(singles[b].packed_len // 128):
            pg = table[b, n]
            assert np.array_equal(p.k_codes[pg], singles[b].k_codes[0, :, n])
            assert np.array_equal(p.v_codes[pg], singles[b].v_codes[0, :, n])
            assert np.array_equal(p.k_params[pg], singles[b].k_params[0, :, n])
            assert np.array_equal(p.v_params[pg], singles[b].v_params[0, :, n])
    # pages no sequence reached stay untouched
    used = {int(table[b, n]) for b in range(B) for n in range(int(p.seq_lens[b]) // 128)}
    for pg in set(range(40)) - used:
        assert not p.k_codes[pg].any() and not p.v_params[pg].any()


def test_empty_sequence_gives_zero_and_errors_are_raised():
    table = np.array([[0, 1], [7, 2]], np.int32)
    p = O.PagedIntCache(2, 1, 4, 4, 2, table)
    K, V = _kv(3, 1, 127)
    p.quant_pack_kv(0, K, V)
    q = np.ones((2, 2, 128), np.float16)
    out = O.decode_attn(p, q, 0.1)
    assert not out[1].any() and np.isfinite(out[0]).all()
    p.quant_pack_kv(1, K, V)
    one = np.ones((2, 1, 128), np.float16)
    with pytest.raises(IndexError):            # sequence 1's first page (7) is outside the pool of 4
        p.append_kv(one, one)
    assert list(p.seq_lens) == [128, 127]      # sequence 0 had been served before the error
    p2 = O.PagedIntCache(1, 1, 4, 4, 2, np.array([[0, 1]], np.int32))
    K, V = _kv(4, 1, 255)
    p2.quant_pack_kv(0, K, V)
    p2.append_kv(one[:1], one[:1])
    K3, V3 = _kv(4, 1, 127)
    p2.quant_pack_kv(0, np.concatenate([K, K3[:, :1]], 1)[:, :256], np.concatenate([V, V3[:, :1]], 1)[:, :256])
    for _ in range(127):
        p2.append_kv(one[:1], one[:1])
    with pytest.raises(OverflowError):         # a third block has no table entry
        p2.append_kv(one[:1], one[:1])


def _kv_bf16(seed, H, L):
    w = W.scaled(W.CONFIGS["cfg4"], batch=1, n_q_heads=H, n_kv_heads=H, context=max(L, 1), seed=seed)
    K, V = W.make_kv(w)
    return K[0, :, :L], V[0, :, :L]


def test_paged_mx_is_a_relocation_of_the_contiguous_cache():
    """Ragged MXFP4 sequences on scattered pages hold, block for block, the bytes of independent
    contiguous caches, after prefill and after appends; attention is identical."""
    rng = np.random.default_rng(9)
    B, H, Hq = 3, 2, 4
    lens = [300, 0, 129]
    table = _table(rng, B, 4, 20)
    p = O.PagedMxCache(B, H, 20, 4, table)
    singles = []
    for b, L in enumerate(lens):
        K, V = _kv_bf16(30 + b, H, L)
        p.quant_pack_kv(b, K, V)
        c = O.MxCache(1, H, 512)
        c.quant_pack_kv(K[None], V[None])
        singles.append(c)
    for step in range(5):
        kn = W.round_to_bf16(rng.standard_normal((B, H, 128)).astype(np.float32))
        vn = W.round_to_bf16(rng.standard_normal((B, H, 128)).astype(np.float32))
        p.append_kv(kn, vn)
        for b in range(B):
            singles[b].append_kv(kn[b:b + 1], vn[b:b + 1])
    assert [int(x) for x in p.seq_lens] == [L + 5 for L in lens]
    q = W.round_to_bf16(np.random.default_rng(6).standard_normal((B, Hq, 128)).astype(np.float32))
    out = O.decode_attn(p, q, 0.09)
    for b in range(B):
        c = singles[b]
        assert np.array_equal(out[b], O.decode_attn(c, q[b:b + 1], 0.09)[0]), b
        for n in range(-(-c.length // 128)):
            pg = table[b, n]
            m = min(128, c.length - 128 * n)
            assert np.array_equal(p.k_codes[pg][:, :m], c.k_codes[0, :, 128 * n:128 * n + m])
            assert np.array_equal(p.k_scales[pg][:, :m], c.k_scales[0, :, 128 * n:128 * n + m])
            assert np.array_equal(p.v_scales[pg][:, :m], c.v_scales[0, :, 128 * n:128 * n + m])
            assert np.array_equal(p.v_codes[pg], c.v_codes[0, :, n])


def test_lazy_flush_of_a_ragged_batch_is_the_per_sequence_lazy_flush():
    """append_kv(flush=False) + attention + flush_if_full(): every sequence on its own behaves as the contiguous
    cache's lazy mode (pinned in test_oracle_quant), only the sequences whose residual reached 128 tokens attend
    fp16 rows, and the pool afterwards is the one eager steps leave."""
    H, D = 2, 128
    lens = [128 + 126, 90, 127, 3 * 128 + 127]
    table = np.array([[3, 9, 0, 14], [5, 1, 13, 8], [2, 11, 6, 15], [7, 4, 12, 10]], np.int32)
    lazy = O.PagedIntCache(4, H, 4, 16, 4, table)
    eager = O.PagedIntCache(4, H, 4, 16, 4, table)
    singles = []
    for b, L in enumerate(lens):
        w = W.scaled(W.CONFIGS["cfg1"], batch=1, n_q_heads=4, n_kv_heads=H, context=L, seed=60 + b)
        K, V = W.make_kv(w)
        lazy.quant_pack_kv(b, K[0], V[0])
        eager.quant_pack_kv(b, K[0], V[0])
        c = O.IntCache(1, H, 4, 512)
        c.quant_pack_kv(K, V)
        singles.append(c)
    wq = W.scaled(W.CONFIGS["cfg1"], batch=4, n_q_heads=4, n_kv_heads=H, context=8, seed=70)
    for step in range(3):       # sequences 2 and 3 fill at step 0, sequence 0 at step 1
        kn, vn = W.make_new_kv(wq, step)
        q = W.make_q(wq, step)
        lazy.append_kv(kn, vn, flush=False)
        assert list(lazy.unflushed) == [[False, False, True, True], [True, False, False, False], [False] * 4][step]
        out = O.decode_attn(lazy, q, 0.09)
        lazy.flush_if_full()
        eager.append_kv(kn, vn)
        out_eager = O.decode_attn(eager, q, 0.09)
        for b in range(4):
            singles[b].append_kv(kn[b:b + 1], vn[b:b + 1], flush=False)
            ref = O.decode_attn(singles[b], q[b:b + 1], 0.09)
            singles[b].flush_if_full()
            assert np.array_equal(out[b], ref[0]), (step, b)
            filled = (lens[b] + step) % 128 == 127
            assert np.array_equal(out[b], out_eager[b]) != filled, (step, b)   # only a filling step differs
        for name in ("k_codes", "v_codes", "k_params", "v_params", "seq_lens"):
            assert np.array_equal(getattr(lazy, name), getattr(eager, name)), (step, name)
    assert not lazy.unflushed.any()
