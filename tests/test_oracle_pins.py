"""Pins for the fp64 CPU oracle.

The paper prints no worked numeric attention output, so the oracle is held to what
the mathematics fixes: a brute force on tiny inputs, closed forms, invariants, and a
library routine on a special case.  Each pin names the mistake it is there to catch.
All of this runs on the CPU.
"""
import math

import numpy as np
import pytest
import torch

from oracle import brute, reference
from paper_2410_18038_amd import workloads as wl
from tests.helpers import logical_kv, oracle_out, request_q, request_rows

F16, BF16 = wl.F16, wl.BF16


def small_batch(seed=7, dtype=F16, hq=4, hkv=2, d=8, block_size=0, prefill=((5, 9), (3, 3)),
                decodes=(1, 6, 11), poison=None):
    return wl.make_batch("small", prefill=list(prefill), decode_kv_lens=list(decodes), n_q_heads=hq,
                         n_kv_heads=hkv, head_dim=d, dtype=dtype, seed=seed, block_size=block_size,
                         poison=poison)


# -- widening ---------------------------------------------------------------- #
def test_widening_matches_numpy_and_torch_for_every_bit_pattern():
    """A wrong exponent bias, a lost subnormal or a sign slip shows here."""
    patterns = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    want16 = patterns.view(np.float16).astype(np.float64)
    want_bf = torch.from_numpy(patterns.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    got16 = np.array([reference.widen(F16, int(b)) for b in patterns])
    got_bf = np.array([reference.widen(BF16, int(b)) for b in patterns])
    assert np.array_equal(np.isnan(got16), np.isnan(want16))
    assert np.array_equal(np.isnan(got_bf), np.isnan(want_bf))
    ok16, ok_bf = ~np.isnan(want16), ~np.isnan(want_bf)
    assert np.array_equal(got16[ok16], want16[ok16])
    assert np.array_equal(got_bf[ok_bf], want_bf[ok_bf])


# -- p1: brute force ---------------------------------------------------------- #
@pytest.mark.parametrize("dtype", [F16, BF16])
@pytest.mark.parametrize("hq,hkv", [(2, 2), (2, 1), (6, 2)])
@pytest.mark.parametrize("block_size", [0, 4])
def test_brute_force_on_tiny_batches(dtype, hq, hkv, block_size):
    """Everything at small scale: mask, head mapping, layout, normalisation."""
    b = small_batch(seed=11 + hq, dtype=dtype, hq=hq, hkv=hkv, d=4, block_size=block_size,
                    prefill=((3, 5), (2, 2)), decodes=(5, 1, 7))
    got = oracle_out(b)
    for req in range(b.n_prefill + b.n_decode):
        k, v = logical_kv(b, req)
        q = request_q(b, req)
        want = np.array(brute.attention_one_request(q.tolist(), k.tolist(), v.tolist(),
                                                    b.softmax_scale, hq, hkv))
        np.testing.assert_allclose(got[request_rows(b, req)], want, rtol=1e-12, atol=1e-13)


# -- p2: normalisation --------------------------------------------------------- #
def test_constant_v_returns_that_row():
    """A missing division by the weight sum, or a sum over the wrong range, breaks this."""
    b = small_batch(dtype=F16)
    v0 = torch.linspace(-1.0, 2.5, b.head_dim).to(torch.float16)
    b.v_cache[:] = v0
    got = oracle_out(b)
    want = np.broadcast_to(v0.double().numpy(), got.shape)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-14)


# -- p3: a single key ---------------------------------------------------------- #
def test_single_key_returns_its_v_row():
    """Boundary j = 0: first row of a chunk with no prefix, and a decode of context 1."""
    b = small_batch(prefill=((4, 4),), decodes=(1, 1), hq=4, hkv=2)
    got = oracle_out(b)
    group = b.n_q_heads // b.n_kv_heads
    for req in (0, 1, 2):
        _, v = logical_kv(b, req)
        row = request_rows(b, req)[0]
        for h in range(b.n_q_heads):
            np.testing.assert_array_equal(got[row, h], v[0, h // group])


# -- p4: decode is the last row of the matching prefill -------------------------- #
@pytest.mark.parametrize("block_size", [0, 4])
def test_decode_equals_last_row_of_equivalent_prefill(block_size):
    """Pins the causal offset: a decode sees the whole context, a chunk row sees up to itself."""
    length = 13
    full = wl.make_batch("full", prefill=[(length, length)], decode_kv_lens=[], n_q_heads=4,
                         n_kv_heads=2, head_dim=8, dtype=F16, seed=3, block_size=block_size)
    dec = wl.make_batch("dec", prefill=[], decode_kv_lens=[length], n_q_heads=4, n_kv_heads=2,
                        head_dim=8, dtype=F16, seed=4, block_size=0)
    k, v = logical_kv(full, 0)
    dec.k_cache[0, :length] = torch.from_numpy(k).to(torch.float16)
    dec.v_cache[0, :length] = torch.from_numpy(v).to(torch.float16)
    dec.decode_q[0] = full.prefill_q[length - 1]
    np.testing.assert_array_equal(oracle_out(dec)[0], oracle_out(full)[length - 1])
    # and a middle row equals a decode over the truncated context
    mid = 6
    dec2 = wl.make_batch("dec2", prefill=[], decode_kv_lens=[mid + 1], n_q_heads=4, n_kv_heads=2,
                         head_dim=8, dtype=F16, seed=5)
    dec2.k_cache[0, :mid + 1] = torch.from_numpy(k[:mid + 1]).to(torch.float16)
    dec2.v_cache[0, :mid + 1] = torch.from_numpy(v[:mid + 1]).to(torch.float16)
    dec2.decode_q[0] = full.prefill_q[mid]
    np.testing.assert_array_equal(oracle_out(dec2)[0], oracle_out(full)[mid])


# -- p5: layouts agree bit for bit ----------------------------------------------- #
@pytest.mark.parametrize("dtype", [F16, BF16])
def test_paged_and_contiguous_layouts_agree_exactly(dtype):
    """Block-table indexing, the partial last block, the per-sequence stride."""
    b = small_batch(dtype=dtype, d=16, prefill=((7, 21),), decodes=(1, 16, 17, 33), poison=float("nan"))
    ref = oracle_out(b)
    for bs in (1, 4, 16):
        paged = wl.regroup(b, bs, seed=99 + bs, poison=float("nan"))
        assert paged.block_table is not None and paged.block_size == bs
        np.testing.assert_array_equal(oracle_out(paged), ref)
        back = wl.regroup(paged, 0, seed=1, poison=float("nan"))
        np.testing.assert_array_equal(oracle_out(back), ref)


@pytest.mark.parametrize("dtype", [wl.F16, wl.BF16])
def test_head_major_and_token_major_caches_agree_exactly(dtype):
    """The head-major cache is the token-major one with its two middle axes swapped (here by a
    numpy-style transpose, not by the oracle's offset rule): identical values, identical output.
    Three K/V heads against 33 or 4 slots: a swapped stride reads another head or a poisoned slot."""
    b = small_batch(dtype=dtype, hq=6, hkv=3, d=16, prefill=((7, 21),), decodes=(1, 16, 17, 33),
                    poison=float("nan"))
    ref = oracle_out(b)
    hm = wl.to_head_major(b)
    assert hm.head_major and hm.k_cache.shape[1] == 3 and hm.k_cache.shape[2] == b.k_cache.shape[1]
    np.testing.assert_array_equal(oracle_out(hm), ref)
    for bs in (1, 4, 16):
        paged = wl.to_head_major(wl.regroup(b, bs, seed=7 + bs, poison=float("nan")))
        assert paged.k_cache.shape[1:3] == (3, bs)
        np.testing.assert_array_equal(oracle_out(paged), ref)


# -- p6: closed form with zero queries -------------------------------------------- #
def test_zero_query_gives_running_mean_and_exact_causal_boundary():
    """Q = 0 makes every weight equal; with V[j] = j the answer is pos / 2.

    Seeing one key too many or too few moves the result by exactly one half.
    """
    b = small_batch(prefill=((6, 20), (4, 4)), decodes=(1, 9, 30), hq=4, hkv=2, d=8)
    b.prefill_q.zero_()
    b.decode_q.zero_()
    ramp = torch.arange(b.v_cache.shape[1], dtype=torch.float16)
    b.v_cache[:] = ramp[None, :, None, None]
    got = oracle_out(b)
    for req in range(b.n_prefill + b.n_decode):
        _, q_len, kv_len, _ = (int(x) for x in b.seq_meta[req])
        for i, row in enumerate(request_rows(b, req)):
            pos = kv_len - q_len + i
            np.testing.assert_allclose(got[row], pos / 2.0, rtol=1e-15, atol=1e-15)


# -- p7: head grouping ------------------------------------------------------------- #
@pytest.mark.parametrize("hq,hkv", [(8, 2), (8, 8), (8, 1), (6, 3)])
def test_query_head_reads_its_group_kv_head(hq, hkv):
    """V constant per K/V head: query head h must return h // (Hq / Hkv)."""
    b = small_batch(hq=hq, hkv=hkv, d=4)
    marks = torch.arange(hkv, dtype=torch.float16)
    b.v_cache[:] = marks[None, None, :, None]
    got = oracle_out(b)
    for h in range(hq):
        np.testing.assert_allclose(got[:, h, :], h // (hq // hkv), rtol=0, atol=1e-14)


# -- p8: log-sum-exp merge identity ------------------------------------------------- #
def test_split_and_merge_identity():
    """Attention over A u B equals the log-sum-exp weighted merge of attention over A and over B.

    This is the identity the GPU's split-KV combine relies on; it also pins the sign
    inside the exponential (flip it and the merge weights invert).
    """
    length, cut = 37, 14
    b = wl.make_batch("m", prefill=[], decode_kv_lens=[length], n_q_heads=4, n_kv_heads=2, head_dim=8,
                      dtype=F16, seed=21)
    whole = oracle_out(b)[0]
    k, v = logical_kv(b, 0)
    q = request_q(b, 0)[0]
    group = 2

    def part(lo, hi):
        sub = wl.make_batch("p", prefill=[], decode_kv_lens=[hi - lo], n_q_heads=4, n_kv_heads=2,
                            head_dim=8, dtype=F16, seed=22)
        sub.k_cache[0, :hi - lo] = torch.from_numpy(k[lo:hi]).to(torch.float16)
        sub.v_cache[0, :hi - lo] = torch.from_numpy(v[lo:hi]).to(torch.float16)
        sub.decode_q[0] = b.decode_q[0]
        out = oracle_out(sub)[0]
        lse = np.array([np.log(np.sum(np.exp(b.softmax_scale * (k[lo:hi, h // group] @ q[h]))))
                        for h in range(4)])
        return out, lse

    out_a, lse_a = part(0, cut)
    out_b, lse_b = part(cut, length)
    top = np.maximum(lse_a, lse_b)
    wa, wb = np.exp(lse_a - top), np.exp(lse_b - top)
    merged = (out_a * wa[:, None] + out_b * wb[:, None]) / (wa + wb)[:, None]
    np.testing.assert_allclose(merged, whole, rtol=1e-12, atol=1e-13)


# -- p9: invariances ------------------------------------------------------------------ #
def test_score_shift_and_key_permutation_leave_the_output_unchanged():
    """A constant added to every score of a row cancels; the order of visible keys is irrelevant."""
    length = 29
    base = wl.make_batch("b", prefill=[], decode_kv_lens=[length], n_q_heads=2, n_kv_heads=1, head_dim=8,
                         dtype=F16, seed=31)
    ref = oracle_out(base)[0]
    # one extra pair of channels: q gets (big, 0), every key gets (big, 0) -> all scores + big^2*scale
    wide = wl.make_batch("w", prefill=[], decode_kv_lens=[length], n_q_heads=2, n_kv_heads=1, head_dim=10,
                         dtype=F16, seed=32, softmax_scale=base.softmax_scale)
    wide.decode_q[:, :, :8] = base.decode_q
    wide.k_cache[:, :, :, :8] = base.k_cache
    wide.v_cache[:, :, :, :8] = base.v_cache
    wide.decode_q[:, :, 8:] = torch.tensor([16.0, 0.0], dtype=torch.float16)
    wide.k_cache[:, :, :, 8:] = torch.tensor([16.0, 0.0], dtype=torch.float16)
    np.testing.assert_allclose(oracle_out(wide)[0][:, :8], ref, rtol=1e-12, atol=1e-13)
    # permute the visible (K, V) pairs of the decode
    perm = np.random.Generator(np.random.PCG64(5)).permutation(length)
    shuf = wl.make_batch("s", prefill=[], decode_kv_lens=[length], n_q_heads=2, n_kv_heads=1, head_dim=8,
                         dtype=F16, seed=31)
    shuf.k_cache[0, :length] = base.k_cache[0, perm]
    shuf.v_cache[0, :length] = base.v_cache[0, perm]
    np.testing.assert_allclose(oracle_out(shuf)[0], ref, rtol=1e-12, atol=1e-13)


# -- p10: masking is by index, not by value -------------------------------------------- #
@pytest.mark.parametrize("block_size", [0, 4])
@pytest.mark.parametrize("poison", [float("nan"), 60000.0, float("-inf")])
def test_poison_outside_the_visible_range_changes_nothing(block_size, poison):
    clean = small_batch(block_size=block_size, prefill=((5, 9), (3, 3)), decodes=(1, 6, 11), poison=None)
    dirty = small_batch(block_size=block_size, prefill=((5, 9), (3, 3)), decodes=(1, 6, 11), poison=poison)
    got = oracle_out(dirty)
    assert np.isfinite(got).all()
    np.testing.assert_array_equal(got, oracle_out(clean))


def test_future_keys_inside_the_chunk_are_ignored():
    """Poison the K/V of later chunk tokens: earlier rows must not move."""
    b = small_batch(prefill=((6, 10),), decodes=())
    ref = oracle_out(b)
    b.k_cache[0, 9] = float("nan")
    b.v_cache[0, 9] = float("nan")
    got = oracle_out(b)
    np.testing.assert_array_equal(got[:5], ref[:5])
    assert np.isnan(got[5]).all()


# -- p11: a library routine on the same problem ------------------------------------------ #
@pytest.mark.parametrize("dtype,hq,hkv,d", [(F16, 4, 4, 64), (BF16, 8, 2, 128), (F16, 8, 1, 32), (BF16, 8, 2, 256),
                                             (F16, 4, 4, 256)])
def test_matches_torch_sdpa_in_float64(dtype, hq, hkv, d):
    """torch's scaled_dot_product_attention in fp64 with an explicit boolean mask."""
    b = wl.make_batch("sdpa", prefill=[(40, 100), (17, 17)], decode_kv_lens=[1, 64, 77], n_q_heads=hq,
                      n_kv_heads=hkv, head_dim=d, dtype=dtype, seed=41, block_size=16)
    got = oracle_out(b)
    group = hq // hkv
    for req in range(b.n_prefill + b.n_decode):
        k, v = logical_kv(b, req)
        q = request_q(b, req)
        q_len, kv_len = q.shape[0], k.shape[0]
        qt = torch.from_numpy(q).permute(1, 0, 2)                              # [Hq, q, d]
        kt = torch.from_numpy(k).permute(1, 0, 2).repeat_interleave(group, 0)  # [Hq, kv, d]
        vt = torch.from_numpy(v).permute(1, 0, 2).repeat_interleave(group, 0)
        i = torch.arange(q_len)[:, None]
        j = torch.arange(kv_len)[None, :]
        mask = j <= (kv_len - q_len + i)
        want = torch.nn.functional.scaled_dot_product_attention(
            qt, kt, vt, attn_mask=mask, scale=b.softmax_scale).permute(1, 0, 2).numpy()
        np.testing.assert_allclose(got[request_rows(b, req)], want, rtol=1e-11, atol=1e-12)


# -- p12: one dominant key ------------------------------------------------------------------ #
def test_one_dominant_key_wins():
    """With one score far above the rest the output tends to that key's V row."""
    length, hot = 40, 23
    b = wl.make_batch("hot", prefill=[], decode_kv_lens=[length], n_q_heads=2, n_kv_heads=1, head_dim=8,
                      dtype=F16, seed=51, softmax_scale=1.0)
    b.k_cache[0, hot, 0] = (b.decode_q[0, 0].float() * 8).to(torch.float16)
    _, v = logical_kv(b, 0)
    q = request_q(b, 0)[0]
    k, _ = logical_kv(b, 0)
    scores = k[:, 0] @ q[0]
    assert scores[hot] - np.delete(scores, hot).max() > 40
    np.testing.assert_allclose(oracle_out(b)[0][0], v[hot, 0], rtol=0, atol=1e-12)


# -- row subsets ------------------------------------------------------------------------------ #
def test_row_subset_equals_full_run():
    b = small_batch(prefill=((5, 9), (3, 3)), decodes=(1, 6, 11))
    full = oracle_out(b)
    rows = [7, 0, 10, 3]
    np.testing.assert_array_equal(oracle_out(b, rows=rows), full[rows])


def test_softmax_scale_is_a_multiplier():
    """Doubling the scale must equal doubling q (exact in fp16: a power of two)."""
    b = small_batch()
    ref_scale = oracle_out(dataclass_replace(b, softmax_scale=2 * b.softmax_scale))
    b.prefill_q.mul_(2)
    b.decode_q.mul_(2)
    np.testing.assert_allclose(oracle_out(b), ref_scale, rtol=1e-13, atol=1e-14)


def dataclass_replace(batch, **kw):
    import dataclasses
    return dataclasses.replace(batch, **kw)


def test_rejects_bad_arguments():
    b = small_batch()
    meta = b.seq_meta.copy()
    meta[0, 2] = meta[0, 1] - 1                       # kv_len < q_len
    with pytest.raises(ValueError):
        oracle_out(dataclass_replace(b, seq_meta=meta))
    meta = b.seq_meta.copy()
    meta[b.n_prefill, 1] = 2                          # decode with two query tokens
    with pytest.raises(ValueError):
        oracle_out(dataclass_replace(b, seq_meta=meta))
    with pytest.raises(ValueError):
        oracle_out(dataclass_replace(b, n_kv_heads=3))
    assert math.isfinite(oracle_out(b).sum())
