"""GPU parity: the HIP library against the fp64 CPU oracle, element by element.

Bar (max-abs over the whole batch, GPU 16-bit output widened to fp64): 2e-3 for fp16 inputs,
1e-2 for bf16 inputs; fp32 accumulation on the GPU.  Every call goes through the C ABI.
"""
import numpy as np
import pytest
import torch

from paper_2410_18038_amd import pod
from paper_2410_18038_amd import workloads as wl
from tests.helpers import oracle_out

pytestmark = pytest.mark.gpu

TOL = {wl.F16: 2e-3, wl.BF16: 1e-2}
ALL_MODES = ["fused", "serial", "streams", "fused_cta"]


def run_gpu(batch, mode="fused", **plan_kw):
    dev_batch = batch.to("cuda:0")
    attn = pod.HybridAttention(dev_batch, **plan_kw)
    out = attn.forward(dev_batch, mode=pod.MODES[mode])
    torch.cuda.synchronize()
    res = out.to(torch.float64).cpu().numpy()
    info = attn.info
    attn.close()
    return res, info


def check(batch, mode="fused", rows=None, **plan_kw):
    print(f"case {batch.name} mode={mode} {plan_kw}", flush=True)
    got, info = run_gpu(batch, mode, **plan_kw)
    want = oracle_out(batch, rows=rows)
    if rows is not None:
        got = got[rows]
    assert np.isfinite(got).all(), "non-finite GPU output"
    err = np.abs(got - want).max()
    assert err <= TOL[batch.dtype], f"max-abs error {err:.3e} > {TOL[batch.dtype]:.0e} ({batch.name}, {mode})"
    return err, info


@pytest.mark.parametrize("mode", ALL_MODES)
def test_config1_tiny_hybrid_batch(mode):
    check(wl.config_batch(1, poison=float("nan")), mode)


@pytest.mark.parametrize("mode", ["prefill_only", "decode_only"])
def test_single_operation_modes_write_only_their_rows(mode):
    batch = wl.config_batch(1, poison=float("nan"))
    dev_batch = batch.to("cuda:0")
    attn = pod.HybridAttention(dev_batch)
    out = torch.full((batch.n_rows, batch.n_q_heads, batch.head_dim), 7.0, dtype=batch.torch_dtype, device="cuda:0")
    attn.forward(dev_batch, out=out, mode=pod.MODES[mode])
    torch.cuda.synchronize()
    got = out.to(torch.float64).cpu().numpy()
    want = oracle_out(batch)
    npr = batch.n_prefill_rows
    mine = slice(0, npr) if mode == "prefill_only" else slice(npr, None)
    other = slice(npr, None) if mode == "prefill_only" else slice(0, npr)
    assert np.abs(got[mine] - want[mine]).max() <= TOL[batch.dtype]
    assert (got[other] == 7.0).all()
    attn.close()


@pytest.mark.parametrize("dtype", [wl.F16, wl.BF16])
@pytest.mark.parametrize("hq,hkv", [(4, 4), (8, 2), (8, 1), (16, 1)])
@pytest.mark.parametrize("d", [64, 128, 256])
@pytest.mark.parametrize("block_size", [0, 16])
def test_shapes_dtypes_layouts(dtype, hq, hkv, d, block_size):
    """Several tiles and ragged tails in both operations; cache tails and spare blocks poisoned."""
    if d == 256 and hq // hkv > 8:
        pytest.skip("head_dim 256 takes at most 8 query heads per K/V head")
    batch = wl.make_batch(f"grid-{hq}/{hkv}-d{d}-bs{block_size}", prefill=[(200, 333), (37, 37)],
                          decode_kv_lens=[1, 31, 32, 33, 257, 700], n_q_heads=hq, n_kv_heads=hkv,
                          head_dim=d, dtype=dtype, seed=1000 + hq * 7 + hkv + d + block_size,
                          block_size=block_size, poison=float("nan"))
    check(batch, "fused")


@pytest.mark.parametrize("hq,hkv", [(5, 5), (9, 3), (10, 5)])
@pytest.mark.parametrize("d", [64, 128, 256])
@pytest.mark.parametrize("block_size", [0, 16, 64, 24])
def test_token_sizes_that_are_no_power_of_two(hq, hkv, d, block_size):
    """K/V head counts of 3 and 5: a cached token of 768 ... 2560 bytes, in the contiguous layout,
    the block-wise paged layouts (16 and 64 keys) and the general one (24 keys)."""
    batch = wl.make_batch(f"odd-{hq}/{hkv}-d{d}-bs{block_size}", prefill=[(150, 401), (64, 64)],
                          decode_kv_lens=[1, 47, 48, 49, 300, 1111], n_q_heads=hq, n_kv_heads=hkv,
                          head_dim=d, dtype=wl.F16, seed=2000 + hq * 7 + hkv + d + block_size,
                          block_size=block_size, poison=float("nan"))
    check(batch, "fused")
    check(batch, "serial", decode_chunk=256, prefill_split_len=128, max_prefill_waves=64)


@pytest.mark.parametrize("dtype,hq,hkv,d", [(wl.F16, 8, 2, 128), (wl.BF16, 6, 3, 64), (wl.F16, 4, 4, 128), (wl.BF16, 8, 2, 256)])
@pytest.mark.parametrize("block_size", [0, 16, 32, 24])
def test_head_major_cache(dtype, hq, hkv, d, block_size):
    """The [.., Hkv, tokens, d] cache order in every address path: contiguous, block-wise paged
    (16 and 32 keys) and general paged (24 keys); unseen slots poisoned."""
    batch = wl.to_head_major(wl.make_batch(
        f"hm-{hq}/{hkv}-d{d}-bs{block_size}", prefill=[(150, 401), (64, 64)],
        decode_kv_lens=[1, 47, 48, 49, 300, 1111], n_q_heads=hq, n_kv_heads=hkv, head_dim=d, dtype=dtype,
        seed=3000 + hq * 7 + hkv + d + block_size, block_size=block_size, poison=float("nan")))
    check(batch, "fused")
    check(batch, "serial", decode_chunk=256, prefill_split_len=128, max_prefill_waves=64)


@pytest.mark.parametrize("mode", ALL_MODES)
@pytest.mark.parametrize("block_size", [0, 16, 48])
@pytest.mark.parametrize("d", [128, 256])
def test_split_kv_paths(mode, block_size, d):
    """Force split-KV in both operations (short chunks, tiny split lengths) and merge the partials."""
    batch = wl.make_batch(f"split-bs{block_size}-d{d}", prefill=[(96, 1500)], decode_kv_lens=[1200, 90, 2047, 640],
                          n_q_heads=8, n_kv_heads=2, head_dim=d, dtype=wl.BF16, seed=77 + block_size,
                          block_size=block_size, poison=float("nan"))
    err, info = check(batch, mode, decode_chunk=256, prefill_split_len=256, max_prefill_waves=64)
    assert info.max_prefill_splits > 1 and info.max_decode_splits > 1


@pytest.mark.parametrize("block_size", [0, 16])
def test_many_requests_of_both_kinds(block_size):
    """Forty prefill chunks (1..300 new tokens over 0..900 cached ones) and 1500 decodes (1..700
    keys) in one batch, every output row against the oracle: request tables, row blocks that mix
    nothing across requests, thousands of short decode units and their queues."""
    rng = np.random.Generator(np.random.PCG64(4242 + block_size))
    prefill = [(int(q), int(q + p)) for q, p in zip(rng.integers(1, 301, 40), rng.integers(0, 901, 40))]
    decodes = rng.integers(1, 701, 1500).tolist()
    batch = wl.make_batch(f"many-bs{block_size}", prefill=prefill, decode_kv_lens=decodes, n_q_heads=16,
                          n_kv_heads=4, head_dim=128, dtype=wl.BF16, seed=4243 + block_size,
                          block_size=block_size, poison=float("nan"))
    err, info = check(batch, "fused")
    assert info.n_decode_units >= 1500 * 4 and info.n_prefill_items >= 40 * 4
    check(batch, "serial")


def test_random_batches_and_tuning_values():
    """Thirty seeded random batches (shapes, layouts, lengths) under random split lengths, split
    caps, policies and planned chip sizes, in a random mode each: all rows against the oracle."""
    rng = np.random.Generator(np.random.PCG64(777))
    for case in range(30):
        n_p, n_d = int(rng.integers(0, 4)), int(rng.integers(0, 40))
        if n_p + n_d == 0:
            n_p = 1
        top = int(rng.choice([60, 600, 3000]))
        prefill = []
        for _ in range(n_p):
            kv = int(rng.integers(1, top + 1))
            prefill.append((int(rng.integers(1, min(kv, 400) + 1)), kv))
        decodes = rng.integers(1, top + 1, n_d).tolist()
        hkv = int(rng.choice([1, 2, 3, 8]))
        group = int(rng.choice([1, 2, 4, 7, 16]))
        dtype = int(rng.choice([wl.F16, wl.BF16]))
        batch = wl.make_batch(f"rand{case}", prefill=prefill, decode_kv_lens=decodes, n_q_heads=hkv * group,
                              n_kv_heads=hkv, head_dim=int(rng.choice([64, 128, 256] if group <= 8 else [64, 128])), dtype=dtype,
                              seed=7000 + case, block_size=int(rng.choice([0, 16, 32, 40])), poison=float("nan"))
        if rng.integers(0, 2):
            batch = wl.to_head_major(batch)
        kw = dict(n_compute_units=int(rng.choice([0, 1, 3, 64, 500])),
                  decode_chunk=int(rng.choice([0, 16, 112, 256, 1024])),
                  prefill_split_len=int(rng.choice([0, 64, 320])),
                  max_prefill_waves=int(rng.choice([0, 1, 64])), policy=int(rng.integers(0, 3)))
        check(batch, str(rng.choice(ALL_MODES)), **kw)


def test_degenerate_batches():
    """Only prefill, only decode, one key, a chunk without prefix."""
    for name, prefill, decodes in [("only-prefill", [(65, 65)], []), ("only-decode", [], [1, 5, 64]),
                                   ("one-key", [(1, 1)], [1]), ("no-prefix", [(130, 130)], [3])]:
        for d in (64, 256):
            batch = wl.make_batch(f"{name}-d{d}", prefill=prefill, decode_kv_lens=decodes, n_q_heads=4, n_kv_heads=2,
                                  head_dim=d, dtype=wl.F16, seed=5, poison=float("nan"))
            for mode in ALL_MODES:
                check(batch, mode)


def test_repeated_launches_are_bit_identical_and_counters_reset():
    """The binder changes who computes a work item, never what it computes."""
    batch = wl.make_batch("repeat", prefill=[(300, 900)], decode_kv_lens=[500] * 40 + [33, 1000],
                          n_q_heads=8, n_kv_heads=2, head_dim=128, dtype=wl.F16, seed=9, block_size=16)
    dev_batch = batch.to("cuda:0")
    attn = pod.HybridAttention(dev_batch, decode_chunk=128)
    first = attn.forward(dev_batch).clone()
    for _ in range(20):
        again = attn.forward(dev_batch)
        assert torch.equal(first.view(torch.int16), again.view(torch.int16))
    serial = attn.forward(dev_batch, mode=pod.MODE_SERIAL)
    assert torch.equal(first.view(torch.int16), serial.view(torch.int16))
    for _ in range(5):                                   # the CTA-parallel launch of the same plan, same counters
        cta = attn.forward(dev_batch, mode=pod.MODES["fused_cta"])
        assert torch.equal(first.view(torch.int16), cta.view(torch.int16))
    torch.cuda.synchronize()
    # the whole counter block at the head of the workspace: per-unit binder state, work counters,
    # per-XCD queue counters (one 128-byte line each) and the words that idle claims add zero to
    hdr_bytes = 4096 + 256 + 8 * 128 + 512 * 128
    assert attn.ws_bytes >= hdr_bytes
    hdr = attn.workspace[(attn.ws_ptr - attn.workspace.data_ptr()):][:hdr_bytes].view(torch.int32)
    assert int(hdr.abs().sum()) == 0, "binder counters not back at zero after the launches"
    attn.close()


def test_decode_through_prefill_path_matches_decode_path():
    """A decode submitted as a one-token prefill chunk must agree with the decode path."""
    lens = [77, 512, 1025]
    as_decode = wl.make_batch("dec", prefill=[], decode_kv_lens=lens, n_q_heads=8, n_kv_heads=2, head_dim=128,
                              dtype=wl.F16, seed=13)
    as_prefill = wl.make_batch("pre", prefill=[(1, l) for l in lens], decode_kv_lens=[], n_q_heads=8,
                               n_kv_heads=2, head_dim=128, dtype=wl.F16, seed=14, max_len=as_decode.max_len)
    as_prefill.prefill_q.copy_(as_decode.decode_q)
    as_prefill.k_cache.copy_(as_decode.k_cache)
    as_prefill.v_cache.copy_(as_decode.v_cache)
    a, _ = run_gpu(as_decode)
    b, _ = run_gpu(as_prefill)
    assert np.abs(a - b).max() <= 2e-3
    assert np.abs(a - oracle_out(as_decode)).max() <= 2e-3


def test_decode_stream_crosses_many_short_units():
    """Hundreds of decode units of 1..3 steps next to a few long ones, on a plan made for two
    compute units: few workers, so every wavefront streams through many units (the load ring then
    holds a unit boundary most of the time, heads run out before their next unit is known, queues
    are emptied and the other XCDs' queues are tried), in all three launch modes."""
    rng = np.random.Generator(np.random.PCG64(321))
    lens = rng.integers(1, 41, size=150).tolist() + [5000, 17, 3001, 1, 16, 4097]
    for hq, hkv, d, bs in [(8, 2, 128, 16), (4, 4, 64, 0), (16, 1, 128, 48), (8, 1, 256, 16)]:
        batch = wl.make_batch(f"stream-{hq}/{hkv}-d{d}-bs{bs}", prefill=[(70, 200)], decode_kv_lens=lens,
                              n_q_heads=hq, n_kv_heads=hkv, head_dim=d, dtype=wl.F16, seed=4242 + d + bs,
                              block_size=bs, poison=float("nan"))
        for mode in ALL_MODES:
            err, info = check(batch, mode, n_compute_units=2, decode_chunk=512)
            assert info.fused_grid == 4 and info.n_decode_units > 150 * hkv
    # and a plan made for more compute units than the GPU has: more workgroups than can be resident
    # at once, so some start only when others have left
    batch = wl.make_batch("oversubscribed", prefill=[(700, 1400)], decode_kv_lens=[300] * 900 + [2000] * 8,
                          n_q_heads=8, n_kv_heads=4, head_dim=128, dtype=wl.BF16, seed=777, block_size=16)
    for mode in ALL_MODES:
        err, info = check(batch, mode, n_compute_units=1000, decode_chunk=128)
        assert info.fused_grid > 1000        # one decode worker per planned unit plus the prefill items


def test_event_log_holds_every_item_and_unit_once():
    """The event log (begin and end of every prefill item and decode unit of one launch) names each
    work id exactly once, with sane times, and logging does not change the result."""
    batch = wl.make_batch("evlog", prefill=[(300, 900)], decode_kv_lens=[500] * 40 + [33, 1000, 7],
                          n_q_heads=8, n_kv_heads=2, head_dim=128, dtype=wl.BF16, seed=99, block_size=16)
    dev_batch = batch.to("cuda:0")
    attn = pod.HybridAttention(dev_batch, decode_chunk=128)
    plain = attn.forward(dev_batch).clone()
    attn.enable_event_log()
    logged = attn.forward(dev_batch)
    ev = attn.read_event_log()
    assert torch.equal(plain.view(torch.int16), logged.view(torch.int16))
    assert len(ev) == attn.info.n_prefill_items + attn.info.n_decode_units
    for kind, n in ((0, attn.info.n_prefill_items), (1, attn.info.n_decode_units)):
        ids = np.sort(ev["item"][ev["kind"] == kind])
        assert ids.tolist() == list(range(n))
    assert (ev["t_end"] >= ev["t_begin"]).all()
    span_us = (int(ev["t_end"].max()) - int(ev["t_begin"].min())) / 100.0
    assert 0 < span_us < 1e5
    attn.disable_event_log()
    again = attn.forward(dev_batch)
    assert torch.equal(plain.view(torch.int16), again.view(torch.int16))
    attn.close()


def _sample_rows(batch, n_p, n_d, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    npr, nd = batch.n_prefill_rows, batch.n_decode
    fixed_p = [r for r in (0, 1, 15, 16, 127, 128, npr // 2, npr - 2, npr - 1) if 0 <= r < npr]
    rows_p = np.unique(np.concatenate([np.array(fixed_p, dtype=np.int64), rng.integers(0, max(npr, 1), size=n_p)]))
    rows_d = npr + np.unique(np.concatenate([np.array([0, nd - 1]), rng.integers(0, max(nd, 1), size=n_d)]))
    return np.concatenate([rows_p[:0] if npr == 0 else rows_p, rows_d[:0] if nd == 0 else rows_d]).astype(np.int32)


@pytest.mark.parametrize("config,index", [(2, 0), (3, 0), (4, 0)] + [(5, i) for i in range(len(wl.RATIO_SWEEP))])
def test_full_size_batches_on_sampled_rows(config, index):
    """The configurations the benchmark times, at full size and with the default plan (the launch
    shape the benchmark uses): a sample of output rows (first, last and tile-edge rows of the chunk,
    random rows, first and last decode request; every head of each) against the oracle, in the fused
    mode, and the serial baseline bit-identical to it."""
    batch = wl.config_batch(config, index, device="cuda:0")
    attn = pod.HybridAttention(batch)
    out = attn.forward(batch)
    torch.cuda.synchronize()
    rows = _sample_rows(batch, 24, 24, seed=config * 10 + index)
    print(f"case {batch.name}: {len(rows)} sampled rows of {batch.n_rows}", flush=True)
    want = oracle_out(batch, rows=rows)
    got = out[torch.from_numpy(rows.astype(np.int64)).to("cuda:0")].to(torch.float64).cpu().numpy()
    assert bool(torch.isfinite(out.to(torch.float32)).all())
    err = np.abs(got - want).max()
    assert err <= TOL[batch.dtype], f"max-abs error {err:.3e} on sampled rows of {batch.name}"
    serial = attn.forward(batch, mode=pod.MODE_SERIAL)
    assert torch.equal(out.view(torch.int16), serial.view(torch.int16))
    cta = attn.forward(batch, mode=pod.MODES["fused_cta"])
    assert torch.equal(out.view(torch.int16), cta.view(torch.int16))
    attn.close()


def test_head_dim_256_at_benchmark_size():
    """A batch of the size of the benchmark configurations at 256 channels per head (16 query heads on 8 K/V
    heads, a 1024-token chunk ending at 4096 beside 64 decodes at 2K-8K keys, 16-key blocks): sampled
    rows against the oracle, serial and CTA-parallel launches bit-identical to the fused one."""
    rng = np.random.Generator(np.random.PCG64(256))
    batch = wl.make_batch("d256-16/8", prefill=[(1024, 4096)], decode_kv_lens=rng.integers(2048, 8193, 64).tolist(),
                          n_q_heads=16, n_kv_heads=8, head_dim=256, dtype=wl.BF16, seed=2560, block_size=16,
                          device="cuda:0")
    attn = pod.HybridAttention(batch)
    out = attn.forward(batch)
    torch.cuda.synchronize()
    rows = _sample_rows(batch, 24, 24, seed=256)
    print(f"case {batch.name}: {len(rows)} sampled rows of {batch.n_rows}, {attn.info.n_prefill_items} items, "
          f"{attn.info.n_decode_units} units", flush=True)
    want = oracle_out(batch, rows=rows)
    got = out[torch.from_numpy(rows.astype(np.int64)).to("cuda:0")].to(torch.float64).cpu().numpy()
    assert bool(torch.isfinite(out.to(torch.float32)).all())
    err = np.abs(got - want).max()
    assert err <= TOL[batch.dtype], f"max-abs error {err:.3e} on sampled rows of {batch.name}"
    for mode in ("serial", "fused_cta"):
        other = attn.forward(batch, mode=pod.MODES[mode])
        assert torch.equal(out.view(torch.int16), other.view(torch.int16)), mode
    attn.close()


@pytest.mark.parametrize("dtype,block_size", [(wl.F16, 0), (wl.BF16, 16)])
def test_contexts_of_128k_tokens(dtype, block_size):
    """Contexts far beyond the benchmark's (128K keys, and lengths that are no multiple of anything):
    offsets, unit counts and split counts at the large end.  Sampled rows, every head of each."""
    batch = wl.make_batch("ctx128k", prefill=[(96, 131072)], decode_kv_lens=[131072, 100003, 65537],
                          n_q_heads=8, n_kv_heads=2, head_dim=128, dtype=dtype, block_size=block_size,
                          seed=77, device="cuda:0")
    attn = pod.HybridAttention(batch)
    out = attn.forward(batch)
    torch.cuda.synchronize()
    rows = _sample_rows(batch, 6, 3, seed=5)
    print(f"case {batch.name}: {len(rows)} sampled rows of {batch.n_rows}, {attn.info.n_decode_units} units, "
          f"{attn.info.n_prefill_items} items", flush=True)
    want = oracle_out(batch, rows=rows)
    got = out[torch.from_numpy(rows.astype(np.int64)).to("cuda:0")].to(torch.float64).cpu().numpy()
    assert bool(torch.isfinite(out.to(torch.float32)).all())
    err = np.abs(got - want).max()
    assert err <= TOL[batch.dtype], f"max-abs error {err:.3e} on sampled rows of {batch.name}"
    serial = attn.forward(batch, mode=pod.MODE_SERIAL)
    assert torch.equal(out.view(torch.int16), serial.view(torch.int16))
    attn.close()


@pytest.mark.parametrize("model,n_decode,chunk", [("yi-6b", 54, 0), ("yi-6b", 55, 31), ("llama-3-8b", 64, 15)])
def test_chunk_series_batches_on_sampled_rows(model, n_decode, chunk):
    """Chunks of a 16K prompt next to decodes at 16K context (the shape of the paper's Figure 6 and
    Table 8; 54 and 55 decodes are its wave-quantization pair): sampled rows against the oracle."""
    base = wl.series_base(model, n_decode, device="cuda:0")
    batch = wl.series_chunk(base, chunk)
    attn = pod.HybridAttention(batch)
    out = attn.forward(batch)
    torch.cuda.synchronize()
    rows = _sample_rows(batch, 16, 16, seed=chunk + n_decode)
    print(f"case {batch.name}: {len(rows)} sampled rows of {batch.n_rows}", flush=True)
    want = oracle_out(batch, rows=rows)
    got = out[torch.from_numpy(rows.astype(np.int64)).to("cuda:0")].to(torch.float64).cpu().numpy()
    err = np.abs(got - want).max()
    assert err <= TOL[batch.dtype], f"max-abs error {err:.3e} on sampled rows of {batch.name}"
    for mode in ("serial", "streams"):
        other = attn.forward(batch, mode=pod.MODES[mode])
        assert torch.equal(out.view(torch.int16), other.view(torch.int16))
    attn.close()


def test_colocation_probe_moves_every_chunk_once():
    """The co-location experiment (Section 3.3): every variant of the fused launch computes c = a + b
    over every chunk exactly once, whatever the binding, and the per-unit binder claims every item."""
    n_items, item_bytes = 700, 16 * 1000
    a = torch.arange(n_items * item_bytes // 4, dtype=torch.float32, device="cuda:0")
    b = torch.full_like(a, 0.5)
    ctr = torch.zeros(1026, dtype=torch.int32, device="cuda:0")
    sink = torch.zeros(4, dtype=torch.float32, device="cuda:0")
    for variant, n_cmp in [(1, 0), (2, 300), (3, 300), (3, 0), (3, 1500)]:
        c = torch.zeros_like(a)
        pod.pod_attn_probe_colocation(variant, a.data_ptr(), b.data_ptr(), c.data_ptr(), item_bytes, n_items, n_cmp,
                                      50, ctr.data_ptr(), sink.data_ptr(), torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        assert torch.equal(c, a + b), f"variant {variant} with {n_cmp} compute items"
        if variant == 3:
            got = ctr.cpu().numpy()
            assert got[:1024].sum() == n_items + n_cmp
            assert got[1024] >= n_cmp and got[1025] >= n_items and got[1024] + got[1025] <= n_items + n_cmp + 2 * (n_items + n_cmp)
    with pytest.raises(pod.PodError):
        pod.pod_attn_probe_colocation(3, a.data_ptr(), b.data_ptr(), a.data_ptr(), 24, 1, 1, 1, ctr.data_ptr(),
                                      sink.data_ptr(), 0)


@pytest.mark.parametrize("mode", ["fused", "serial"])
def test_forward_can_be_captured_in_a_graph_and_replayed(mode):
    """`pod_attn_forward` launches kernels only (no allocation, no memset, no host wait), so a caller
    may record it into a HIP graph.  Replays, with eager launches and synchronisations between them,
    give the eager result bit for bit, and the counters are back at zero after each."""
    batch = wl.make_batch("graph", prefill=[(200, 700)], decode_kv_lens=[900] * 30 + [64, 2500],
                          n_q_heads=8, n_kv_heads=2, head_dim=128, dtype=wl.F16, seed=31, block_size=16)
    dev_batch = batch.to("cuda:0")
    attn = pod.HybridAttention(dev_batch, decode_chunk=256)
    eager = attn.forward(dev_batch, mode=pod.MODES[mode]).clone()
    torch.cuda.synchronize()
    out = torch.zeros_like(eager)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        attn.forward(dev_batch, out=out, mode=pod.MODES[mode])        # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            attn.forward(dev_batch, out=out, mode=pod.MODES[mode])
    torch.cuda.current_stream().wait_stream(side)
    for i in range(4):
        out.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), eager.view(torch.int16)), f"replay {i}"
        again = attn.forward(dev_batch, mode=pod.MODES[mode])              # eager work between replays
        torch.cuda.synchronize()
        assert torch.equal(again.view(torch.int16), eager.view(torch.int16))
    attn.close()


@pytest.mark.parametrize("config", [2, 4])
def test_both_operations_are_resident_on_every_compute_unit(config):
    """Section 4.1's guarantee, read off the library's own records of one fused launch of a
    benchmark batch (parity cannot see placement): at least 95 % of the hardware units that took
    part hold one workgroup that started with prefill and one that started with decode; every
    prefill item and decode unit ran exactly once; and on at least 95 % of the units a decode unit
    was streaming while a prefill item was running on the same unit."""
    from paper_2410_18038_amd import trace_report
    batch = wl.config_batch(config, device="cuda:0")
    attn = pod.HybridAttention(batch)
    plain = attn.forward(batch).clone()
    attn.enable_trace()
    attn.enable_event_log()
    traced = attn.forward(batch)
    trace, events = attn.read_trace(), attn.read_event_log()
    assert torch.equal(plain.view(torch.int16), traced.view(torch.int16))
    info = attn.info
    rep = trace_report.colocation(trace, events, info.n_prefill_items, info.n_decode_units)
    print(trace_report.as_text(batch.name, rep), flush=True)
    assert rep["workgroups"] == info.fused_grid == 2 * info.n_compute_units
    assert rep["hardware_units"] >= 0.95 * info.n_compute_units
    assert rep["units_with_both_first_roles"] >= 0.95 * rep["hardware_units"]
    assert rep["prefill_items_logged_once"] and rep["decode_units_logged_once"]
    assert rep["units_where_roles_overlap_in_time"] >= 0.95 * rep["hardware_units"]
    # configuration 2's items all run beside the decode stream; configuration 4's prefill outlasts it
    assert rep["share_of_prefill_time_with_decode_on_same_unit"] > (0.8 if config == 2 else 0.2)
    # the records of the workgroups agree with the plan: prefill items are counted per workgroup
    n_items = int(trace["n_first"][trace["first_role"] == 0].sum() + trace["n_second"][trace["first_role"] == 1].sum())
    assert n_items == info.n_prefill_items
    assert (trace["t_switch"] >= trace["t_begin"]).all() and (trace["t_end"] >= trace["t_switch"]).all()
    attn.close()


# ---- the prefill-heavy configuration (Section 4.2.2's second configuration) --------------------------
HEAVY_MODES = ["fused_heavy", "prefill_only_heavy", "decode_only_lite"]


def check_rows_of(batch, mode):
    """`check` for a mode that writes only one operation's rows."""
    npr = batch.n_prefill_rows
    rows = None
    if mode.startswith("prefill_only"):
        rows = np.arange(0, npr)
    elif mode.startswith("decode_only"):
        rows = np.arange(npr, batch.n_rows)
    return check(batch, mode, rows=rows)


@pytest.mark.parametrize("mode", HEAVY_MODES)
@pytest.mark.parametrize("dtype", [wl.F16, wl.BF16])
@pytest.mark.parametrize("hq,hkv", [(4, 4), (8, 2), (16, 1), (10, 5)])
@pytest.mark.parametrize("block_size", [0, 16, 64])
def test_prefill_heavy_configuration_matches_the_oracle(mode, dtype, hq, hkv, block_size):
    """Both kernels of the configuration, alone and together, over group sizes 1 to 16, a token size
    that is no power of two, both cache layouts it is built for, and decode contexts that end
    inside, at and just past a 16-key step."""
    batch = wl.make_batch(
        f"heavy-{hq}q{hkv}kv-bs{block_size}", prefill=[(70, 200), (129, 129)],
        decode_kv_lens=[1, 15, 16, 17, 31, 33, 257, 700, 2049], n_q_heads=hq, n_kv_heads=hkv, head_dim=128,
        dtype=dtype, seed=500 + hq + block_size, block_size=block_size, poison=float("nan"))
    check_rows_of(batch, mode)


def test_prefill_heavy_configuration_with_split_kv_and_head_major_cache():
    batch = wl.make_batch("heavy-split", prefill=[(300, 2300)], decode_kv_lens=[5000, 77, 1234, 3000],
                          n_q_heads=8, n_kv_heads=2, head_dim=128, dtype=wl.BF16, seed=41, block_size=16,
                          poison=float("nan"))
    for mode in HEAVY_MODES:
        print(f"case {batch.name} mode={mode} forced splits", flush=True)
        got, info = run_gpu(batch, mode, decode_chunk=256, prefill_split_len=512, max_prefill_waves=8)
        assert info.max_decode_splits > 1 and info.max_prefill_splits > 1
        want = oracle_out(batch)
        npr = batch.n_prefill_rows
        sl = slice(0, npr) if mode.startswith("prefill_only") else slice(npr, None) if mode.startswith("decode_only") else slice(None)
        assert np.abs(got[sl] - want[sl]).max() <= TOL[batch.dtype]
    hm = wl.to_head_major(wl.make_batch("heavy-hnd", prefill=[(40, 90)], decode_kv_lens=[3, 64, 999], n_q_heads=8,
                                        n_kv_heads=2, head_dim=128, dtype=wl.F16, seed=42, block_size=32,
                                        poison=float("nan")))
    for mode in HEAVY_MODES:
        check_rows_of(hm, mode)


def test_prefill_heavy_configuration_is_refused_where_it_is_not_built():
    batch = wl.make_batch("heavy-d64", prefill=[(40, 90)], decode_kv_lens=[3, 64], n_q_heads=4, n_kv_heads=2,
                          head_dim=64, dtype=wl.F16, seed=43)
    dev_batch = batch.to("cuda:0")
    attn = pod.HybridAttention(dev_batch)
    with pytest.raises(pod.PodError) as e:
        attn.forward(dev_batch, mode=pod.MODES["fused_heavy"])
    assert e.value.status == -2
    attn.close()


def test_prefill_heavy_configuration_places_three_workgroups_on_every_unit():
    """What the configuration is for, read off the trace records of one launch of the MFMA-bound
    benchmark batch: when a unit's decode workgroup starts, two prefill workgroups are running on
    that unit, on at least 90 % of the units; nearly every unit has one decode workgroup; the decode
    kernel ends while the prefill kernel is still running; the output is within the parity bar."""
    batch = wl.config_batch(4, device="cuda:0")
    attn = pod.HybridAttention(batch)
    mode = pod.MODES["fused_heavy"]
    for _ in range(3):
        attn.forward(batch, mode=mode)
    attn.enable_trace()
    out = attn.forward(batch, mode=mode)
    torch.cuda.synchronize()
    info = attn.info
    n_p, n_d = info.n_prefill_items, info.n_compute_units
    trace = attn.trace.cpu().numpy().view(pod.TRACE_DTYPE)[: n_p + n_d].copy()
    P, D = trace[:n_p], trace[n_p:]
    assert (P["first_role"] == 0).all() and (D["first_role"] == 1).all() and (trace["t_end"] > 0).all()
    units, per_unit = np.unique(D["cu"], return_counts=True)
    assert len(units) >= 0.9 * info.n_compute_units and (per_unit == 1).mean() >= 0.9
    settle = 500                                                  # 5 us of the 100 MHz clock
    resident = np.array([int(((P["cu"] == d["cu"]) & (P["t_begin"] <= d["t_begin"] + settle) &
                              (P["t_end"] > d["t_begin"] + settle)).sum()) for d in D])
    print("prefill workgroups resident beside each decode workgroup:", np.bincount(resident).tolist(), flush=True)
    assert (resident == 2).mean() >= 0.9
    assert int(D["n_first"].sum()) > 0                           # units run by the first wavefront of each workgroup
    assert D["t_end"].max() < P["t_end"].max()
    rows = np.concatenate([np.arange(0, batch.n_prefill_rows, 97), np.arange(batch.n_prefill_rows, batch.n_rows)])
    want = oracle_out(batch, rows=rows)
    got = out.to(torch.float64).cpu().numpy()[rows]
    assert np.abs(got - want).max() <= TOL[batch.dtype]
    attn.close()


def test_prefill_heavy_configuration_with_many_short_units_and_long_contexts():
    """The light decode kernel's own claim path: hundreds of units of 1..3 steps beside a few long
    ones on a plan made for two compute units (every wavefront runs through many units, empties its
    queue and tries the others), a plan with more decode workgroups than can be resident, and
    contexts of 128K keys (sampled rows)."""
    rng = np.random.Generator(np.random.PCG64(322))
    lens = rng.integers(1, 41, size=150).tolist() + [5000, 17, 3001, 1, 16, 4097]
    for hq, hkv, bs in [(8, 2, 16), (16, 1, 0)]:
        batch = wl.make_batch(f"heavy-stream-{hq}/{hkv}-bs{bs}", prefill=[(70, 200)], decode_kv_lens=lens,
                              n_q_heads=hq, n_kv_heads=hkv, head_dim=128, dtype=wl.F16, seed=4343 + bs,
                              block_size=bs, poison=float("nan"))
        for mode in ("fused_heavy", "decode_only_lite"):
            print(f"case {batch.name} mode={mode}", flush=True)
            got, info = run_gpu(batch, mode, n_compute_units=2, decode_chunk=512)
            assert info.n_decode_units > 150 * hkv
            want = oracle_out(batch)
            sl = slice(batch.n_prefill_rows, None) if mode == "decode_only_lite" else slice(None)
            assert np.abs(got[sl] - want[sl]).max() <= TOL[batch.dtype]
    batch = wl.make_batch("heavy-oversubscribed", prefill=[(700, 1400)], decode_kv_lens=[300] * 900 + [2000] * 8,
                          n_q_heads=8, n_kv_heads=4, head_dim=128, dtype=wl.BF16, seed=778, block_size=16)
    check(batch, "fused_heavy", n_compute_units=1000, decode_chunk=128)
    big = wl.make_batch("heavy-ctx128k", prefill=[(96, 131072)], decode_kv_lens=[131072, 100003, 65537],
                        n_q_heads=8, n_kv_heads=2, head_dim=128, dtype=wl.BF16, block_size=16, seed=78, device="cuda:0")
    attn = pod.HybridAttention(big)
    out = attn.forward(big, mode=pod.MODES["fused_heavy"])
    torch.cuda.synchronize()
    rows = _sample_rows(big, 6, 3, seed=6)
    want = oracle_out(big, rows=rows)
    got = out[torch.from_numpy(rows.astype(np.int64)).to("cuda:0")].to(torch.float64).cpu().numpy()
    assert bool(torch.isfinite(out.to(torch.float32)).all())
    assert np.abs(got - want).max() <= TOL[big.dtype]
    attn.close()
