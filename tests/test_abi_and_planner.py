"""CPU tests of the C-ABI library: symbols, argument validation, the host planner, the model of the device's claim protocol.

No compute call is made here; the planner needs no GPU once n_compute_units is given.
"""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2410_18038_amd import pod
from paper_2410_18038_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLDEN = os.path.join(ROOT, "tests", "golden")


def params_for(batch, **kw):
    base = dict(n_prefill=batch.n_prefill, n_decode=batch.n_decode, n_q_heads=batch.n_q_heads,
                n_kv_heads=batch.n_kv_heads, head_dim=batch.head_dim, dtype=batch.dtype,
                softmax_scale=batch.softmax_scale, block_size=batch.block_size,
                max_blocks_per_seq=batch.max_blocks_per_seq, n_cache_rows=batch.n_cache_rows,
                n_blocks=batch.n_blocks, kv_seq_stride=batch.kv_seq_stride, n_compute_units=256)
    base.update(kw)
    return pod.make_params(**base)


def meta_only(name, prefill, decodes, hq=32, hkv=8, d=128, block_size=16):
    """A batch descriptor without tensors worth mentioning (tiny head_dim is not allowed, so keep d)."""
    n_seqs = len(prefill) + len(decodes)
    meta = np.zeros((n_seqs, 4), dtype=np.int32)
    q0 = 0
    for r, (q_len, kv_len) in enumerate(prefill):
        meta[r] = (q0, q_len, kv_len, r)
        q0 += q_len
    for i, kv_len in enumerate(decodes):
        meta[len(prefill) + i] = (i, 1, kv_len, len(prefill) + i)
    longest = int(meta[:, 2].max()) if n_seqs else 1
    prm = pod.make_params(n_prefill=len(prefill), n_decode=len(decodes), n_q_heads=hq, n_kv_heads=hkv,
                          head_dim=d, dtype=wl.BF16, softmax_scale=d ** -0.5, block_size=block_size,
                          max_blocks_per_seq=(longest + 15) // 16 if block_size else 0, n_cache_rows=max(n_seqs, 1),
                          n_blocks=10 ** 6 if block_size else 0,
                          kv_seq_stride=0 if block_size else longest * hkv * d, n_compute_units=256)
    return prm, meta


# -- the library and its symbols ------------------------------------------------------------- #
def test_library_loads_and_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "pod_attn.h")).read()
    declared = sorted(set(re.findall(r"\b(pod_attn_[a-z_]+)\s*\(", header)))
    assert declared, "no declarations found in the header"
    lib = ctypes.CDLL(pod.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), f"{name} is declared in include/pod_attn.h but not exported"
    assert sorted(pod.EXPORTS) == declared
    assert "gfx950" in pod.pod_attn_version()


def test_struct_layouts_match_the_header(tmp_path):
    """Compile the public header as plain C and compare struct sizes and a few offsets with ctypes."""
    import subprocess
    src = tmp_path / "sizes.c"
    src.write_text(
        '#include <stdio.h>\n#include <stddef.h>\n#include "pod_attn.h"\n'
        'int main(void){printf("%zu %zu %zu %zu %zu %zu\\n", sizeof(pod_attn_params), sizeof(pod_attn_plan_info),'
        ' offsetof(pod_attn_params, kv_seq_stride), offsetof(pod_attn_params, n_compute_units),'
        ' offsetof(pod_attn_params, kv_order), offsetof(pod_attn_plan_info, workspace_bytes)); return 0;}\n')
    exe = tmp_path / "sizes"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)],
                   check=True)
    got = [int(x) for x in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()]
    assert got == [ctypes.sizeof(pod.Params), ctypes.sizeof(pod.PlanInfo), pod.Params.kv_seq_stride.offset,
                   pod.Params.n_compute_units.offset, pod.Params.kv_order.offset,
                   pod.PlanInfo.workspace_bytes.offset]


# -- validation ------------------------------------------------------------------------------- #
def test_invalid_arguments_are_rejected_with_a_message():
    b = wl.config_batch(1)
    good = params_for(b)
    pod.pod_attn_plan_create(good, b.seq_meta).close()

    def expect(status, prm=None, meta=None):
        with pytest.raises(pod.PodError) as e:
            pod.pod_attn_plan_create(prm or params_for(b), b.seq_meta if meta is None else meta)
        assert e.value.status == status, str(e.value)
        assert len(str(e.value)) > 20

    expect(-1, params_for(b, n_kv_heads=3))
    expect(-2, params_for(b, head_dim=96))
    expect(-2, params_for(b, head_dim=256, n_q_heads=64, n_kv_heads=4))        # 16 query heads per K/V head at 256 channels
    expect(-2, params_for(b, dtype=5))
    expect(-2, params_for(b, n_q_heads=32, n_kv_heads=1))          # 32 query heads on one K/V head
    expect(-1, params_for(b, softmax_scale=0.0))
    expect(-1, params_for(b, softmax_scale=float("nan")))
    expect(-1, params_for(b, kv_seq_stride=0))
    expect(-1, params_for(b, kv_order=2))
    expect(-1, params_for(b, kv_seq_stride=b.kv_seq_stride + 4))                                 # rows off 16 bytes
    expect(-1, params_for(b, kv_order=pod.KV_HEAD_MAJOR, kv_seq_stride=b.kv_seq_stride + 8))   # no whole token count
    pod.pod_attn_plan_create(params_for(b, kv_order=pod.KV_HEAD_MAJOR), b.seq_meta).close()
    expect(-1, params_for(b, block_size=16, max_blocks_per_seq=0))
    for col, val in [(1, 0), (2, 100), (3, 99), (0, -1)]:          # q_len 0; kv_len < q_len; row; q_start
        m = b.seq_meta.copy()
        m[0, col] = val
        expect(-1, meta=m)
    m = b.seq_meta.copy()
    m[b.n_prefill, 1] = 2                                             # a decode with two query tokens
    expect(-1, meta=m)
    m = b.seq_meta.copy()
    m[b.n_prefill + 1, 0] = m[b.n_prefill, 0]                        # two decodes on one output row
    expect(-1, meta=m)
    m = b.seq_meta.copy()
    m[0, 2] = 513                                                     # longer than the cache slot
    expect(-1, meta=m)
    m = b.seq_meta.copy()
    m[0, 0] = 5                                                       # prefill rows must tile [0, sum q_len)
    expect(-1, meta=m)


def test_forward_rejects_missing_buffers_without_touching_the_gpu():
    b = wl.config_batch(1)
    plan = pod.pod_attn_plan_create(params_for(b), b.seq_meta)
    with pytest.raises(pod.PodError) as e:
        pod.pod_attn_forward(0, 0, 0, 0, 0, 0, 0, plan, 0, 0)
    assert e.value.status == -1
    with pytest.raises(pod.PodError) as e:
        pod.pod_attn_forward(8, 8, 8, 8, 8, 0, 8, plan, 0, 0)
    assert e.value.status == -3
    with pytest.raises(pod.PodError) as e:
        pod.pod_attn_forward(8, 8, 8, 8, 8, 0, 8, plan, 256, 1 << 30, mode=9)
    assert e.value.status == -1
    with pytest.raises(pod.PodError) as e:                     # rows must be 16-byte aligned: rejected before any launch
        pod.pod_attn_forward(8, 8, 8, 8, 8, 0, 8, plan, 256, 1 << 30)
    assert e.value.status == -1 and "aligned" in str(e.value)
    plan.close()


def test_static_scratch_entry_point_checks_sizes_before_touching_the_gpu():
    """`pod_attn_forward_static` refuses a plan whose workspace exceeds its fixed array, and the
    two-stream mode, with a message and without any device call (this runs without a GPU)."""
    meta = np.zeros((512, 4), dtype=np.int32)
    meta[:, 0] = np.arange(512)
    meta[:, 1] = 1
    meta[:, 2] = 16384
    meta[:, 3] = np.arange(512)
    prm = pod.make_params(n_prefill=0, n_decode=512, n_q_heads=32, n_kv_heads=8, head_dim=128, dtype=wl.BF16,
                          softmax_scale=128 ** -0.5, block_size=16, max_blocks_per_seq=1024, n_cache_rows=512,
                          n_blocks=1 << 20, decode_chunk=256, n_compute_units=256)
    plan = pod.pod_attn_plan_create(prm, meta)
    assert pod.pod_attn_workspace_size(plan) > pod.STATIC_SCRATCH_BYTES
    with pytest.raises(pod.PodError) as e:
        pod.pod_attn_forward_static(0, 256, 256, 256, 256, 256, 256, plan)
    assert e.value.status == -3 and str(pod.STATIC_SCRATCH_BYTES) in str(e.value)
    plan.close()
    b = wl.config_batch(1)
    plan = pod.pod_attn_plan_create(params_for(b), b.seq_meta)
    with pytest.raises(pod.PodError) as e:
        pod.pod_attn_forward_static(256, 256, 256, 256, 256, 0, 256, plan, mode=pod.MODE_STREAMS)
    assert e.value.status == -2
    with pytest.raises(pod.PodError) as e:                       # null buffers are caught as in pod_attn_forward
        pod.pod_attn_forward_static(0, 0, 0, 0, 0, 0, 0, plan)
    assert e.value.status == -1
    header = open(os.path.join(ROOT, "include", "pod_attn.h")).read()
    assert "#define POD_ATTN_STATIC_SCRATCH_BYTES ((size_t)64 << 20)" in header and pod.STATIC_SCRATCH_BYTES == 64 << 20
    plan.close()


def test_prefill_heavy_flag_is_checked_before_touching_the_gpu():
    """The prefill-heavy configuration goes with the fused mode (or one operation alone), not with
    the CTA-parallel launch, and only with the shapes its kernels are built for; the entry point
    that allocates nothing refuses it, as it refuses the two-stream mode (runs without a GPU)."""
    heavy = pod.MODE_FLAG_PREFILL_HEAVY
    b = wl.config_batch(1)                                       # head_dim 64: not built
    plan = pod.pod_attn_plan_create(params_for(b), b.seq_meta)
    ws = pod.pod_attn_workspace_size(plan)
    args = (256, 256, 256, 256, 256, 0, 256, plan, 256, ws)
    for mode, status in [(pod.MODE_FUSED | heavy | pod.MODE_FLAG_CTA_PARALLEL, -1), (pod.MODE_SERIAL | heavy, -1),
                         (pod.MODE_STREAMS | heavy, -1), (pod.MODE_FUSED | heavy, -2), (pod.MODE_DECODE_ONLY | heavy, -2)]:
        with pytest.raises(pod.PodError) as e:
            pod.pod_attn_forward(*args, mode)
        assert e.value.status == status, (mode, str(e.value))
    plan.close()
    meta = np.array([[0, 64, 64, 0], [0, 1, 100, 1]], dtype=np.int32)
    for block_size, ok in [(0, True), (16, True), (64, True), (8, False), (48, False)]:
        prm = pod.make_params(n_prefill=1, n_decode=1, n_q_heads=8, n_kv_heads=2, head_dim=128, dtype=wl.F16,
                              softmax_scale=128 ** -0.5, block_size=block_size, max_blocks_per_seq=16 if block_size else 0,
                              n_cache_rows=2, n_blocks=64 if block_size else 0, kv_seq_stride=0 if block_size else 128 * 2 * 128,
                              n_compute_units=256)
        plan = pod.pod_attn_plan_create(prm, meta)
        with pytest.raises(pod.PodError) as e:                   # the static entry point: refused whatever the shape
            pod.pod_attn_forward_static(256, 256, 256, 256, 256, 256 if block_size else 0, 256, plan, mode=pod.MODE_FUSED | heavy)
        assert e.value.status == -2
        if not ok:
            with pytest.raises(pod.PodError) as e:
                pod.pod_attn_forward(256, 256, 256, 256, 256, 256, 256, plan, 256, pod.pod_attn_workspace_size(plan),
                                     pod.MODE_FUSED | heavy)
            assert e.value.status == -2 and "head_dim 128" in str(e.value)
        plan.close()


def test_workgroup_order_of_prefill_items_keeps_a_kv_head_on_its_xcds():
    """The stand-alone prefill kernels run item b of a second table in workgroup b, and the hardware
    deals workgroups to the eight XCDs round-robin: the table must hold every item exactly once, and
    the workgroups of one XCD (b % 8 equal) must work on as few K/V heads as the batch allows."""
    cases = [(32, 4, 2048, 32768, 1), (32, 32, 1024, 4096, 4), (32, 8, 512, 8192, 1), (8, 2, 300, 1000, 2)]
    for hq, hkv, q_len, kv_len, heads_per_xcd in cases:
        meta = np.array([[0, q_len, kv_len, 0], [0, 1, 777, 1]], dtype=np.int32)
        prm = pod.make_params(n_prefill=1, n_decode=1, n_q_heads=hq, n_kv_heads=hkv, head_dim=128, dtype=wl.BF16,
                              softmax_scale=128 ** -0.5, block_size=16, max_blocks_per_seq=kv_len // 16 + 1,
                              n_cache_rows=2, n_blocks=2 * (kv_len // 16 + 1), n_compute_units=256, max_prefill_waves=2)
        plan = pod.pod_attn_plan_create(prm, meta)
        items, by_wg = plan.prefill_items(), plan.prefill_items_by_workgroup()
        assert sorted(map(tuple, items.tolist())) == sorted(map(tuple, by_wg.tolist()))
        for x in range(8):
            heads = np.unique(by_wg[x::8, 1])
            assert len(heads) <= heads_per_xcd, (hq, hkv, x, heads)
        with pytest.raises(pod.PodError):
            pod.pod_attn_plan_prefill_item_of_workgroup(plan, len(items))
        plan.close()


def test_planner_advises_the_prefill_heavy_configuration_where_prefill_outweighs_decode():
    """Section 4.2.2 picks the occupancy configuration per batch.  Here the plan says which one suits
    the batch (matrix time of the prefill above 1.2 x the byte time of the K/V stream, and a shape
    the configuration is built for); of the benchmark batches that is the MFMA-bound one only."""
    advised = {}
    rng = np.random.Generator(np.random.PCG64(5))
    shapes = {(2, 0): meta_only("c2", [(1024, 4096)], [4096] * 64, hq=32, hkv=32, block_size=0),
              (3, 0): meta_only("c3", [(512, 8192)], rng.integers(2048, 16385, size=128).tolist()),
              (4, 0): meta_only("c4", [(2048, 32768)], [32768] * 32, hq=32, hkv=4)}
    for i, (chunk, nd) in enumerate(wl.RATIO_SWEEP):
        shapes[(5, i)] = meta_only("c5", [(chunk, 4096)], rng.integers(4096, 16385, size=nd).tolist())
    for key, (prm, meta) in shapes.items():
        plan = pod.pod_attn_plan_create(prm, meta)
        advised[key] = plan.info().prefill_heavy_advised
        plan.close()
    assert advised[(4, 0)] == 1
    assert all(v == 0 for k, v in advised.items() if k != (4, 0))
    # the same shape with 64 channels is not built, and a batch without decodes has nothing to co-run
    meta = np.array([[0, 2048, 32768, 0], [0, 1, 4096, 1]], dtype=np.int32)
    base = dict(n_prefill=1, n_decode=1, n_q_heads=32, n_kv_heads=4, head_dim=128, dtype=wl.BF16, softmax_scale=0.1,
                block_size=16, max_blocks_per_seq=2049, n_cache_rows=2, n_blocks=4200, n_compute_units=256)
    for change, want in [({}, 1), ({"head_dim": 64}, 0), ({"block_size": 48, "max_blocks_per_seq": 700}, 0),
                         ({"n_decode": 0}, 0)]:
        prm = pod.make_params(**{**base, **change})
        plan = pod.pod_attn_plan_create(prm, meta[: prm.n_prefill + prm.n_decode])
        assert plan.info().prefill_heavy_advised == want, change
        plan.close()


# -- planner: every (row, key) pair and every decode token is covered exactly once --------------- #
def coverage_check(prm, meta):
    plan = pod.pod_attn_plan_create(prm, meta)
    info = plan.info()
    group = prm.n_q_heads // prm.n_kv_heads
    items, units = plan.prefill_items(), plan.decode_units()
    assert len(items) == info.n_prefill_items and len(units) == info.n_decode_units
    # decode workers are persistent: at most one per compute unit, never more than a wave per unit
    n_workers = min(info.n_compute_units, (len(units) + 3) // 4)
    full_round = n_workers == info.n_compute_units and len(items) > 0
    assert info.fused_grid == (2 * info.n_compute_units if full_round
                               else min(2 * info.n_compute_units, len(items) + n_workers))
    # prefill: per (request, kv head, row block) the key ranges tile [0, kmax) without gaps
    item_rows, tile = (64, 32) if prm.head_dim == 256 else (128, 64)       # shape of a prefill item by head_dim
    blocks = {}
    for req, kvh, row0, n_rows, k0, k1, prow0, split in items:
        assert row0 % item_rows == 0 and 1 <= n_rows <= item_rows and k0 % tile == 0 and k0 < k1
        blocks.setdefault((req, kvh, row0, n_rows), []).append((k0, k1, prow0, split))
    want_blocks = 0
    for r in range(prm.n_prefill):
        q_len, kv_len = int(meta[r, 1]), int(meta[r, 2])
        rows = q_len * group
        for kvh in range(prm.n_kv_heads):
            for row0 in range(0, rows, item_rows):
                n_rows = min(item_rows, rows - row0)
                kmax = kv_len - q_len + (row0 + n_rows - 1) // group + 1
                parts = sorted(blocks[(r, kvh, row0, n_rows)])
                assert parts[0][0] == 0 and parts[-1][1] == kmax
                for a, b in zip(parts, parts[1:]):
                    assert a[1] == b[0]
                assert all((p[2] >= 0) == (len(parts) > 1) for p in parts)
                assert sorted(p[3] for p in parts) == list(range(len(parts)))
                want_blocks += 1
    assert len(blocks) == want_blocks
    # decode: token ranges tile [0, kv_len)
    ranges = {}
    for req, kvh, t0, t1, prow0, split, _, _ in units:
        assert t0 % 16 == 0 and t0 < t1
        ranges.setdefault((req, kvh), []).append((t0, t1, prow0))
    for r in range(prm.n_prefill, prm.n_prefill + prm.n_decode):
        for kvh in range(prm.n_kv_heads):
            parts = sorted(ranges[(r, kvh)])
            assert parts[0][0] == 0 and parts[-1][1] == int(meta[r, 2])
            for a, b in zip(parts, parts[1:]):
                assert a[1] == b[0]
            assert all((p[2] >= 0) == (len(parts) > 1) for p in parts)
    assert len(ranges) == prm.n_decode * prm.n_kv_heads
    # partial rows do not overlap
    spans = [(p, p + item_rows) for *_, p, _ in [tuple(i) for i in items] if p >= 0]
    spans += [(int(u[4]), int(u[4]) + group) for u in units if u[4] >= 0]
    spans.sort()
    for a, b in zip(spans, spans[1:]):
        assert a[1] <= b[0]
    assert (spans[-1][1] if spans else 0) <= info.n_partial_rows
    # prefill items: one queue per XCD ((request, K/V head) stream modulo 8; with fewer streams than
    # queues a stream's row blocks are dealt over 8 / streams queues), queues in order, longest
    # first inside a queue
    n_streams = prm.n_prefill * prm.n_kv_heads
    per = 8 // n_streams if 0 < n_streams < 8 else 1
    queues = [(int(i[0] * prm.n_kv_heads + i[1]) * per + (int(i[2]) // item_rows) % per) % 8 for i in items]
    assert queues == sorted(queues)
    for q in set(queues):
        lens = [int(i[5] - i[4]) for i, qq in zip(items, queues) if qq == q]
        assert lens == sorted(lens, reverse=True)
    # decode units: fixed first units (four per seat, at most one seat per compute unit), then 8
    # queues that tile the rest; longest first inside each range, and no fixed unit is shorter
    # than a queued one
    lens = [int(u[3] - u[2]) for u in units]
    queues_d = plan.decode_queues()
    n_fixed = queues_d[0][0]
    assert n_fixed == 4 * min(info.n_compute_units, len(units) // 4)
    assert lens[:n_fixed] == sorted(lens[:n_fixed], reverse=True)
    at = n_fixed
    for b, e in queues_d:
        assert b == at and e >= b
        assert lens[b:e] == sorted(lens[b:e], reverse=True)
        at = e
    assert at == len(units)
    if n_fixed and n_fixed < len(units):
        assert min(lens[:n_fixed]) >= max(lens[n_fixed:])
    sizes = [e - b for b, e in queues_d]
    assert max(sizes) - min(sizes) <= 1
    # every unit carries its request's first query row and cache row
    for u in units:
        assert int(u[6]) == int(meta[u[0], 0]) and int(u[7]) == int(meta[u[0], 3])
    assert pod.pod_attn_workspace_size(plan) == info.workspace_bytes >= 4352
    plan.close()
    return info


@pytest.mark.parametrize("config,index", [(1, 0), (5, 0), (5, 11)])
def test_plan_covers_small_benchmark_batches(config, index):
    b = wl.config_batch(config, index) if config == 1 else None
    if b is not None:
        coverage_check(params_for(b), b.seq_meta)
        return
    chunk, nd = wl.RATIO_SWEEP[index]
    rng = np.random.Generator(np.random.PCG64(index))
    prm, meta = meta_only("sweep", [(chunk, 4096)], rng.integers(4096, 16385, size=nd).tolist())
    coverage_check(prm, meta)


def test_plan_shapes_for_the_large_configs():
    # config 2: 32 heads x 8 row blocks = 256 items.  With a decode worker on every unit the items fill
    # the other slots once: no split; asked for two rounds, 512 items in 2 splits of >= 1024 keys
    prm, meta = meta_only("c2", [(1024, 4096)], [4096] * 64, hq=32, hkv=32, block_size=0)
    info = coverage_check(prm, meta)
    assert info.n_prefill_items == 256 and info.max_prefill_splits == 1
    assert info.n_decode_units == 64 * 32 * info.max_decode_splits
    prm.max_prefill_waves = 2
    info = coverage_check(prm, meta)
    assert info.n_prefill_items == 512 and info.max_prefill_splits == 2
    # the same chunk with little decode work beside it: two rounds by default
    prm, meta = meta_only("c2-few", [(1024, 4096)], [4096] * 2, hq=32, hkv=32, block_size=0)
    info = coverage_check(prm, meta)
    assert info.n_prefill_items == 512 and info.max_prefill_splits == 2
    # config 4: 4 kv heads x 128 row blocks = 512 items = two rounds -> no split (Section 4.2.4)
    prm, meta = meta_only("c4", [(2048, 32768)], [32768] * 32, hq=32, hkv=4)
    info = coverage_check(prm, meta)
    assert info.n_prefill_items == 512 and info.max_prefill_splits == 1
    # config 3: 128 row blocks -> 2 splits (256 items) beside its decodes, 4 (512 items) in two rounds
    prm, meta = meta_only("c3", [(512, 8192)], [9000] * 128, hq=32, hkv=8)
    info = coverage_check(prm, meta)
    assert info.max_prefill_splits == 2 and info.n_prefill_items <= 256
    prm.max_prefill_waves = 2
    info = coverage_check(prm, meta)
    assert info.max_prefill_splits == 4 and info.n_prefill_items <= 512


def test_split_cap_follows_max_prefill_waves():
    """Section 4.2.4: prefill work items fill at most `max_prefill_waves` chip-wide rounds."""
    prm, meta = meta_only("cap", [(256, 8192)], [4096] * 8)
    for waves, limit in [(1, 256), (2, 512), (4, 1024)]:
        prm.max_prefill_waves = waves
        prm.prefill_split_len = 64
        info = coverage_check(prm, meta)
        assert info.n_prefill_items <= limit
        assert info.n_prefill_items > limit // 2


def test_ragged_and_degenerate_batches_plan_cleanly():
    for prefill, decodes in [([], [1]), ([(1, 1)], []), ([(129, 129), (7, 4000)], [1, 31, 33, 5000]),
                             ([(2048, 2048)], [])]:
        prm, meta = meta_only("rag", prefill, decodes, hq=8, hkv=2)
        coverage_check(prm, meta)
    prm, meta = meta_only("empty", [], [])
    plan = pod.pod_attn_plan_create(prm, np.zeros((0, 4), dtype=np.int32))
    assert plan.info().fused_grid == 0
    plan.close()


def test_random_batches_and_tuning_values_plan_cleanly():
    """120 seeded random batches (0..5 chunks, 0..60 decodes, lengths 1..20000, 1..16 heads per
    group) under random tuning values and chip sizes: every plan passes the coverage check."""
    rng = np.random.Generator(np.random.PCG64(20241018))
    for case in range(120):
        n_p, n_d = int(rng.integers(0, 6)), int(rng.integers(0, 61))
        if n_p + n_d == 0:
            n_d = 1
        top = int(rng.choice([40, 700, 20000]))
        prefill = []
        for _ in range(n_p):
            kv = int(rng.integers(1, top + 1))
            prefill.append((int(rng.integers(1, min(kv, 3000) + 1)), kv))
        decodes = rng.integers(1, top + 1, n_d).tolist()
        hkv = int(rng.choice([1, 2, 3, 5, 8]))
        group = int(rng.choice([1, 2, 3, 4, 8, 16]))
        prm, meta = meta_only(f"rand{case}", prefill, decodes, hq=hkv * group, hkv=hkv,
                              d=int(rng.choice([64, 128, 256])) if group <= 8 else int(rng.choice([64, 128])),
                              block_size=int(rng.choice([0, 16])))
        prm.n_compute_units = int(rng.choice([1, 2, 7, 64, 256, 304]))
        prm.decode_chunk = int(rng.choice([0, 0, 16, 100, 256, 4096]))
        prm.prefill_split_len = int(rng.choice([0, 0, 64, 300, 1 << 20]))
        prm.max_prefill_waves = int(rng.choice([0, 1, 2, 64]))
        prm.policy = int(rng.integers(0, 3))
        coverage_check(prm, meta)


# -- role ratio and the binder model -------------------------------------------------------------- #
def read_golden(name):
    rows = []
    for line in open(os.path.join(GOLDEN, name)):
        line = line.split("#")[0].strip()
        if line:
            rows.append(line.split())
    return rows


def test_proportional_policy_reproduces_the_papers_example():
    """Section 5.4.2: 50 prefill and 100 decode CTAs give the per-unit order prefill, decode, decode."""
    (n_p, n_d, pattern), = read_golden("policy_example.txt")
    n_p, n_d = int(n_p), int(n_d)
    prm, meta = meta_only("pol", [(128 * n_p // 2, 128 * n_p // 2)], [256] * (n_d * 4 // 2), hq=2, hkv=2,
                          block_size=0)
    prm.decode_chunk = 256
    prm.prefill_split_len = 1 << 20          # one item per row block
    prm.policy = pod.POLICY_PROPORTIONAL
    plan = pod.pod_attn_plan_create(prm, meta)
    info = plan.info()
    assert (info.n_prefill_items, (info.n_decode_units + 3) // 4) == (n_p, n_d)
    assert (info.prefill_ratio, info.decode_ratio) == (1, 2)
    plan.close()
    # the automatic policy never starts more decode than prefill workgroups on a unit (a unit seats
    # one decode worker), but follows the proportion when prefill is the larger side
    prm.policy = pod.POLICY_AUTO
    plan = pod.pod_attn_plan_create(prm, meta)
    assert (plan.info().prefill_ratio, plan.info().decode_ratio) == (1, 1)
    plan.close()
    # all arrivals on one compute unit: their first operations follow the printed pattern
    roles = [pod.pod_attn_role_for_ticket(t, 1, 2, 0) for t in range(12)]
    assert "".join("PD"[r] for r in roles) == pattern * 4
    # 50:50 alternates
    prm.policy = pod.POLICY_ALTERNATE
    plan = pod.pod_attn_plan_create(prm, meta)
    assert (plan.info().prefill_ratio, plan.info().decode_ratio) == (1, 1)
    plan.close()
    assert "".join("PD"[pod.pod_attn_role_for_ticket(t, 1, 1, 0)] for t in range(6)) == "PDPDPD"
    assert pod.pod_attn_role_for_ticket(-1, 1, 1, 0) == -1 and pod.pod_attn_role_for_ticket(0, 0, 0, 0) == -1


def test_wave_quantization_example():
    """Section 3.2: 54 decodes x 4 K/V heads = 216 CTAs = two full rounds of 108 units; 55 -> 220."""
    for n_dec, heads, units, ctas, rounds in [tuple(int(x) for x in r) for r in read_golden("wave_quantization.txt")]:
        assert n_dec * heads == ctas
        assert -(-ctas // units) == rounds
        prm, meta = meta_only("wq", [], [16384] * n_dec, hq=32, hkv=heads)
        prm.decode_chunk = 16384
        plan = pod.pod_attn_plan_create(prm, meta)
        assert plan.info().n_decode_units == ctas          # one unit per (request, K/V head)
        plan.close()


def hardware_units(n_cus):
    """Hardware unit ids as the device reports them: xcc << 6 | se << 4 | cu, 8 XCDs."""
    per_xcd = max(1, -(-n_cus // 8))
    return [((i // per_xcd) % 8) << 6 | ((i % per_xcd) // 8) << 4 | (i % per_xcd) % 8 for i in range(n_cus)]


def launch_model_check(plan, placement, order):
    info = plan.info()
    steps, first, seat, items, units = pod.pod_attn_simulate_launch(plan, placement, order)
    assert steps >= 0, "a work id was handed out twice" if steps == -2 else "bad arguments"
    assert (items >= 0).all() and (items < len(placement)).all(), "a prefill item was never claimed"
    assert (units >= 0).all() and (units < 4 * len(placement)).all(), "a decode unit was never claimed"
    assert set(first.tolist()) <= {0, 1}
    # seats are handed out once each, and the first seats (which carry the fixed units) are all taken
    taken = sorted(x for x in seat.tolist() if x >= 0)
    assert taken == list(range(len(taken)))
    n_workers = min(info.n_compute_units, (info.n_decode_units + 3) // 4)
    assert len(taken) >= min(n_workers, len(placement)) or info.n_decode_units == 0
    # a fixed unit 4*s + v is run by wavefront v of the workgroup on seat s
    n_fixed = plan.decode_queues()[0][0]
    wg_of_seat = {int(x): w for w, x in enumerate(seat.tolist()) if x >= 0}
    for u in range(n_fixed):
        assert units[u] == 4 * wg_of_seat[u // 4] + u % 4
    return first, seat, items, units


@pytest.mark.parametrize("seed", range(8))
def test_device_claim_protocol_hands_out_every_work_id_exactly_once(seed):
    """The protocol the fused kernel runs (ticket, decode seats with fixed first units, per-XCD queues
    with a walk over the other queues, one switch of operation), under random placements of the
    workgroups on hardware units and random interleavings of their steps: every prefill item and
    every decode unit is run exactly once and the launch drains (Section 4.1: the scheme does not
    depend on how the hardware places workgroups)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    n_cus = int(rng.choice([1, 3, 64, 256]))
    n_p, n_d = int(rng.integers(0, 4)), int(rng.integers(0, 50))
    if n_p + n_d == 0:
        n_d = 3
    prefill = [(int(q), int(q + pre)) for q, pre in zip(rng.integers(1, 1500, n_p), rng.integers(0, 6000, n_p))]
    decodes = rng.integers(1, 9000, n_d).tolist()
    hkv = int(rng.choice([1, 2, 8]))
    prm, meta = meta_only(f"model{seed}", prefill, decodes, hq=hkv * int(rng.choice([1, 4])), hkv=hkv)
    prm.n_compute_units = n_cus
    prm.decode_chunk = int(rng.choice([0, 64, 512]))
    prm.policy = int(rng.integers(0, 3))
    plan = pod.pod_attn_plan_create(prm, meta)
    grid = plan.info().fused_grid
    hw = hardware_units(n_cus)
    for trial in range(4):
        # placements: two per unit in order; random units (some crowded, some empty); all on one unit
        if trial == 0:
            placement = [hw[(w // 2) % n_cus] for w in range(grid)]
        elif trial == 3:
            placement = [hw[0]] * grid
        else:
            placement = [hw[int(rng.integers(n_cus))] for _ in range(grid)]
        # interleavings: none (pure round-robin drain), or a long random sequence of actors, or
        # one straggler workgroup that only moves when everybody else is done
        if trial == 0:
            order = []
        elif trial == 1:
            order = rng.integers(0, 4 * max(grid, 1), size=20000).tolist()
        else:
            order = [a for a in rng.integers(0, 4 * max(grid, 1), size=20000).tolist() if a // 4 != 0]
        launch_model_check(plan, placement, order)
    plan.close()


def test_every_unit_gets_one_workgroup_of_each_operation():
    """With two workgroups per unit and a 1:1 ratio (what the automatic policy plans for every
    benchmark batch) each unit's two tickets give it one prefill-first and one decode-first
    workgroup, whichever arrives first; the decode-first ones take the seats."""
    prm, meta = meta_only("c2", [(1024, 4096)], [4096] * 64, hq=32, hkv=32, block_size=0)
    plan = pod.pod_attn_plan_create(prm, meta)
    info = plan.info()
    assert (info.prefill_ratio, info.decode_ratio, info.fused_grid) == (1, 1, 512)
    hw = hardware_units(256)
    rng = np.random.Generator(np.random.PCG64(5))
    placement = [hw[w % 256] for w in range(512)]          # the hardware deals round-robin
    first, seat, items, units = launch_model_check(plan, placement, rng.integers(0, 2048, size=50000).tolist())
    for u in range(256):
        assert sorted([int(first[u]), int(first[u + 256])]) == [0, 1]
    # decode-first workgroups hold all 256 seats unless a prefill-first one ran out of items earlier
    assert (seat >= 0).all()
    plan.close()


def test_decode_last_piece_is_cut_into_half_and_quarters():
    """The last piece of a split request is cut again (half, quarter, quarter) while the quarters
    stay at least 128 keys; a request that fits one piece stays whole; cuts are multiples of 16."""
    prm, meta = meta_only("taper", [], [4096, 1000, 4090, 600], hq=8, hkv=1)
    prm.decode_chunk = 2048
    plan = pod.pod_attn_plan_create(prm, meta)
    pieces = {}
    for req, kvh, t0, t1, prow0, split, _, _ in plan.decode_units():
        pieces.setdefault(int(req), []).append((int(t0), int(t1), int(prow0)))
    got = {r: sorted(p) for r, p in pieces.items()}
    assert [(a, b) for a, b, _ in got[0]] == [(0, 2048), (2048, 3072), (3072, 3584), (3584, 4096)]
    assert [(a, b) for a, b, _ in got[1]] == [(0, 1000)] and got[1][0][2] == -1
    assert [(a, b) for a, b, _ in got[2]] == [(0, 2048), (2048, 3056), (3056, 3568), (3568, 4090)]
    assert [(a, b) for a, b, _ in got[3]] == [(0, 600)]
    prm.decode_chunk = 512                       # last piece of 88 keys: too short to cut again
    plan2 = pod.pod_attn_plan_create(prm, meta)
    last = sorted((int(u[2]), int(u[3])) for u in plan2.decode_units() if u[0] == 3)
    assert last == [(0, 304), (304, 600)]
    plan.close(); plan2.close()


def test_binder_spreads_a_long_pattern_over_the_units():
    """A unit holds two workgroups, so unit u counts its tickets from 2u: with 4 prefill : 1 decode
    every fifth slot of the chip starts in the decode operation, and with 1 : 1 every unit still
    gets one of each (Section 4.1's ticket rule, applied chip-wide)."""
    n_units = 40
    slots = [pod.pod_attn_role_for_ticket(t, 4, 1, u) for u in range(n_units) for t in range(2)]
    assert slots == [0 if s % 5 < 4 else 1 for s in range(2 * n_units)]
    for u in range(n_units):
        assert sorted(pod.pod_attn_role_for_ticket(t, 1, 1, u) for t in range(2)) == [0, 1]


def test_event_log_and_queue_arguments_are_checked():
    """Host-side checks only (no GPU call): the event log must be 16-byte aligned and hold at least
    one record; a decode queue index must be 0..7."""
    prm, meta = meta_only("args", [(64, 64)], [100, 200])
    plan = pod.pod_attn_plan_create(prm, meta)
    with pytest.raises(pod.PodError):
        pod.pod_attn_plan_set_event_log(plan, 4096, 40)          # too small
    with pytest.raises(pod.PodError):
        pod.pod_attn_plan_set_event_log(plan, 4096 + 8, 4096)    # misaligned
    pod.pod_attn_plan_set_event_log(plan, 4096, 4096)            # accepted (never dereferenced here)
    pod.pod_attn_plan_set_event_log(plan, 0, 0)                  # off again
    for q in (-1, 8):
        with pytest.raises(pod.PodError):
            pod.pod_attn_plan_decode_queue(plan, q)
    assert len(plan.decode_queues()) == 8
    plan.close()
