"""The entry point that allocates nothing (`pod_attn_forward_static`) against `pod_attn_forward`.

Both run the same kernels; the only difference is where counters, work tables and split-KV partials
live (the library's static device array instead of a caller workspace), so the outputs must agree
bit for bit, which is stricter than the parity tolerance.  Collected last on purpose.
"""
import numpy as np
import pytest
import torch

from paper_2410_18038_amd import pod
from paper_2410_18038_amd import workloads as wl
from tests.helpers import oracle_out

TOL = {wl.F16: 2e-3, wl.BF16: 1e-2}


def _ptr(t):
    return 0 if t is None or t.numel() == 0 else t.data_ptr()


def _static(batch, attn, out, mode=pod.MODE_FUSED):
    pod.pod_attn_forward_static(_ptr(batch.prefill_q), _ptr(batch.decode_q), _ptr(batch.k_cache), _ptr(batch.v_cache),
                                attn.seq_meta_dev.data_ptr(), _ptr(batch.block_table), out.data_ptr(), attn.plan,
                                mode, torch.cuda.current_stream().cuda_stream)


@pytest.mark.gpu
def test_static_scratch_entry_point_matches_the_workspace_one():
    """Two calls in a row on the shared static array, the second with a smaller batch (fewer
    counters in use, shorter tables, fewer partial rows: whatever the first call left behind must
    not matter), then the first batch again, then the serial mode; each against the workspace entry
    point bit for bit, and the first also against the oracle."""
    big = wl.make_batch("static-big", prefill=[(300, 1500), (40, 40)], decode_kv_lens=[1200, 90, 2047, 640] * 20,
                        n_q_heads=8, n_kv_heads=2, head_dim=128, dtype=wl.BF16, seed=4100, block_size=16,
                        poison=float("nan")).to("cuda:0")
    small = wl.make_batch("static-small", prefill=[(50, 333)], decode_kv_lens=[700, 31, 257],
                          n_q_heads=4, n_kv_heads=4, head_dim=64, dtype=wl.F16, seed=4101,
                          poison=float("nan")).to("cuda:0")
    kw = dict(decode_chunk=256, prefill_split_len=256, max_prefill_waves=64)     # split-KV in both operations
    runs = []
    for batch in (big, small):
        attn = pod.HybridAttention(batch, **kw)
        assert attn.info.max_decode_splits > 1 and attn.info.n_partial_rows > 0
        assert attn.ws_bytes <= pod.STATIC_SCRATCH_BYTES
        runs.append((batch, attn, attn.forward(batch).clone()))
    torch.cuda.synchronize()
    for step, (which, mode) in enumerate([(0, pod.MODE_FUSED), (1, pod.MODE_FUSED), (0, pod.MODE_FUSED),
                                          (0, pod.MODE_FUSED), (1, pod.MODE_SERIAL), (0, pod.MODE_DECODE_ONLY)]):
        batch, attn, want = runs[which]
        print(f"step {step}: {batch.name} mode {mode}", flush=True)
        out = torch.full_like(want, float("nan"))
        _static(batch, attn, out, mode)
        torch.cuda.synchronize()
        if mode == pod.MODE_DECODE_ONLY:
            npr = batch.n_prefill_rows
            assert torch.equal(out[npr:].view(torch.int16), want[npr:].view(torch.int16))
            assert bool(torch.isnan(out[:npr].to(torch.float32)).all())
        else:
            assert torch.equal(out.view(torch.int16), want.view(torch.int16)), f"step {step}"
    batch, attn, want = runs[0]
    err = np.abs(want.to(torch.float64).cpu().numpy() - oracle_out(batch)).max()
    assert err <= TOL[batch.dtype]
    # the workspace entry point still works after the static one, on its own workspace
    again = attn.forward(batch)
    assert torch.equal(again.view(torch.int16), want.view(torch.int16))
    for _, attn, _ in runs:
        attn.close()


@pytest.mark.gpu
def test_static_scratch_entry_point_rejects_what_it_cannot_hold():
    """A batch whose workspace exceeds the static array, and the two-stream mode, are refused with a
    message before anything is launched; a later valid call is not affected."""
    lens = [16384] * 512
    batch_meta = np.zeros((512, 4), dtype=np.int32)
    batch_meta[:, 0] = np.arange(512)
    batch_meta[:, 1] = 1
    batch_meta[:, 2] = lens
    batch_meta[:, 3] = np.arange(512)
    prm = pod.make_params(n_prefill=0, n_decode=512, n_q_heads=32, n_kv_heads=8, head_dim=128, dtype=wl.BF16,
                          softmax_scale=128 ** -0.5, block_size=16, max_blocks_per_seq=1024, n_cache_rows=512,
                          n_blocks=1 << 20, decode_chunk=256, n_compute_units=256)
    plan = pod.pod_attn_plan_create(prm, batch_meta)
    assert pod.pod_attn_workspace_size(plan) > pod.STATIC_SCRATCH_BYTES
    with pytest.raises(pod.PodError) as e:
        pod.pod_attn_forward_static(0, 256, 256, 256, 256, 256, 256, plan)
    assert e.value.status == -3 and str(pod.STATIC_SCRATCH_BYTES) in str(e.value)
    plan.close()
    small = wl.make_batch("static-ok", prefill=[(20, 100)], decode_kv_lens=[64, 300], n_q_heads=4, n_kv_heads=2,
                          head_dim=64, dtype=wl.F16, seed=4102).to("cuda:0")
    attn = pod.HybridAttention(small)
    want = attn.forward(small).clone()
    out = torch.zeros_like(want)
    with pytest.raises(pod.PodError) as e:
        _static(small, attn, out, pod.MODE_STREAMS)
    assert e.value.status == -2
    _static(small, attn, out)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), want.view(torch.int16))
    attn.close()
