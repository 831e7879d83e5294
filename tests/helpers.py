"""Glue shared by the tests: run the CPU oracle on a HybridBatch."""
import numpy as np

from oracle import reference
from paper_2410_18038_amd import workloads as wl


def oracle_out(batch: wl.HybridBatch, rows=None) -> np.ndarray:
    """float64 [rows, Hq, d] from the C oracle for every row (or the listed rows)."""
    return reference.attention(
        wl.bits(batch.prefill_q), wl.bits(batch.decode_q), wl.bits(batch.k_cache),
        wl.bits(batch.v_cache), batch.seq_meta,
        None if batch.block_table is None else batch.block_table.cpu().numpy(),
        n_prefill=batch.n_prefill, n_decode=batch.n_decode, n_q_heads=batch.n_q_heads,
        n_kv_heads=batch.n_kv_heads, head_dim=batch.head_dim, dtype=batch.dtype,
        softmax_scale=batch.softmax_scale, block_size=batch.block_size,
        max_blocks_per_seq=batch.max_blocks_per_seq, kv_seq_stride=batch.kv_seq_stride,
        head_major=batch.head_major, rows=rows)


def logical_kv(batch: wl.HybridBatch, req: int):
    """float64 (K, V) of one request as [kv_len, Hkv, d], resolved through the layout."""
    _, _, kv_len, row = (int(x) for x in batch.seq_meta[req])
    if batch.head_major:
        raise ValueError("logical_kv reads token-major caches only")
    if batch.block_size > 0:
        tbl = batch.block_table.cpu().numpy()
        t = np.arange(kv_len)
        slots = tbl[row, t // batch.block_size].astype(np.int64) * batch.block_size + t % batch.block_size
        k = wl.as_f64(batch.k_cache).reshape(-1, batch.n_kv_heads, batch.head_dim)[slots]
        v = wl.as_f64(batch.v_cache).reshape(-1, batch.n_kv_heads, batch.head_dim)[slots]
    else:
        k = wl.as_f64(batch.k_cache)[row, :kv_len]
        v = wl.as_f64(batch.v_cache)[row, :kv_len]
    return k, v


def request_q(batch: wl.HybridBatch, req: int) -> np.ndarray:
    """float64 query rows of one request as [q_len, Hq, d]."""
    q_start, q_len, _, _ = (int(x) for x in batch.seq_meta[req])
    if req < batch.n_prefill:
        return wl.as_f64(batch.prefill_q)[q_start:q_start + q_len]
    return wl.as_f64(batch.decode_q)[q_start:q_start + 1]


def request_rows(batch: wl.HybridBatch, req: int) -> np.ndarray:
    """Global output row indices of one request."""
    q_start, q_len, _, _ = (int(x) for x in batch.seq_meta[req])
    if req < batch.n_prefill:
        return np.arange(q_start, q_start + q_len)
    return np.array([batch.n_prefill_rows + q_start])
