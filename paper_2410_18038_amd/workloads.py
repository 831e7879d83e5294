"""Seeded synthetic hybrid batches (inputs only: none of the attention arithmetic lives here).

A hybrid batch is what the paper's Section 2.1 and Table 1 describe: a few prefill
chunks (normally one) of ``q_len`` new tokens each, plus many decode requests with
one query token each, all reading a KV cache that already holds every token seen
so far, the new ones included.  The shapes below are the benchmark configurations
this repository is measured on (model shapes of the paper's Table 4; chunk sizes
and context lengths inside the ranges of its Section 5.1 sweep).

Both the GPU library's tests and the CPU oracle's tests draw their inputs from
here; this module imports neither of them.
"""
from __future__ import annotations

import dataclasses
import math
from typing import List, Optional, Sequence, Tuple

import numpy as np
import torch

BASE_SEED = 20241018
F16, BF16 = 0, 1
_TORCH_DTYPE = {F16: torch.float16, BF16: torch.bfloat16}


@dataclasses.dataclass
class HybridBatch:
    """One batch, with the cache in either layout.

    seq_meta: int32 [n_prefill + n_decode, 4] = (q_start, q_len, kv_len, cache_row),
    prefill requests first.  Contiguous cache: [n_seqs, max_len, Hkv, d]; paged
    cache: [n_blocks, block_size, Hkv, d] with block_table [n_seqs, max_blocks_per_seq]
    (entries past a sequence's last block are -1).  With ``head_major`` the two middle
    dimensions of either cache change places: [.., Hkv, tokens, d].
    """
    name: str
    n_prefill: int
    n_decode: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: int
    softmax_scale: float
    block_size: int
    max_blocks_per_seq: int
    kv_seq_stride: int
    n_cache_rows: int
    n_blocks: int
    max_len: int
    seq_meta: np.ndarray
    prefill_q: torch.Tensor
    decode_q: torch.Tensor
    k_cache: torch.Tensor
    v_cache: torch.Tensor
    block_table: Optional[torch.Tensor]
    head_major: bool = False

    @property
    def n_prefill_rows(self) -> int:
        return int(self.prefill_q.shape[0])

    @property
    def n_rows(self) -> int:
        return self.n_prefill_rows + self.n_decode

    @property
    def torch_dtype(self):
        return _TORCH_DTYPE[self.dtype]

    def to(self, device) -> "HybridBatch":
        kw = {f.name: getattr(self, f.name) for f in dataclasses.fields(self)}
        for key in ("prefill_q", "decode_q", "k_cache", "v_cache", "block_table"):
            if kw[key] is not None:
                kw[key] = kw[key].to(device)
        return HybridBatch(**kw)

    # --- bookkeeping used for the roofline figures (counts only) -------------
    def visible_pairs(self) -> int:
        """Sum over prefill query rows of the number of keys each one sees."""
        total = 0
        for r in range(self.n_prefill):
            _, q_len, kv_len, _ = (int(x) for x in self.seq_meta[r])
            prefix = kv_len - q_len
            total += q_len * prefix + q_len * (q_len + 1) // 2
        return total

    def prefill_flops(self) -> int:
        """4*d flops per visible (query row, key) pair per query head (QK^T and PV)."""
        return 4 * self.head_dim * self.visible_pairs() * self.n_q_heads

    def kv_bytes(self) -> int:
        """Bytes of K and V each request must read once per K/V head."""
        tokens = int(self.seq_meta[:, 2].sum())
        return tokens * self.n_kv_heads * self.head_dim * 2 * 2


def bits(t: torch.Tensor) -> np.ndarray:
    """uint16 bit patterns of a 16-bit float tensor, on the host."""
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def as_f64(t: torch.Tensor) -> np.ndarray:
    """Exact float64 copy of a 16-bit float tensor, on the host."""
    return t.detach().cpu().to(torch.float64).numpy()


def make_batch(name: str, *, prefill: Sequence[Tuple[int, int]], decode_kv_lens: Sequence[int],
               n_q_heads: int, n_kv_heads: int, head_dim: int, dtype: int, seed: int,
               block_size: int = 0, softmax_scale: Optional[float] = None,
               device="cpu", poison: Optional[float] = None, spare_blocks: int = 3,
               max_len: Optional[int] = None) -> HybridBatch:
    """Build a batch from (q_len, kv_len) prefill pairs and decode context lengths.

    Every Q, K, V element is an independent N(0,1) draw rounded to the 16-bit type.
    Cache slots that no request can see (positions >= kv_len, spare blocks) hold
    ``poison`` when given (tests use NaN), else zeros.  For the paged layout the
    block table is a seeded random permutation of all physical blocks.
    """
    tdt = _TORCH_DTYPE[dtype]
    dev = torch.device(device)
    rng = np.random.Generator(np.random.PCG64(seed))
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    if softmax_scale is None:
        softmax_scale = 1.0 / math.sqrt(head_dim)

    n_prefill, n_decode = len(prefill), len(decode_kv_lens)
    meta = np.zeros((n_prefill + n_decode, 4), dtype=np.int32)
    q_start = 0
    for r, (q_len, kv_len) in enumerate(prefill):
        meta[r] = (q_start, q_len, kv_len, r)
        q_start += q_len
    for i, kv_len in enumerate(decode_kv_lens):
        meta[n_prefill + i] = (i, 1, kv_len, n_prefill + i)
    n_seqs = n_prefill + n_decode
    kv_lens = meta[:, 2].astype(np.int64)
    longest = int(kv_lens.max()) if n_seqs else 1

    def randn(*shape):
        return torch.randn(*shape, generator=gen, device=dev, dtype=torch.float32).to(tdt)

    prefill_q = randn(q_start, n_q_heads, head_dim)
    decode_q = randn(n_decode, n_q_heads, head_dim)
    fill = 0.0 if poison is None else poison
    tok = n_kv_heads * head_dim

    if block_size > 0:
        blocks_per_seq = [(int(l) + block_size - 1) // block_size for l in kv_lens]
        n_used = int(sum(blocks_per_seq))
        n_blocks = n_used + spare_blocks
        perm = rng.permutation(n_blocks).astype(np.int32)
        max_blocks = max(blocks_per_seq) if blocks_per_seq else 1
        table = np.full((max(n_seqs, 1), max_blocks), -1, dtype=np.int32)
        at = 0
        for s, nb in enumerate(blocks_per_seq):
            table[s, :nb] = perm[at:at + nb]
            at += nb
        k_cache = torch.full((n_blocks, block_size, n_kv_heads, head_dim), fill, dtype=tdt, device=dev)
        v_cache = torch.full((n_blocks, block_size, n_kv_heads, head_dim), fill, dtype=tdt, device=dev)
        k_flat = k_cache.view(n_blocks * block_size, tok)
        v_flat = v_cache.view(n_blocks * block_size, tok)
        for s in range(n_seqs):
            n = int(kv_lens[s])
            t = np.arange(n, dtype=np.int64)
            slots = table[s, t // block_size].astype(np.int64) * block_size + t % block_size
            idx = torch.from_numpy(slots).to(dev)
            k_flat.index_copy_(0, idx, randn(n, tok))
            v_flat.index_copy_(0, idx, randn(n, tok))
        block_table = torch.from_numpy(table).to(dev)
        stride, cap = 0, max_blocks * block_size
    else:
        cap = longest if max_len is None else max(max_len, longest)
        n_blocks, max_blocks, block_table = 0, 0, None
        k_cache = torch.full((max(n_seqs, 1), cap, n_kv_heads, head_dim), fill, dtype=tdt, device=dev)
        v_cache = torch.full((max(n_seqs, 1), cap, n_kv_heads, head_dim), fill, dtype=tdt, device=dev)
        for s in range(n_seqs):
            n = int(kv_lens[s])
            k_cache[s, :n] = randn(n, n_kv_heads, head_dim)
            v_cache[s, :n] = randn(n, n_kv_heads, head_dim)
        stride = cap * tok

    return HybridBatch(name=name, n_prefill=n_prefill, n_decode=n_decode, n_q_heads=n_q_heads,
                       n_kv_heads=n_kv_heads, head_dim=head_dim, dtype=dtype,
                       softmax_scale=float(softmax_scale), block_size=block_size,
                       max_blocks_per_seq=max_blocks, kv_seq_stride=stride,
                       n_cache_rows=max(n_seqs, 1), n_blocks=n_blocks, max_len=cap, seq_meta=meta,
                       prefill_q=prefill_q, decode_q=decode_q, k_cache=k_cache, v_cache=v_cache,
                       block_table=block_table)


def to_head_major(batch: HybridBatch) -> HybridBatch:
    """The same batch with a head-major cache ([.., Hkv, tokens, d]); values are moved, never changed."""
    if batch.head_major:
        return batch
    return dataclasses.replace(batch, name=batch.name + "/head-major", head_major=True,
                               k_cache=batch.k_cache.transpose(1, 2).contiguous(),
                               v_cache=batch.v_cache.transpose(1, 2).contiguous())


def regroup(batch: HybridBatch, block_size: int, seed: int, poison: Optional[float] = None
            ) -> HybridBatch:
    """The same logical batch with its cache stored in the other layout.

    block_size > 0: paged with that block size and a fresh seeded permutation;
    block_size == 0: contiguous.  Values are moved, never changed.
    """
    tdt = batch.torch_dtype
    dev = batch.k_cache.device
    rng = np.random.Generator(np.random.PCG64(seed))
    n_seqs = batch.n_prefill + batch.n_decode
    tok = batch.n_kv_heads * batch.head_dim
    kv_lens = batch.seq_meta[:, 2].astype(np.int64)
    fill = 0.0 if poison is None else poison

    def logical(cache, s):
        n = int(kv_lens[s])
        row = int(batch.seq_meta[s, 3])
        if batch.block_size > 0:
            t = np.arange(n, dtype=np.int64)
            tbl = batch.block_table.cpu().numpy()
            slots = tbl[row, t // batch.block_size].astype(np.int64) * batch.block_size + t % batch.block_size
            return cache.view(-1, tok)[torch.from_numpy(slots).to(dev)]
        return cache[row, :n].reshape(n, tok)

    kw = {f.name: getattr(batch, f.name) for f in dataclasses.fields(batch)}
    meta = batch.seq_meta.copy()
    meta[:, 3] = np.arange(n_seqs)
    if block_size > 0:
        per = [(int(l) + block_size - 1) // block_size for l in kv_lens]
        n_blocks = int(sum(per)) + 3
        perm = rng.permutation(n_blocks).astype(np.int32)
        max_blocks = max(per)
        table = np.full((n_seqs, max_blocks), -1, dtype=np.int32)
        at = 0
        for s, nb in enumerate(per):
            table[s, :nb] = perm[at:at + nb]
            at += nb
        k_new = torch.full((n_blocks, block_size, batch.n_kv_heads, batch.head_dim), fill, dtype=tdt, device=dev)
        v_new = torch.full_like(k_new, fill)
        for s in range(n_seqs):
            n = int(kv_lens[s])
            t = np.arange(n, dtype=np.int64)
            slots = torch.from_numpy(table[s, t // block_size].astype(np.int64) * block_size + t % block_size).to(dev)
            k_new.view(-1, tok).index_copy_(0, slots, logical(batch.k_cache, s))
            v_new.view(-1, tok).index_copy_(0, slots, logical(batch.v_cache, s))
        kw.update(block_size=block_size, max_blocks_per_seq=max_blocks, kv_seq_stride=0,
                  n_blocks=n_blocks, max_len=max_blocks * block_size,
                  block_table=torch.from_numpy(table).to(dev))
    else:
        cap = int(kv_lens.max())
        k_new = torch.full((n_seqs, cap, batch.n_kv_heads, batch.head_dim), fill, dtype=tdt, device=dev)
        v_new = torch.full_like(k_new, fill)
        for s in range(n_seqs):
            n = int(kv_lens[s])
            k_new[s, :n] = logical(batch.k_cache, s).view(n, batch.n_kv_heads, batch.head_dim)
            v_new[s, :n] = logical(batch.v_cache, s).view(n, batch.n_kv_heads, batch.head_dim)
        kw.update(block_size=0, max_blocks_per_seq=0, kv_seq_stride=cap * tok, n_blocks=0,
                  max_len=cap, block_table=None)
    kw.update(seq_meta=meta, k_cache=k_new, v_cache=v_new, n_cache_rows=n_seqs,
              name=batch.name + ("/paged%d" % block_size if block_size else "/contig"))
    return HybridBatch(**kw)


# --------------------------------------------------------------------------- #
# The benchmark configurations.
# --------------------------------------------------------------------------- #
RATIO_SWEEP: List[Tuple[int, int]] = [(c, nd) for c in (256, 512, 1024, 2048) for nd in (16, 64, 256)]


def config_seed(config: int, batch_index: int = 0) -> int:
    return BASE_SEED + 1000 * config + batch_index


def config_batch(config: int, batch_index: int = 0, device="cpu",
                 poison: Optional[float] = None) -> HybridBatch:
    """Configurations 1-5 (config 5 is a 12-batch prefill/decode ratio sweep).

    1: tiny, fp16, 4 q = 4 kv heads, d 64, contiguous; chunk 128 at 384..511;
       8 decodes with context uniform in [64, 512].
    2: 32 q = 32 kv heads, d 128, fp16, contiguous; chunk 1024 over 3072 cached;
       64 decodes at context 4096.
    3: 32 q / 8 kv, d 128, bf16, paged 16; chunk 512 ending at 8192; 128 decodes
       with context uniform in [2048, 16384].
    4: 32 q / 4 kv, d 128, bf16, paged 16; chunk 2048 ending at 32768; 32 decodes
       at context 32768.
    5: 32 q / 8 kv, d 128, bf16, paged 16; chunk in {256..2048} ending at 4096;
       {16, 64, 256} decodes with context uniform in [4096, 16384].
    6: (an extra, not one of the benchmark configurations) 16 q / 8 kv, d 256, bf16,
       paged 16; chunk 1024 ending at 4096; 64 decodes with context uniform in
       [2048, 8192]: the one shape that exercises 256 channels per head.
    """
    seed = config_seed(config, batch_index)
    rng = np.random.Generator(np.random.PCG64(seed ^ 0x5EED))
    common = dict(seed=seed, device=device, poison=poison)
    if config == 1:
        lens = rng.integers(64, 513, size=8).tolist()
        return make_batch("config1-tiny", prefill=[(128, 512)], decode_kv_lens=lens, n_q_heads=4,
                          n_kv_heads=4, head_dim=64, dtype=F16, softmax_scale=0.125, **common)
    if config == 2:
        return make_batch("config2-llama2-7b-mha", prefill=[(1024, 4096)], decode_kv_lens=[4096] * 64,
                          n_q_heads=32, n_kv_heads=32, head_dim=128, dtype=F16, **common)
    if config == 3:
        lens = rng.integers(2048, 16385, size=128).tolist()
        return make_batch("config3-llama3-8b-gqa", prefill=[(512, 8192)], decode_kv_lens=lens,
                          n_q_heads=32, n_kv_heads=8, head_dim=128, dtype=BF16, block_size=16, **common)
    if config == 4:
        return make_batch("config4-yi-6b-32k", prefill=[(2048, 32768)], decode_kv_lens=[32768] * 32,
                          n_q_heads=32, n_kv_heads=4, head_dim=128, dtype=BF16, block_size=16, **common)
    if config == 5:
        chunk, nd = RATIO_SWEEP[batch_index]
        lens = rng.integers(4096, 16385, size=nd).tolist()
        return make_batch(f"config5-sweep-c{chunk}-d{nd}", prefill=[(chunk, 4096)], decode_kv_lens=lens,
                          n_q_heads=32, n_kv_heads=8, head_dim=128, dtype=BF16, block_size=16, **common)
    if config == 6:
        lens = rng.integers(2048, 8193, size=64).tolist()
        return make_batch("extra-d256-gqa2", prefill=[(1024, 4096)], decode_kv_lens=lens, n_q_heads=16,
                          n_kv_heads=8, head_dim=256, dtype=BF16, block_size=16, **common)
    raise ValueError("config must be 1..6")


# ----------------------------------------------------------------------------------------------
# Chunk series (the shape of the paper's Figure 6 and Table 8): every chunk of one long prompt,
# each co-scheduled with the same set of decode requests.
# ----------------------------------------------------------------------------------------------
SERIES_MODELS = {"yi-6b": (32, 4, 128), "llama-3-8b": (32, 8, 128)}   # q heads, K/V heads, head_dim
SERIES_PROMPT, SERIES_CHUNK, SERIES_DECODE_CTX = 16384, 512, 16384


def series_base(model: str, n_decode: int, device="cpu", poison: Optional[float] = None) -> HybridBatch:
    """One prompt of 16K tokens (its whole K/V in the cache) and ``n_decode`` decodes at 16K context.

    ``series_chunk`` turns it into the batch of one chunk; all chunks share the tensors."""
    hq, hkv, d = SERIES_MODELS[model]
    seed = BASE_SEED + 100000 + 1000 * sorted(SERIES_MODELS).index(model) + n_decode
    return make_batch(f"series-{model}-d{n_decode}", prefill=[(SERIES_CHUNK, SERIES_PROMPT)],
                      decode_kv_lens=[SERIES_DECODE_CTX] * n_decode, n_q_heads=hq, n_kv_heads=hkv,
                      head_dim=d, dtype=BF16, block_size=16, seed=seed, device=device, poison=poison)


def series_chunk(base: HybridBatch, chunk_index: int) -> HybridBatch:
    """The batch of chunk ``chunk_index`` (0-based): 512 new tokens over 512 * chunk_index cached
    ones.  The query values are those of the base batch; only the visible length changes."""
    n_chunks = SERIES_PROMPT // SERIES_CHUNK
    if not 0 <= chunk_index < n_chunks:
        raise ValueError("chunk_index out of range")
    meta = base.seq_meta.copy()
    meta[0, 2] = SERIES_CHUNK * (chunk_index + 1)
    return dataclasses.replace(base, name=f"{base.name}-chunk{chunk_index}", seq_meta=meta)
