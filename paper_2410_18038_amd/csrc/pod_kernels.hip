// gfx950 kernels for hybrid-batch attention: the prefill path (MFMA, LDS-staged K/V tiles,
// online softmax), the decode path (one wavefront per unit, coalesced K/V streaming), the
// split-KV combine, and the fused kernel whose workgroups bind their operation at run time
// from the compute unit they landed on (paper Section 4.1).
//
// Both paths compute S^T = K Q^T rather than S, so that every lane owns one query row:
// the MFMA result then already has the register layout the second product (O^T = V^T P^T)
// wants for its P operand, and the running max and sum of a row are per-lane scalars.
#include <hip/hip_runtime.h>

#include <mutex>
#include <type_traits>

#include "pod_common.h"
#include "pod_launch.h"

namespace pod {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

#define POD_LDS __attribute__((address_space(3)))
#define POD_CONST __attribute__((address_space(4)))

template <int DT> struct Num;
template <> struct Num<0> {   // IEEE binary16
    using v8 = f16x8;
    using v4 = f16x4;
    using elem = _Float16;
    static __device__ __forceinline__ f32x16 mfma32(v8 a, v8 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ f32x4 mfma16(v8 a, v8 b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
    }
    // 16x16x16: `a` arrives as the raw result of an LDS transpose read
    static __device__ __forceinline__ f32x4 mfma16k16(s16x4 a, v4 b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(v4, a), b, c, 0, 0, 0);
    }
    // acc + sum of the eight 16-bit values (one dot-product instruction per pair)
    static __device__ __forceinline__ float add_all(v8 p, float acc) {
        typedef _Float16 v2 __attribute__((ext_vector_type(2)));
        const v2 ones = {(_Float16)1.f, (_Float16)1.f};
#pragma unroll
        for (int i = 0; i < 4; ++i) acc = __builtin_amdgcn_fdot2(v2{p[2 * i], p[2 * i + 1]}, ones, acc, false);
        return acc;
    }
};
template <> struct Num<1> {   // bfloat16
    using v8 = bf16x8;
    using v4 = bf16x4;
    using elem = __bf16;
    static __device__ __forceinline__ f32x16 mfma32(v8 a, v8 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ f32x4 mfma16(v8 a, v8 b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ f32x4 mfma16k16(s16x4 a, v4 b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, __builtin_bit_cast(s16x4, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ float add_all(v8 p, float acc) {
        typedef __bf16 v2 __attribute__((ext_vector_type(2)));
        const v2 ones = {(__bf16)1.f, (__bf16)1.f};
#pragma unroll
        for (int i = 0; i < 4; ++i) acc = __builtin_amdgcn_fdot2_f32_bf16(v2{p[2 * i], p[2 * i + 1]}, ones, acc, false);
        return acc;
    }
};

__device__ __forceinline__ float neg_inf() { return -__builtin_inff(); }
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Cross-lane reductions over the lanes that share a query column, with the gfx950 lane-swap
// instructions (VALU speed, no LDS round trip).  permlane32_swap(x, x) yields {lower half twice,
// upper half twice}; permlane16_swap(x, x) yields {even 16-lane rows twice, odd rows twice}.
__device__ __forceinline__ float max_across_32(float x)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_across_32(float x)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float max_across_16(float x)
{
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_across_16(float x)
{
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// The running maximum is only moved when a new score exceeds it by more than this many powers of
// two; until then weights may reach 2^kMaxSlack, which 16-bit P and fp32 sums hold easily.  The
// accumulators are then rescaled rarely instead of at every step.
constexpr float kMaxSlack = 8.f;

// LDS transpose read: within each group of 16 lanes, lane n receives element n of the four
// 32-byte rows formed by the 8-byte pieces that lanes 4r..4r+3 point at (r = 0..3).
__device__ __forceinline__ s16x4 lds_read_tr(const POD_LDS unsigned char *p)
{
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((POD_LDS s16x4 *)p);
}

// Element offset (head 0, channel 0) of token t of a cache row.  Both cache orders go through the
// same three strides: elements between the tokens of a head, between the heads of a sequence or
// block (added by the callers), and between blocks.
template <bool PAGED>
__device__ __forceinline__ int64_t token_offset(const KernelArgs &a, int cache_row, int t, int token_elems)
{
    if constexpr (PAGED) {
        int bi, off;
        if (a.bs_shift >= 0) { bi = t >> a.bs_shift; off = t & (a.block_size - 1); }
        else { bi = t / a.block_size; off = t - bi * a.block_size; }
        const int blk = a.block_table[(int64_t)cache_row * a.max_blocks_per_seq + bi];
        return (int64_t)blk * a.block_elems + (int64_t)off * token_elems;
    } else {
        return (int64_t)cache_row * a.kv_seq_stride + (int64_t)t * token_elems;
    }
}

// Orders LDS traffic among the lanes of one wavefront.  A wavefront's LDS instructions execute in
// program order, so no hardware wait is needed; this only stops the compiler from moving a
// lane's LDS access across the point where other lanes' data is exchanged.
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ void write_trace(const KernelArgs &a, int slot, int cu, int first_role,
                                            int n_first, int n_second, uint64_t t0, uint64_t t_switch)
{
    TraceRecord r;
    r.cu = cu; r.first_role = first_role; r.n_first = n_first; r.n_second = n_second;
    r.t_begin = t0; r.t_switch = t_switch; r.t_end = wall_clock64(); r.pad = 0;
    a.trace[slot] = r;
}

// Stores the compiler's bookkeeping of outstanding memory operations does not see.  On this
// target loads and stores share one counter; once a store may be outstanding the compiler assumes
// that the counter no longer falls in issue order and makes every later wait for a load a wait
// for everything.  The decode worker keeps a ring of loads in flight while it writes a finished
// unit's results, so it issues those few stores this way.  A wait sized for the loads alone is
// still safe with extra stores in flight: loads complete in order among themselves, so by the
// time all but the newest N operations have completed, the oldest load is among the completed.
// Nothing in these kernels reads the stored data back, and a kernel's end completes its stores.
__device__ __forceinline__ void store16_untracked(void *p, u32x4 v)
{
    asm volatile("global_store_dwordx4 %0, %1, off" ::"v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void store8_untracked(void *p, u32x2 v)
{
    asm volatile("global_store_dwordx2 %0, %1, off" ::"v"(p), "v"(v) : "memory");
}

// Append one record to the event log (one lane calls this).
__device__ __forceinline__ void log_event(const KernelArgs &a, int kind, int item, uint64_t t_begin)
{
    const uint64_t t_end = wall_clock64();
    const uint32_t k = atomicAdd(a.evlog, 1u);
    if (k < a.evlog_cap) {
        EventRecord *r = (EventRecord *)(a.evlog + 4) + k;
        const uint32_t cu = __smid() & (kCuSlots - 1);
        const uint32_t wg = blockIdx.x * kWavesPerWg + (threadIdx.x >> 6);
        store16_untracked(r, u32x4{(uint32_t)kind, (uint32_t)item, cu, wg});
        store16_untracked(&r->t_begin, u32x4{(uint32_t)t_begin, (uint32_t)(t_begin >> 32), (uint32_t)t_end,
                                             (uint32_t)(t_end >> 32)});
    }
}

__device__ __forceinline__ u32x4 load16(const void *p) { return *(const u32x4 *)p; }
// Same, for data that is read once: marked non-temporal so that it does not push reusable
// data (the prefill operation's K/V tiles, shared by the workgroups of a K/V head) out of L2.
__device__ __forceinline__ u32x4 load16_stream(const void *p) { return __builtin_nontemporal_load((const u32x4 *)p); }

// ------------------------------------------------------------------------------------------
// Prefill path (Sections 2.1 and 4.3: the prefill operation as a device function that takes
// its work id as a parameter).  One workgroup = 4 wavefronts x 32 packed query rows.
//
// K/V tiles of 64 keys go from HBM/L2 straight into LDS (16-byte direct-to-LDS loads, no
// register staging), double buffered, one workgroup barrier per tile.  A direct load writes a
// wavefront's 64 chunks to consecutive LDS addresses, so rows cannot be padded; bank conflicts
// are avoided instead by choosing WHICH 16-byte chunk of a row each lane fetches (an XOR
// swizzle applied on the global side and undone by the readers).  The loop is software
// pipelined: while the softmax of tile j runs on the vector ALUs, the matrix unit already
// computes the scores of tile j+1, so K runs one tile ahead of V.
// ------------------------------------------------------------------------------------------
template <int D> struct PrefillLds {
    static constexpr int kRowBytes = D * 2;
    static constexpr int kTileBytes = prefill_kv_tile(D) * kRowBytes;
    static constexpr int kBytes = 4 * kTileBytes;          // K[2] then V[2]
};

// Which chunk position of its LDS row a 16-byte chunk c of row `row` is stored at.
template <int D> __device__ __forceinline__ int k_swizzle(int row, int c)
{
    return D >= 128 ? (c ^ (row & 15)) : (c ^ ((row >> 1) & 7));
}
template <int D> __device__ __forceinline__ int v_swizzle(int row, int c)
{
    return D >= 128 ? (c ^ ((row & 3) << 2)) : (c ^ (((row >> 1) & 1) << 2));
}

// 16 bytes per lane from global memory straight into LDS: lane i of the wavefront lands at
// lds_addr + 16*i.  The global address is sbase + voff (uniform 64-bit base, 32-bit lane offset).
// M0 carries the LDS address.  These kernels use no other instruction that reads M0 (no GDS,
// message, relative-move or interpolation instruction), so it is written without being restored.
__device__ __forceinline__ void dma16(uint32_t lds_addr, uint32_t voff, const void *sbase)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_addr), "v"(voff), "s"(sbase) : "memory", "m0");
}
// Same, for data that is read once (the decode stream): marked non-temporal like load16_stream.
__device__ __forceinline__ void dma16_stream(uint32_t lds_addr, uint32_t voff, const void *sbase)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt"
                 :: "s"(lds_addr), "v"(voff), "s"(sbase) : "memory", "m0");
}
__device__ __forceinline__ void dma16_vaddr(uint32_t lds_addr, const void *vaddr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :: "s"(lds_addr), "v"(vaddr) : "memory", "m0");
}
__device__ __forceinline__ void wait_all_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

template <int DT, int D, int LAYOUT>
__device__ __forceinline__ void prefill_item_run(const KernelArgs &a, const PrefillItem it,
                                                 unsigned char *smem)
{
    using N = Num<DT>;
    using v8 = typename N::v8;
    using L = PrefillLds<D>;
    constexpr int KS = D / 16;                     // 16-channel slices of the QK^T contraction
    constexpr int WPG = D == 256 ? 2 : 1;          // wavefronts per 32-row group: each owns D / WPG output channels
    constexpr int MB = D / 32 / WPG;               // 32-channel blocks of the output owned by this wavefront
    constexpr int CH = D / 8;                      // 16-byte chunks per K/V row
    constexpr int RPW = kWaveSize / CH;            // rows one wavefront loads per pass (2, 4 or 8)
    constexpr int RPP = RPW * kWavesPerWg;         // rows per pass of the workgroup
    constexpr int T = prefill_kv_tile(D);          // keys per staged tile
    constexpr int NTB = T / 32;                    // 32-key blocks per tile
    constexpr int NPASS = T / RPP;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int rg = wave / WPG;                     // row group of this wavefront
    const int cb0 = (wave % WPG) * MB;             // its first 32-channel output block
    const int n32 = lane & 31;                     // query column owned by this lane
    const int h = lane >> 5;                       // which half of the contraction slots
    const int i16 = lane & 15;
    const int b16 = (lane >> 4) & 1;

    const POD_CONST int32_t *meta = (const POD_CONST int32_t *)a.seq_meta + 4 * it.req;
    const int q_start = meta[0], q_len = meta[1], kv_len = meta[2], cache_row = meta[3];
    const int prefix = kv_len - q_len;
    const int group = a.group;
    const int token_elems = a.tok_stride;           // elements between consecutive tokens of a head
    const int rows_total = q_len * group;

    // This lane's query row.
    const int R = it.row0 + rg * 32 + n32;
    const bool row_ok = R < rows_total && (rg * 32 + n32) < it.n_rows;
    const int tok = R / group;
    const int hq = it.kv_head * group + (R - tok * group);
    const int pos = row_ok ? prefix + tok : 0x7fffffff;    // last visible key
    // Causal limits of this wavefront (rows are ordered by token).
    const int w_first = it.row0 + rg * 32;
    const int w_last = min(it.row0 + it.n_rows, it.row0 + rg * 32 + 32) - 1;
    const bool wave_has_rows = w_first < it.row0 + it.n_rows;
    const int wave_minpos = prefix + w_first / group;
    const int wave_maxpos = wave_has_rows ? prefix + w_last / group : -1;

    v8 q[KS];
    {
        const typename N::elem *qp = (const typename N::elem *)a.prefill_q +
            ((int64_t)(q_start + tok) * a.n_q_heads + hq) * D + h * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            u32x4 raw = {0u, 0u, 0u, 0u};
            if (row_ok) raw = load16(qp + ks * 16);
            q[ks] = __builtin_bit_cast(v8, raw);
        }
    }

    // ---- LDS addresses -----------------------------------------------------------------
    // All LDS traffic goes through pointers in the LDS address space: K buffers at 0 and
    // kTileBytes, V buffers at 2 and 3 times kTileBytes.
    POD_LDS unsigned char *const lds = (POD_LDS unsigned char *)smem;
    const uint32_t lds0 = (uint32_t)(uintptr_t)lds;       // LDS byte address of the region
    // readers: byte offsets inside a tile, without the compile-time row blocks.  The swizzles are
    // XORs of the chunk index, so slice ks of K sits at k_rd0 ^ (ks << 5) and block mb of V at
    // v_rd0 ^ (mb << 6): one register each, and one XOR with a constant at the point of use
    // (ten registers fewer than a table of addresses at D = 128, which this loop needs for its
    // LDS reads in flight).
    const uint32_t k_rd0 = (uint32_t)(n32 * L::kRowBytes + k_swizzle<D>(n32, h) * 16);
    uint32_t v_rd0;
    {
        const int row = 4 * h + (i16 >> 2);
        const int c = b16 * 2 + ((i16 & 3) >> 1);
        v_rd0 = (uint32_t)(row * L::kRowBytes + v_swizzle<D>(row, c) * 16 + (i16 & 1) * 8);
    }
    static_assert((D == 256 || D == 128 || D == 64) && KS * 32 <= L::kRowBytes && WPG * MB * 64 <= L::kRowBytes, "swizzle algebra");
    // writers: this lane's LDS chunk in pass p is row p*RPP + wave*RPW + lane/CH, position lane%CH.
    // Lane offsets (bytes) of the source chunk for full tiles.  Contiguous cache: relative to the
    // tile's first row.  Paged cache: relative to the first row of this wavefront's rows in the
    // pass, which lie inside one block.
    const int wr_row = lane / CH, wr_pos = lane % CH;
    const int tok_bytes = token_elems * 2;
    // Up to 128 channels the rows a lane loads in the passes of a tile are a multiple of 16 rows
    // apart, which the swizzles do not see: one offset serves every pass, and the distance between
    // the passes' rows (contiguous cache only) is added to the uniform base of the pass.
    constexpr int NSRC = D <= 128 ? 1 : NPASS;
    static_assert(D > 128 || (RPP % 16 == 0), "row(p) - row(0) must not reach the swizzles");
    uint32_t k_src[NSRC], v_src[NSRC];
#pragma unroll
    for (int p = 0; p < NSRC; ++p) {
        const int row = p * RPP + wave * RPW + wr_row;
        // contiguous: row inside the tile; paged: row inside the wavefront's rows of the pass, plus
        // the wavefront's fixed row inside its block in the 16-key-block case
        const int src_row = LAYOUT == kLayoutContiguous ? row
                            : (LAYOUT == kLayoutPaged16 && D == 128 && a.bs_shift == 4 && a.max_blocks_per_seq >= 4)
                                  ? wave * RPW + wr_row : wr_row;
        k_src[p] = (uint32_t)(src_row * tok_bytes + k_swizzle<D>(row, wr_pos) * 16);
        v_src[p] = (uint32_t)(src_row * tok_bytes + v_swizzle<D>(row, wr_pos) * 16);
    }
    // bytes between the rows of consecutive passes, where the lane offsets above do not hold them
    const int64_t pass_bytes = (NSRC == 1 && LAYOUT == kLayoutContiguous) ? (int64_t)RPP * tok_bytes : 0;

    const typename N::elem *kc = (const typename N::elem *)a.k_cache + it.kv_head * a.head_stride;
    const typename N::elem *vc = (const typename N::elem *)a.v_cache + it.kv_head * a.head_stride;
    const POD_CONST int32_t *table = (const POD_CONST int32_t *)a.block_table +
                                     (int64_t)cache_row * a.max_blocks_per_seq;
    const int n_tiles = (it.kv_end - it.kv_begin + T - 1) / T;

    // Byte offsets (from the start of the cache, K/V head 0) of the rows each pass of this
    // wavefront loads, for a full tile: one uniform 64-bit value per pass.  For the paged layout
    // the block ids come from the block table through scalar loads that are issued one tile
    // earlier than they are needed (TileBlocks), so their latency is never waited for.
    struct TileBases { int64_t b[NPASS]; };
    struct TileBlocks { int32_t id[NPASS]; };
    // With 16-key blocks and head_dim 128 a pass is exactly one block and the four ids of a tile
    // are neighbours in the table: one 16-byte scalar load, and the wavefront's row offset inside
    // its block never changes (it is folded into the lane offsets below).
    typedef int32_t i32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));
    const bool blocks16 = LAYOUT == kLayoutPaged16 && D == 128 && a.bs_shift == 4 && a.max_blocks_per_seq >= 4;
    auto tile_blocks = [&](int jt) {
        TileBlocks tb;
        if constexpr (LAYOUT == kLayoutPaged16) {
            if (D == 128 && blocks16) {
                const int i0 = min((it.kv_begin + jt * T) >> 4, a.max_blocks_per_seq - 4);
                const i32x4_a4 ids = *(const POD_CONST i32x4_a4 *)(table + i0);
#pragma unroll
                for (int p = 0; p < NPASS; ++p) tb.id[p] = ids[p & 3];
            } else {
#pragma unroll
                for (int p = 0; p < NPASS; ++p) {
                    const int t = min(it.kv_begin + jt * T + p * RPP + wave * RPW, it.kv_end - 1);
                    tb.id[p] = table[t >> a.bs_shift];
                }
            }
        } else {
#pragma unroll
            for (int p = 0; p < NPASS; ++p) tb.id[p] = 0;
        }
        return tb;
    };
    auto tile_bases = [&](int jt, const TileBlocks &blk) {
        TileBases tb;
        const int j0 = it.kv_begin + jt * T;
        if constexpr (LAYOUT == kLayoutContiguous) {
            const int64_t off = ((int64_t)cache_row * a.kv_seq_stride + (int64_t)j0 * token_elems) * 2;
#pragma unroll
            for (int p = 0; p < NPASS; ++p) tb.b[p] = off + p * pass_bytes;
        } else if constexpr (LAYOUT == kLayoutPaged16) {
            // the block size is a power of two in this layout; bytes per token need not be (the
            // K/V head count of a model or of its tensor-parallel shard can be 5, 6, 10, 40 ...)
            const uint32_t block_bytes = (uint32_t)a.block_elems * 2u;
#pragma unroll
            for (int p = 0; p < NPASS; ++p) {
                const uint32_t t = (uint32_t)(j0 + p * RPP + wave * RPW);
                const uint64_t block_off = (uint64_t)(uint32_t)blk.id[p] * block_bytes;
                const uint64_t row_off = (uint64_t)((t & (uint32_t)(a.block_size - 1)) * (uint32_t)tok_bytes);
                tb.b[p] = (int64_t)(blocks16 ? block_off : block_off + row_off);
            }
        } else {
#pragma unroll
            for (int p = 0; p < NPASS; ++p) tb.b[p] = 0;
        }
        return tb;
    };
    // Fast path for a full tile of the contiguous layout and of paged layouts with power-of-two blocks.
    auto issue_fast = [&](const TileBases &tb, int buf, bool is_k) {
        const char *src = is_k ? (const char *)kc : (const char *)vc;
#pragma unroll
        for (int p = 0; p < NPASS; ++p) {
            const uint32_t dst = lds0 + (uint32_t)((is_k ? buf : 2 + buf) * L::kTileBytes +
                                                  (p * kWgThreads + wave * kWaveSize) * 16);
            dma16(dst, is_k ? k_src[NSRC == 1 ? 0 : p] : v_src[NSRC == 1 ? 0 : p], src + tb.b[p]);
        }
    };
    auto tile_is_fast = [&](int jt) {
        return LAYOUT != kLayoutPagedAny && it.kv_end - (it.kv_begin + jt * T) >= T;
    };

    // General path: any layout, and the last tile of an item when it is not full.  Rows past the
    // item's last key re-read its last row: finite data, masked out of the softmax by index.
    auto issue_tile = [&](int jt, int buf, bool want_k, bool want_v) {
        const int j0 = it.kv_begin + jt * T;
        const int last_row = it.kv_end - 1 - j0;                // >= 0
#pragma unroll
        for (int p = 0; p < NPASS; ++p) {
            const int row_base = p * RPP + wave * RPW;           // uniform
            const int base_eff = min(row_base, last_row & ~(RPW - 1));
            const uint32_t dst_k = lds0 + (uint32_t)(buf * L::kTileBytes + (p * kWgThreads + wave * kWaveSize) * 16);
            const uint32_t dst_v = dst_k + 2 * L::kTileBytes;
            if constexpr (LAYOUT == kLayoutPagedAny) {
                const int row = min(row_base + wr_row, last_row);
                const int64_t off = token_offset<true>(a, cache_row, j0 + row, token_elems);
                const int lrow = row_base + wr_row;              // swizzle follows the LDS row
                if (want_k) dma16_vaddr(dst_k, kc + off + k_swizzle<D>(lrow, wr_pos) * 8);
                if (want_v) dma16_vaddr(dst_v, vc + off + v_swizzle<D>(lrow, wr_pos) * 8);
            } else {
                const int t = j0 + base_eff;
                int64_t base;
                if constexpr (LAYOUT == kLayoutContiguous) {
                    base = (int64_t)cache_row * a.kv_seq_stride + (int64_t)t * token_elems;
                } else {
                    const int blk = table[t >> a.bs_shift];
                    base = (int64_t)blk * a.block_elems + (int64_t)(t & (a.block_size - 1)) * token_elems;
                }
                const int lrow = row_base + wr_row;
                const int rl = min(lrow, last_row) - base_eff;
                const uint32_t ko = (uint32_t)(rl * token_elems + k_swizzle<D>(lrow, wr_pos) * 8) * 2u;
                const uint32_t vo = (uint32_t)(rl * token_elems + v_swizzle<D>(lrow, wr_pos) * 8) * 2u;
                if (want_k) dma16(dst_k, ko, kc + base);
                if (want_v) dma16(dst_v, vo, vc + base);
            }
        }
    };

    f32x16 o[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[mb][r] = 0.f;
    float m_run = neg_inf(), l_run = 0.f;
    const float c = a.scale_log2;

    // S^T = K Q^T for one tile: rows = keys, columns = this wavefront's query rows.
    // Register r of block tb holds key j0 + tb*32 + 8*(r/4) + 4*h + r%4.
    auto scores = [&](int kbuf, f32x16 (&s)[NTB]) {
        const POD_LDS unsigned char *kb = lds + kbuf * L::kTileBytes;
        uint32_t k_base = k_rd0;
        asm("" : "+v"(k_base));                   // opaque copy: the XORs below stay inside the loop
        // Operation i = (key block i / KS, slice i % KS).  The LDS reads are written, and pinned,
        // three operations ahead of the matrix instructions that use them: inlined into the fused
        // kernel this block is otherwise emitted read-wait-multiply, sixteen times, and every
        // matrix instruction waits a full LDS latency.  0x100 = LDS read, 0x008 = matrix op.
        constexpr int kAhead = 3, kOps = NTB * KS;
        auto k_frag = [&](int i) __attribute__((always_inline)) {
            return *(const POD_LDS v8 *)(kb + (i / KS) * 32 * L::kRowBytes + (k_base ^ (uint32_t)((i % KS) << 5)));
        };
        v8 kk[kOps];
#pragma unroll
        for (int i = 0; i < kAhead; ++i) kk[i] = k_frag(i);
#pragma unroll
        for (int tb = 0; tb < NTB; ++tb)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[tb][r] = 0.f;
#pragma unroll
        for (int i = 0; i < kOps; ++i) {
            if (i + kAhead < kOps) kk[i + kAhead] = k_frag(i + kAhead);
            s[i / KS] = N::mfma32(kk[i], q[i % KS], s[i / KS]);
        }
        __builtin_amdgcn_sched_group_barrier(0x100, kAhead, 0);
#pragma unroll
        for (int i = 0; i < kOps - kAhead; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, kAhead, 0);
    };

    if (n_tiles <= 0) return;                                // never planned; keeps the loop simple
    __syncthreads();                                         // previous use of this LDS is over
    TileBases carry = {};                                     // bases of tile jt+1 inside the loop
    if (tile_is_fast(0)) {
        const TileBases t0 = tile_bases(0, tile_blocks(0));
        issue_fast(t0, 0, true);
        issue_fast(t0, 0, false);
    } else {
        issue_tile(0, 0, true, true);
    }
    if (n_tiles > 1) {
        if (tile_is_fast(1)) {
            carry = tile_bases(1, tile_blocks(1));
            issue_fast(carry, 1, true);
        } else {
            issue_tile(1, 1, true, false);
        }
    }
    TileBlocks blocks_ahead = tile_blocks(2);                // for the K loads of the first iteration
    wait_all_loads();
    __syncthreads();
    // Two score buffers swap roles from one tile to the next; the loop body exists twice (even
    // and odd tiles) so that the swap is a matter of names, not of 32 register moves per tile, and
    // the LDS buffer of a tile is known at compile time.
    f32x16 s_even[NTB], s_odd[NTB];
    if (it.kv_begin <= wave_maxpos) scores(0, s_even);
    __syncthreads();                                         // K tile 0 is free to be overwritten

    auto tile_step = [&](const int jt, auto parity, f32x16 (&s_cur)[NTB], f32x16 (&s_next)[NTB])
                         __attribute__((always_inline)) {
        const int j0 = it.kv_begin + jt * T;
        constexpr int cur = decltype(parity)::value;
        // K tile jt was consumed in the previous iteration and V tile jt-1 as well (barrier below).
        TileBases fresh = carry;
        if (jt + 2 < n_tiles) {
            if (tile_is_fast(jt + 2)) {
                fresh = tile_bases(jt + 2, blocks_ahead);
                issue_fast(fresh, cur, true);
            } else {
                issue_tile(jt + 2, cur, true, false);
            }
        }
        if (jt + 1 < n_tiles) {
            if (tile_is_fast(jt + 1)) issue_fast(carry, cur ^ 1, false);
            else issue_tile(jt + 1, cur ^ 1, false, true);
        }
        carry = fresh;
        blocks_ahead = tile_blocks(jt + 3);                  // used by the next iteration

        const bool live = j0 <= wave_maxpos;                 // something visible to this wavefront
        const bool next_live = (jt + 1 < n_tiles) && (j0 + T <= wave_maxpos);
        if (next_live) scores(cur ^ 1, s_next);              // matrix unit: scores of the next tile
        if (live) {
            // vector ALUs: softmax of the current tile
            const bool need_mask = (j0 + T - 1 > wave_minpos) || (j0 + T > it.kv_end);
            if (__builtin_expect(need_mask, 0)) {
                const int lim = min(pos, it.kv_end - 1);
#pragma unroll
                for (int tb = 0; tb < NTB; ++tb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int key = j0 + tb * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                        if (key > lim) s_cur[tb][r] = neg_inf();
                    }
            }
            float mx = neg_inf();
#pragma unroll
            for (int tb = 0; tb < NTB; ++tb)
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s_cur[tb][r]);
            mx = max_across_32(mx) * c;
            const bool grow = mx > m_run + kMaxSlack;        // also true for the first visible key
            if (__builtin_amdgcn_ballot_w64(grow) != 0) {
                const float alpha = grow ? fast_exp2(m_run - mx) : 1.f;   // mx is finite where grow holds
                m_run = grow ? mx : m_run;
                l_run *= alpha;
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o[mb][r] *= alpha;
            }
            const float m_use = (m_run == neg_inf()) ? 0.f : m_run;
            v8 pk[NTB][2];
#pragma unroll
            for (int tb = 0; tb < NTB; ++tb)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    pk[tb][r >> 3][r & 7] = (typename N::elem)fast_exp2(__builtin_fmaf(s_cur[tb][r], c, -m_use));
            // the weight sum is taken over the rounded weights, the ones the PV product uses
#pragma unroll
            for (int tb = 0; tb < NTB; ++tb)
#pragma unroll
                for (int u = 0; u < 2; ++u) l_run = N::add_all(pk[tb][u], l_run);
            // O^T += V^T P^T : rows = channels, contraction over the keys in S's own register order.
            const POD_LDS unsigned char *vb = lds + (2 + cur) * L::kTileBytes;
            uint32_t v_base = v_rd0;
            asm("" : "+v"(v_base));               // as for K above
            // Operation j = (channel block j / (2 NTB), key block (j / 2) % NTB, half j % 2); its V
            // fragment is two transposing reads.  As for K, the reads are written and pinned two
            // operations ahead of the matrix instruction that uses them.
            constexpr int kAheadV = 2, kOpsV = 2 * NTB * MB;
            auto v_frag = [&](int j) __attribute__((always_inline)) {
                const POD_LDS unsigned char *vp = vb + (((j >> 1) % NTB) * 32 + 16 * (j & 1)) * L::kRowBytes +
                                                  (v_base ^ (uint32_t)((cb0 + j / (2 * NTB)) << 6));
                const s16x4 lo = lds_read_tr(vp);
                const s16x4 hi = lds_read_tr(vp + 8 * L::kRowBytes);
                return __builtin_bit_cast(v8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
            };
            v8 vv[kOpsV];
#pragma unroll
            for (int j = 0; j < kAheadV; ++j) vv[j] = v_frag(j);
#pragma unroll
            for (int j = 0; j < kOpsV; ++j) {
                if (j + kAheadV < kOpsV) vv[j + kAheadV] = v_frag(j + kAheadV);
                o[j / (2 * NTB)] = N::mfma32(vv[j], pk[(j >> 1) % NTB][j & 1], o[j / (2 * NTB)]);
            }
            __builtin_amdgcn_sched_group_barrier(0x100, 2 * kAheadV, 0);
#pragma unroll
            for (int j = 0; j < kOpsV - kAheadV; ++j) {
                __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, kAheadV, 0);
        }
        wait_all_loads();                                    // K tile jt+2 and V tile jt+1 have landed
        __syncthreads();                                     // ... for every wavefront; tile jt is done
    };
    for (int jt = 0; jt < n_tiles; jt += 2) {
        tile_step(jt, std::integral_constant<int, 0>{}, s_even, s_odd);
        if (jt + 1 >= n_tiles) break;
        tile_step(jt + 1, std::integral_constant<int, 1>{}, s_odd, s_even);
    }

    // Epilogue.  o[mb][r] is channel (cb0 + mb)*32 + 8*(r/4) + 4*h + r%4 of this lane's query row.
    const float l_tot = sum_across_32(l_run);
    if (it.prow0 < 0) {
        if (row_ok) {
            const float inv = 1.f / l_tot;
            typename N::elem *op = (typename N::elem *)a.out +
                ((int64_t)(q_start + tok) * a.n_q_heads + hq) * D;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int rq = 0; rq < 4; ++rq) {
                    typename N::v4 w;
#pragma unroll
                    for (int e = 0; e < 4; ++e) w[e] = (typename N::elem)(o[mb][rq * 4 + e] * inv);
                    *(typename N::v4 *)(op + (cb0 + mb) * 32 + 8 * rq + 4 * h) = w;
                }
        }
    } else {
        const int64_t prow = (int64_t)it.prow0 + rg * 32 + n32;
        float *po = a.part_o + prow * D;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                f32x4 w = {o[mb][rq * 4 + 0], o[mb][rq * 4 + 1], o[mb][rq * 4 + 2], o[mb][rq * 4 + 3]};
                *(f32x4 *)(po + (cb0 + mb) * 32 + 8 * rq + 4 * h) = w;
            }
        if (h == 0 && cb0 == 0) {
            a.part_ml[prow * 2 + 0] = m_run;
            a.part_ml[prow * 2 + 1] = l_tot;
        }
    }
}

// ------------------------------------------------------------------------------------------
// Decode path (Section 4.2.3: a decode workgroup is cut into one-wavefront virtual units, so
// no workgroup barrier is used here).  A wavefront is a persistent worker over a stream of decode
// units.  It reads K and V rows once from HBM with fully coalesced 16-byte loads, in steps of 16
// keys; while one step is computed the next ones are in flight in a short ring of registers.
// The ring runs on across unit boundaries: the "head" (the step being requested from memory)
// moves into the next unit while the "tail" (the step being computed) finishes the current one,
// so a boundary costs no drained pipeline.  For that the next unit is claimed, its descriptor
// read and its query heads copied to LDS a few steps before the head needs them.  A small
// wavefront-private LDS region turns 16 rows at a time into MFMA operands.  The query heads of
// the group are the (zero padded) 16 columns of the products, so the matrix unit is busy for a
// few percent of the time only (Section 4.2.1).
// ------------------------------------------------------------------------------------------
template <int D> struct DecodeLds {
    static constexpr int kStep = decode_step_keys(D);          // keys per step
    static constexpr int kKStride = D * 2 + 16;
    static constexpr int kVStride = D * 2 + 32;
    static constexpr int kKBytes = kStep * kKStride;
    static constexpr int kVBytes = kStep * kVStride;
    // Query heads of a unit as MFMA operands: per 32-channel slice one 16-byte piece for each of 4
    // channel groups x kQCols columns (heads of the group).  Up to 128 channels every lane of the
    // wavefront has a piece (16 columns, zero padded); at 256 channels the group is at most 8 heads
    // and only those 8 columns are stored, which halves the buffers.
    static constexpr int kQCols = D == 256 ? kMaxGroup256 : 16;
    static constexpr int kQSlice = 4 * kQCols * 16;
    static constexpr int kQBuf = (D / 32) * kQSlice;           // one unit's query heads as MFMA operands
    static constexpr int kQBytes = 2 * kQBuf;                  // the tail's unit and the unit fetched ahead
    static constexpr int kBytesPerWave = kKBytes + kVBytes + kQBytes;
    static constexpr int kBytes = kBytesPerWave * kWavesPerWg;
};

template <int D, int LAYOUT> struct DecodeRing {
    // A slot holds the K and V rows of 16 keys: D / 4 registers, 8 KB at D = 128.  One slot in
    // flight per streaming wavefront while the other is computed keeps HBM busy; deeper rings only
    // lengthen the queues in the memory system, which measured slower for the decode role itself
    // (6.1 -> 6.3 TB/s going from 5 slots to 2 on 64 requests x 32 heads x 4096 keys with eight
    // streaming wavefronts per unit; with the four there are now, 2, 3 and 4 slots measure the
    // same) and for the prefill role running beside it (its tile loads wait in the same queues).
    // The price: a wavefront alone on the chip streams 10.7 instead of 12.8 GB/s.  The any-block-size layout looks up block ids with vector loads before each
    // step and gets one more slot to cover them; D = 64 slots are half the size.
    static constexpr int kDepth = D >= 128 ? (LAYOUT == kLayoutPagedAny ? 3 : 2) : 4;
};

// Placed right after a branch on a per-lane condition inside code that keeps wavefront-uniform
// state: the join of that branch stays a block of its own, so the compiler does not merge it
// with joins of uniform branches (which would make it treat the uniform state as per-lane and
// move it to vector registers).  Emits no instruction.
__device__ __forceinline__ void lane_test_done() { __builtin_amdgcn_wave_barrier(); }

template <int N_OPS> __device__ __forceinline__ void wait_loads_but()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N_OPS) : "memory");
}

// A decode worker.  Worker number `seat` (seats are handed out once per workgroup) starts with the
// fixed units 4*seat .. 4*seat+3, one per wavefront, when seat < n_static_seats: a chip-wide
// burst of claims at the start of a launch would be served one at a time by the memory system.
// After that a wavefront claims units from the queue of its XCD, then from the other queues.
// Returns the number of units the wavefront ran.
template <int DT, int D, int LAYOUT>
__device__ __forceinline__ int decode_worker_run(const KernelArgs &a, unsigned char *smem, const int seat,
                                                 const int xcd)
{
    using N = Num<DT>;
    using v8 = typename N::v8;
    using elem = typename N::elem;
    using L = DecodeLds<D>;
    constexpr int KS = D / 32;                     // 32-channel slices of the QK^T contraction
    constexpr int MB = D / 16;                     // 16-channel blocks of the output
    constexpr int CH = D / 8;                      // 16-byte chunks per row
    constexpr int RPI = kWaveSize / CH;            // rows per load instruction
    constexpr int STEP = L::kStep;                 // keys per step (16; 8 at 256 channels)
    constexpr int NLD = STEP / RPI;                // load instructions per step, for K and for V
    constexpr int QC = L::kQCols;                  // query columns held in LDS
    constexpr int R = DecodeRing<D, LAYOUT>::kDepth;
    constexpr int kDummy = 0x3fffffff;             // slot holds no step (all its keys are masked)
    constexpr int kClaimAhead = 2 * R;             // the head claims its next unit this many steps before it runs out

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int n16 = lane & 15;                     // query column (head within the group)
    const int b4 = lane >> 4;
    const int group = a.group;
    const int token_elems = a.tok_stride;           // elements between consecutive tokens of a head
    const bool col_ok = n16 < group;
    const float c = a.scale_log2;
    const int ld_row = lane / CH, ld_chunk = lane % CH;
    POD_LDS unsigned char *const lds_k = (POD_LDS unsigned char *)(smem + wave * L::kBytesPerWave);
    POD_LDS unsigned char *const lds_v = lds_k + L::kKBytes;
    POD_LDS unsigned char *const lds_q = lds_v + L::kVBytes;
    const POD_CONST int32_t *const dq = (const POD_CONST int32_t *)a.dq_begin;

    // Unit descriptors and everything derived from them are wavefront-uniform: they are read
    // through the constant address space so that they live in scalar registers.
    struct Desc { int id, kv_head, t0, t1, prow0, q_start, cache_row; };
    auto load_desc = [&](int idx) __attribute__((always_inline)) -> Desc {
        idx = __builtin_amdgcn_readfirstlane(idx);
        const POD_CONST int32_t *w = (const POD_CONST int32_t *)a.dunits + 8 * (int64_t)idx;
        Desc d;
        d.id = idx;
        d.kv_head = w[1]; d.t0 = w[2]; d.t1 = w[3]; d.prow0 = w[4]; d.q_start = w[6]; d.cache_row = w[7];
        return d;
    };

    // ---- claims ------------------------------------------------------------------------
    // The compiler keeps exact counts of the loads in flight only as long as every path through
    // the ring's loop issues the same memory operations.  So a claim that must be waited for on
    // the spot is one opaque instruction pair (the atomic and its wait), and the claim issued
    // ahead of its use is part of every turn of the ring: a turn that wants no unit adds zero to
    // a word of its own workgroup instead.
    int cq = __builtin_amdgcn_readfirstlane(xcd) & (kXcdQueues - 1), tried = 0;
    auto claim_now = [&]() __attribute__((always_inline)) -> int {
        uint32_t v = 0;
        if (lane == 0) {
            uint32_t *ctr = &a.hdr->next_dunit_xcd[cq][0];
            asm volatile("global_atomic_add %0, %1, %2, off sc0\n\ts_waitcnt vmcnt(0)"
                         : "=&v"(v) : "v"(ctr), "v"(1u) : "memory");
        }
        lane_test_done();
        return (int)__builtin_amdgcn_readfirstlane(v);
    };
    // Turns a claimed counter value into a unit index.  When the queue is used up it claims from
    // the next queues (and waits for those claims); -1 when no unit is left anywhere.
    auto claim_resolve = [&](int k) __attribute__((always_inline)) -> int {
        for (;;) {
            const int q0 = dq[cq], q1 = dq[cq + 1];
            if (k < q1 - q0) return q0 + k;
            do {
                cq = (cq + 1) & (kXcdQueues - 1);
                ++tried;
            } while (tried < kXcdQueues && dq[cq + 1] == dq[cq]);
            if (tried >= kXcdQueues) return -1;
            k = claim_now();
        }
    };

    // ---- the next unit's query heads: global memory -> LDS, asynchronously ----------------
    // The query heads of the next unit are copied to LDS ahead of time (two buffers, used in
    // turn) and moved to registers when the tail enters the unit.  Lanes of columns beyond the
    // group read zeros written once.
    int q_cur = 0;                                 // buffer of the tail's unit
    // A direct-to-LDS load puts lane i's piece at position i of the slice, so the lane that copies
    // piece (column, channel group) is the lane whose number is that piece's position: every lane
    // with 16 columns (position = channel group * 16 + column), lanes 0..31 with 8 columns
    // (position = channel group * 8 + column).
    const int cp_col = QC == 16 ? n16 : (lane & 7), cp_b4 = QC == 16 ? b4 : (lane >> 3);
    const bool cp_slot = QC == 16 || lane < 4 * QC;           // this lane has a position in a slice
    const bool cp_ok = cp_slot && cp_col < group;             // ... and a query head to copy there
    if (cp_slot && !cp_ok) {
#pragma unroll
        for (int i = 0; i < 2 * KS; ++i) *(POD_LDS u32x4 *)(lds_q + i * L::kQSlice + lane * 16) = u32x4{0u, 0u, 0u, 0u};
    }
    lane_test_done();
    auto q_dma = [&](const Desc &d, int buf) __attribute__((always_inline)) {
        const char *qb = (const char *)((const elem *)a.decode_q +
                                        ((int64_t)d.q_start * a.n_q_heads + d.kv_head * group) * D);
        const uint32_t vo = (uint32_t)(cp_col * D + cp_b4 * 8) * 2u;
        const uint32_t dst = (uint32_t)(uintptr_t)lds_q + (uint32_t)(buf * L::kQBuf);
        if (cp_ok) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) dma16_vaddr(dst + ks * L::kQSlice, qb + vo + ks * 64);
        }
        lane_test_done();
    };
    v8 q[KS];
    const int q_piece = QC == 16 ? lane : b4 * QC + (n16 & (QC - 1));   // this lane's piece of a slice as an MFMA operand
    auto q_from_lds = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            q[ks] = *(const POD_LDS v8 *)(lds_q + q_cur * L::kQBuf + ks * L::kQSlice + q_piece * 16);
            if constexpr (QC < 16) {
                // columns beyond the stored ones are zero
                const u32x4 raw = __builtin_bit_cast(u32x4, q[ks]);
                const u32x4 zero = {0u, 0u, 0u, 0u};
                q[ks] = __builtin_bit_cast(v8, n16 < QC ? raw : zero);
            }
        }
    };

    // ---- head: the step whose rows are requested next ----------------------------------------
    Desc hu, cu, nx;                               // units of the head, of the tail, and the one fetched ahead
    int h_t = 0;                                   // first key of the head's next step; >= hu.t1: the head has run out
    int h_addr_t = 0;                              // first key of the step the addresses below point at
    int64_t h_base = 0;                            // element offset (head 0, channel 0) of that step
    uint32_t voff[NLD];                            // per-lane byte offsets inside that step
    const elem *kc = nullptr, *vc = nullptr;
    const POD_CONST int32_t *table = nullptr;
    // State bits (one word: separate flags end up addressed through a common pointer and then
    // live in scratch memory).
    constexpr uint32_t kHeadInTail = 1u;           // head and tail are in the same unit
    constexpr uint32_t kNextValid = 2u;            // `nx` holds a fetched unit, its query heads are in (or on their way to) LDS
    constexpr uint32_t kClaimPending = 4u;         // a claim has been issued and not looked at yet
    constexpr uint32_t kExhausted = 8u;            // every queue has been found empty
    constexpr uint32_t kDone = 16u;                // the tail has finished the last unit
    // In the CTA-parallel launch a wavefront runs the one unit it was given: the queues count as
    // used up from the start, so no claim is ever issued and the worker ends with its unit.
    uint32_t st = kHeadInTail | (a.single_unit ? kExhausted : 0u);
    uint32_t claim_v = 0;                          // lane 0: counter value returned by the claim of the current turn
    int n_iss = 0, q_mark = 0;                     // steps issued so far; their count when the last Q copy was issued

    // Rows past the end of a unit's last step re-read its last row (the keys are masked out of the
    // softmax by index), so every load is in bounds and none sits behind a branch.
    auto set_voff = [&](int t_first, int t1) __attribute__((always_inline)) {
        const int last_row = min(t1 - 1 - t_first, STEP - 1);
#pragma unroll
        for (int p = 0; p < NLD; ++p) {
            const int row = min(p * RPI + ld_row, last_row);
            voff[p] = (uint32_t)(row * token_elems + ld_chunk * 8) * 2u;
        }
    };
    auto base_of = [&](int cache_row, int t) __attribute__((always_inline)) -> int64_t {
        if constexpr (LAYOUT == kLayoutContiguous) {
            return (int64_t)cache_row * a.kv_seq_stride + (int64_t)t * token_elems;
        } else if constexpr (LAYOUT == kLayoutPaged16) {
            // block_size is a power of two >= 16 and t a multiple of 16: a step never straddles blocks
            const int bi = t >> a.bs_shift, off = t & (a.block_size - 1);
            const int blk = table[bi];
            return (int64_t)blk * a.block_elems + (int64_t)off * token_elems;
        } else {
            return 0;
        }
    };
    auto set_head = [&](const Desc &d) __attribute__((always_inline)) {
        hu = d;
        h_t = d.t0;
        h_addr_t = d.t0;
        kc = (const elem *)a.k_cache + d.kv_head * a.head_stride;
        vc = (const elem *)a.v_cache + d.kv_head * a.head_stride;
        table = (const POD_CONST int32_t *)a.block_table + (int64_t)d.cache_row * a.max_blocks_per_seq;
        h_base = base_of(d.cache_row, d.t0);
        set_voff(d.t0, d.t1);
    };

    struct Slot { u32x4 k[NLD], v[NLD]; };
    // Request the head's step into a slot.  When the head has run out, the last step is read again
    // and the slot is marked as holding nothing.
    auto issue_step = [&](Slot &sl, int &slot_t) __attribute__((always_inline)) {
        slot_t = h_t < hu.t1 ? h_t : kDummy;
        if constexpr (LAYOUT == kLayoutPagedAny) {
            const int last_row = hu.t1 - 1 - h_addr_t;       // >= 0
#pragma unroll
            for (int p = 0; p < NLD; ++p) {
                const int row = min(p * RPI + ld_row, last_row);
                const int64_t off = token_offset<true>(a, hu.cache_row, h_addr_t + row, token_elems) + ld_chunk * 8;
                sl.k[p] = load16_stream(kc + off);
                sl.v[p] = load16_stream(vc + off);
            }
        } else {
            const char *kb = (const char *)(kc + h_base);
            const char *vb = (const char *)(vc + h_base);
#pragma unroll
            for (int p = 0; p < NLD; ++p) {
                sl.k[p] = load16_stream(kb + voff[p]);
                sl.v[p] = load16_stream(vb + voff[p]);
            }
        }
        ++n_iss;
    };
    auto advance_head = [&]() __attribute__((always_inline)) {
        if (h_t < hu.t1) {
            h_t += STEP;
            if (h_t < hu.t1) {
                h_addr_t = h_t;
                if constexpr (LAYOUT == kLayoutContiguous) h_base += (int64_t)STEP * token_elems;
                else h_base = base_of(hu.cache_row, h_t);
                if (h_t + STEP > hu.t1) set_voff(h_t, hu.t1);     // ragged last step
            }
        }
    };
    // Claim result -> descriptor -> query copy.  Waits for the claim and for the descriptor.
    auto fetch_next = [&]() __attribute__((always_inline)) {
        int idx = -1;
        if (st & kClaimPending) idx = claim_resolve((int)__builtin_amdgcn_readfirstlane(claim_v));
        else if (!(st & kExhausted)) idx = claim_resolve(claim_now());
        st &= ~kClaimPending;
        nx = load_desc(max(idx, 0));
        q_mark = idx >= 0 ? n_iss : q_mark;
        st |= idx >= 0 ? kNextValid : kExhausted;
        if (idx >= 0) q_dma(nx, q_cur ^ 1);
    };

    // ---- tail: the step being computed ------------------------------------------------------------
    f32x4 o[MB];
    float m_run, l_run;
    auto reset_acc = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) o[mb] = f32x4{0.f, 0.f, 0.f, 0.f};
        m_run = neg_inf();
        l_run = 0.f;
    };
    auto consume = [&](const Slot &sl, const int t_first) __attribute__((always_inline)) {
#pragma unroll
        for (int p = 0; p < NLD; ++p) {
            const int row = p * RPI + ld_row;
            *(POD_LDS u32x4 *)(lds_k + row * L::kKStride + ld_chunk * 16) = sl.k[p];
            *(POD_LDS u32x4 *)(lds_v + row * L::kVStride + ld_chunk * 16) = sl.v[p];
        }
        wave_lds_sync();                           // rows written by some lanes are read by others
        // S^T tile: register r holds key t_first + 4*b4 + r of query column n16.  (With 8-key steps
        // the matrix rows 8..15 repeat rows 0..7 and are masked like keys past the unit's end.)
        f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const v8 kk = *(const POD_LDS v8 *)(lds_k + (n16 & (STEP - 1)) * L::kKStride + (ks * 32 + b4 * 8) * 2);
            s = N::mfma16(kk, q[ks], s);
        }
        const int n_valid = min(cu.t1 - t_first, STEP) - 4 * b4;         // keys of this lane that exist
#pragma unroll
        for (int r = 0; r < 4; ++r) s[r] = (r < n_valid) ? s[r] : neg_inf();
        float mx = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
        mx = max_across_32(max_across_16(mx)) * c;
        const bool grow = mx > m_run + kMaxSlack;          // also true for the first key
        if (__builtin_amdgcn_ballot_w64(grow) != 0) {
            const float alpha = grow ? fast_exp2(m_run - mx) : 1.f;
            m_run = grow ? mx : m_run;
            l_run *= alpha;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) o[mb] = o[mb] * alpha;
        }
        const float m_use = (m_run == neg_inf()) ? 0.f : m_run;
        typename N::v4 pk;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float p = fast_exp2(__builtin_fmaf(s[r], c, -m_use));
            l_run += p;
            pk[r] = (elem)p;
        }
        // O^T += V^T P^T over these 16 keys: lane's contraction slots 4*b4 + r are keys 4*b4 + r.
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const POD_LDS unsigned char *vp = lds_v + ((4 * b4 + (n16 >> 2)) & (STEP - 1)) * L::kVStride +
                                      (mb * 16 + (n16 & 3) * 4) * 2;
            o[mb] = N::mfma16k16(lds_read_tr(vp), pk, o[mb]);
        }
        wave_lds_sync();                           // all reads issued before the next step overwrites
    };
    // o[mb][r] is channel mb*16 + 4*b4 + r of query column n16.
    auto finish_unit = [&](const Desc &d) __attribute__((always_inline)) {
        const float l_tot = sum_across_32(sum_across_16(l_run));
        if (col_ok) {
        if (d.prow0 < 0) {
            const float inv = 1.f / l_tot;
            elem *op = (elem *)a.out +
                ((int64_t)(a.n_prefill_rows + d.q_start) * a.n_q_heads + d.kv_head * group + n16) * D;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                typename N::v4 w;
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = (elem)(o[mb][e] * inv);
                store8_untracked(op + mb * 16 + 4 * b4, __builtin_bit_cast(u32x2, w));
            }
        } else {
            const int64_t prow = (int64_t)d.prow0 + n16;
            float *po = a.part_o + prow * D;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) store16_untracked(po + mb * 16 + 4 * b4, __builtin_bit_cast(u32x4, o[mb]));
            if (b4 == 0)
                store8_untracked(a.part_ml + prow * 2, u32x2{__float_as_uint(m_run), __float_as_uint(l_tot)});
        }
        }
        lane_test_done();
    };

    // ---- first unit -------------------------------------------------------------------------------
    int n_done = 0;
    {
        int idx0;
        if (seat < a.n_static_seats) idx0 = __builtin_amdgcn_readfirstlane(seat) * kWavesPerWg + wave;
        else idx0 = claim_resolve(claim_now());
        if (idx0 < 0 || idx0 >= a.n_dunits) return 0;
        set_head(load_desc(idx0));
        cu = hu;
        q_dma(cu, 0);
    }
    uint64_t tb = a.evlog ? wall_clock64() : 0;
    reset_acc();

    Slot ring[R];
    int slot_t[R];
    uint32_t *const null_ctr = &a.hdr->null_claim[blockIdx.x & (kNullClaimLines - 1)][wave];
#pragma unroll
    for (int r = 0; r < R - 1; ++r) {
        issue_step(ring[r], slot_t[r]);
        __builtin_amdgcn_sched_barrier(0);         // loads return in issue order: keep oldest first
        advance_head();
    }
    // The query copy is older than every ring load (the any-block-size layout issues more loads
    // than counted here and only waits longer).
    wait_loads_but<(R - 1) * 2 * NLD>();
    q_from_lds();

    // A full turn of the ring.  The rarely taken blocks below hold no K/V load, so the compiler's
    // load counters stay exact on the common path and a step waits only for its own slot.
    while (!(st & kDone)) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (r == 0) {
                // Claim ahead, once the head is close to the end of its unit: the answer is picked
                // up at the end of this turn, by when the slot requested right after the claim
                // has been waited for, and memory operations return in issue order.
                const bool want = st == kHeadInTail && hu.t1 - h_t <= kClaimAhead * STEP;
                st |= want ? kClaimPending : 0u;
                uint32_t *ctr = want ? &a.hdr->next_dunit_xcd[cq][0] : null_ctr;
                if (lane == 0) claim_v = atomicAdd(ctr, want ? 1u : 0u);
                lane_test_done();
            }
            // The head moves on once it has run out of its unit, the next unit is known and the
            // tail has reached the head's unit (the ring holds at most one unit boundary).
            if (h_t >= hu.t1 && (st & (kNextValid | kHeadInTail)) == (kNextValid | kHeadInTail)) {
                set_head(nx);
                st &= ~(kNextValid | kHeadInTail);
            }
            issue_step(ring[(r + R - 1) % R], slot_t[(r + R - 1) % R]);
            __builtin_amdgcn_sched_barrier(0);     // the new loads go out before this step's work
            advance_head();
            const int t_first = slot_t[r];
            consume(ring[r], t_first);
            __builtin_amdgcn_sched_barrier(0);
            if (t_first != kDummy && t_first + STEP >= cu.t1) {
                // last step of the tail's unit
                finish_unit(cu);
                if (a.evlog) {
                    if (lane == 0) log_event(a, kDecode, cu.id, tb);
                    lane_test_done();
                }
                ++n_done;
                if (st & kHeadInTail) {
                    // the head has run out of this unit and has nowhere to go yet
                    if (!(st & kNextValid)) fetch_next();
                    // Nothing left: the turn is finished with empty slots (leaving the loop from
                    // inside a turn makes the compiler lose its exact load counts), then the
                    // worker returns.
                    if (st & kNextValid) set_head(nx);
                    else st |= kDone;
                    st &= ~kNextValid;
                }
                cu = hu;
                st |= kHeadInTail;
                if (n_iss - q_mark < R) wait_all_loads();    // the query copy may still be in flight
                q_cur ^= 1;
                q_from_lds();
                reset_acc();
                if (a.evlog) tb = wall_clock64();
            }
            if (r == R - 1) {
                // (the claim's answer is read in every turn, wanted or not, so that every path
                // through a turn has the same outstanding operations)
                claim_v = (uint32_t)__builtin_amdgcn_readfirstlane(claim_v);
                if (st & kClaimPending) fetch_next();
            }
        }
    }
    return n_done;
}


template <int D> struct FusedLds {
    static constexpr int kBytes = PrefillLds<D>::kBytes > DecodeLds<D>::kBytes ? PrefillLds<D>::kBytes
                                                                               : DecodeLds<D>::kBytes;
};

// ------------------------------------------------------------------------------------------
// Stand-alone kernels: the in-house serial and two-stream baselines (Section 3.1).
// ------------------------------------------------------------------------------------------
template <int DT, int D, int LAYOUT>
__global__ __launch_bounds__(kWgThreads, 2) void prefill_kernel(KernelArgs a)
{
    __shared__ __attribute__((aligned(16))) unsigned char smem[PrefillLds<D>::kBytes];
    const uint64_t t0 = a.trace ? wall_clock64() : 0;
    prefill_item_run<DT, D, LAYOUT>(a, a.pitems_by_wg[blockIdx.x], smem);
    if (a.trace && threadIdx.x == 0)
        write_trace(a, blockIdx.x, __smid() & (kCuSlots - 1), kPrefill, 1, 0, t0, wall_clock64());
}

// A prefill worker: the workgroup claims prefill items until none is left, first from the queue
// of the XCD it runs on (the items of a K/V head sit in one queue, so their K/V tiles are re-read
// from that XCD's L2), then from the other XCDs' queues.
template <int DT, int D, int LAYOUT>
__device__ __forceinline__ int prefill_worker_run(const KernelArgs &a, unsigned char *smem, int *slot, int xcd)
{
    int n_done = 0;
    int q = xcd & (kXcdQueues - 1), tried = 0;
    for (;;) {
        __syncthreads();                            // previous item done with LDS and with *slot
        if (threadIdx.x == 0) {
            int item = -1;
            while (tried < kXcdQueues) {
                const int len = a.pq_begin[q + 1] - a.pq_begin[q];
                const int k = len > 0 ? (int)atomicAdd(&a.hdr->next_pitem_xcd[q], 1u) : len;
                if (k < len) { item = a.pq_begin[q] + k; break; }
                q = (q + 1) & (kXcdQueues - 1);     // this queue is empty for good: move on
                ++tried;
            }
            slot[0] = item;
            slot[1] = q | (tried << 8);
        }
        __syncthreads();
        // The claimed index is the same for every thread, but it comes out of LDS: say so, and read
        // the item through the constant address space, so that the item and everything derived
        // from it (key range, tile bases, block ids) stays in scalar registers as in the
        // stand-alone kernel.  Held in vector registers it cost the tile loop ~15 registers it
        // needs to keep LDS reads ahead of the matrix instructions.
        const int item = __builtin_amdgcn_readfirstlane(slot[0]);
        const int packed = __builtin_amdgcn_readfirstlane(slot[1]);
        q = packed & 255;
        tried = packed >> 8;
        if (item < 0) break;
        const uint64_t tb = a.evlog ? wall_clock64() : 0;
        PrefillItem it;
        {
            const POD_CONST int32_t *w = (const POD_CONST int32_t *)a.pitems + 8 * (int64_t)item;
            it.req = w[0]; it.kv_head = w[1]; it.row0 = w[2]; it.n_rows = w[3];
            it.kv_begin = w[4]; it.kv_end = w[5]; it.prow0 = w[6]; it.split = w[7];
        }
        prefill_item_run<DT, D, LAYOUT>(a, it, smem);
        if (a.evlog && threadIdx.x == 0) log_event(a, kPrefill, item, tb);
        ++n_done;
    }
    return n_done;
}

// Last workgroup of a launch that used the counters leaves them at zero for the next launch.
__device__ __forceinline__ void finish_and_reset(WsHeader *hdr, int *flag)
{
    __syncthreads();
    if (threadIdx.x == 0) {
        __threadfence();
        const uint32_t done = atomicAdd(&hdr->done, 1u);
        *flag = (done == gridDim.x - 1) ? 1 : 0;
    }
    __syncthreads();
    if (*flag) {
        for (int i = threadIdx.x; i < kCuSlots; i += kWgThreads) hdr->cu_state[i] = 0u;
        if (threadIdx.x == 0) {
            hdr->next_item[0] = 0u;
            hdr->next_item[1] = 0u;
            for (int q = 0; q < kXcdQueues; ++q) hdr->next_dunit_xcd[q][0] = 0u;
            hdr->done = 0u;
            for (int q = 0; q < kXcdQueues; ++q) hdr->next_pitem_xcd[q] = 0u;
        }
    }
}

template <int DT, int D, int LAYOUT>
__global__ __launch_bounds__(kWgThreads, 2) void decode_kernel(KernelArgs a)
{
    __shared__ __attribute__((aligned(16))) unsigned char smem[DecodeLds<D>::kBytes];
    __shared__ int flag;
    const uint64_t t0 = a.trace ? wall_clock64() : 0;
    // every workgroup of this kernel is a decode worker; its seat is its index
    const int xcd = __builtin_amdgcn_readfirstlane((int)(__smid() >> 6));
    const int n_done = decode_worker_run<DT, D, LAYOUT>(a, smem, blockIdx.x, xcd);
    if (a.trace) {
        __syncthreads();
        if (threadIdx.x == 0)
            write_trace(a, a.n_pitems + blockIdx.x, __smid() & (kCuSlots - 1), kDecode, n_done, 0, t0, wall_clock64());
    }
    finish_and_reset(a.hdr, &flag);
}

// ------------------------------------------------------------------------------------------
// The prefill-heavy configuration (the second of the two occupancy configurations of
// Section 4.2.2).  A compute unit holds 512 registers per SIMD lane and 160 KB of LDS; a prefill
// wavefront can be held to 208 registers and a prefill workgroup needs 64 KB, so two prefill
// workgroups leave 96 registers per lane and 28 KB of LDS on every unit (measured: a third
// workgroup with 28 KB is placed, one with 32 KB is not).  The decode workgroup below is built to
// fit exactly there: launched beside the prefill kernel it runs as the third workgroup of every
// unit, and the prefill work keeps both of its slots for the whole launch.  A register budget is a
// property of a kernel, not of a workgroup, so the two operations are two kernels here, started
// together on two streams; what places them on the same units is the resource arithmetic above
// (the trace records of both kernels show where each workgroup ran).
//
// With so little room the decode wavefront cannot keep its K/V stream in registers: the V rows
// of a 16-key step go straight into a 4 KB LDS region (direct-to-LDS loads, which need no
// destination registers), the K rows are loaded in matrix-operand order (lane = key row, 16 bytes
// of 8 channels) into 16 registers that are consumed by four matrix instructions as soon as they
// arrive and re-requested at once for the next step.  One step is in flight per wavefront while
// the previous one is computed: ~8 KB per wavefront, 32 KB per unit.  Alone on the chip that
// streams within 3-10 % of the full decode worker; beside two prefill workgroups per unit at
// about two thirds of it.
// ------------------------------------------------------------------------------------------
// Register budgets of the two kernels (the attribute below counts half of the unified file):
// 2 x 208 + 96 = 512 per SIMD lane.
constexpr int kHeavyPrefillVgprs = 208, kLiteVgprs = 96;
static_assert(2 * kHeavyPrefillVgprs + kLiteVgprs <= 512, "two prefill wavefronts and one decode wavefront per SIMD");
constexpr int kLiteLdsPerWave = 4 * 1024;      // V rows of one step: four groups of 4 keys x 256 bytes
constexpr int kLiteLdsBytes = kWavesPerWg * kLiteLdsPerWave;

template <int DT, int LAYOUT>
__global__ __launch_bounds__(kWgThreads) __attribute__((amdgpu_num_vgpr(kLiteVgprs / 2))) void decode_lite_kernel(KernelArgs a)
{
    static_assert(LAYOUT == kLayoutContiguous || LAYOUT == kLayoutPaged16, "a step must lie in one block");
    constexpr int D = 128, KS = D / 32, MB = D / 16, STEP = 16;
    using N = Num<DT>;
    using v8 = typename N::v8;
    using elem = typename N::elem;
    __shared__ __attribute__((aligned(4096))) unsigned char smem[kLiteLdsBytes];
    __shared__ int flag;
    const uint64_t t_start = a.trace ? wall_clock64() : 0;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int n16 = lane & 15;                     // K: key row of this lane; Q, S, P, O: query column (head of the group)
    const int b4 = lane >> 4;                      // K, Q: 8-channel piece of a 32-channel slice; S, P: keys 4*b4 .. 4*b4+3
    const int group = a.group;
    const int tok_bytes = a.tok_stride * 2;
    const bool col_ok = n16 < group;
    const float c = a.scale_log2;
    POD_LDS unsigned char *const lds_v = (POD_LDS unsigned char *)smem + wave * kLiteLdsPerWave;
    const uint32_t lds0 = (uint32_t)(uintptr_t)lds_v;
    const POD_CONST int32_t *const dq = (const POD_CONST int32_t *)a.dq_begin;

    // V in LDS.  Group g of a step (keys 4g .. 4g+3) is one direct load: lane (row b4, position
    // n16) lands at byte 16 * lane of the group's 1 KB.  Which 16-byte chunk of its row a lane
    // fetches is swizzled on the global side, chunk = position ^ (row << 2 | g), so that the
    // transposing reads below (16 lanes: 4 rows x 32 bytes of one group, the four groups at once)
    // spread over all banks.  Source offsets: row b4 of the group, the chunk for g = 0; group g
    // flips bits 4-5 of it (rows are at least 256 bytes apart, so the row part is not touched).
    const uint32_t v_src0 = (uint32_t)(b4 * tok_bytes + ((n16 ^ (b4 << 2)) << 4));
    // Reader: key 4*b4 + r4 (group b4, row r4), channels mb*16 + (n16 & 3)*4 .. +3, i.e. chunk
    // 2*mb + p1 and its upper or lower half; position = chunk ^ (r4 << 2 | b4).  Everything but mb
    // is fixed per lane, and mb only flips bits 5-7.
    const int r4 = n16 >> 2, p1 = (n16 >> 1) & 1;
    const uint32_t v_rd0 = (uint32_t)(b4 * 1024 + r4 * 256 + ((p1 ^ ((r4 << 2) | b4)) << 4) + (n16 & 1) * 8);
    // K in registers, in operand order: lane = (key row n16, channels 32*ks + 8*b4 .. +7).
    const uint32_t k_src0 = (uint32_t)(n16 * tok_bytes + b4 * 16);

    // ---- unit claims (the protocol of the decode worker: fixed first units, then the queues) ----
    int cq = __builtin_amdgcn_readfirstlane((int)(__smid() >> 6)) & (kXcdQueues - 1), tried = 0;
    auto claim_now = [&]() __attribute__((always_inline)) -> int {
        uint32_t v = 0;
        if (lane == 0) {
            uint32_t *ctr = &a.hdr->next_dunit_xcd[cq][0];
            asm volatile("global_atomic_add %0, %1, %2, off sc0\n\ts_waitcnt vmcnt(0)"
                         : "=&v"(v) : "v"(ctr), "v"(1u) : "memory");
        }
        lane_test_done();
        return (int)__builtin_amdgcn_readfirstlane(v);
    };
    auto claim_unit = [&]() __attribute__((always_inline)) -> int {
        if (tried >= kXcdQueues) return -1;
        int k = claim_now();
        for (;;) {
            const int q0 = dq[cq], q1 = dq[cq + 1];
            if (k < q1 - q0) return q0 + k;
            do {
                cq = (cq + 1) & (kXcdQueues - 1);
                ++tried;
            } while (tried < kXcdQueues && dq[cq + 1] == dq[cq]);
            if (tried >= kXcdQueues) return -1;
            k = claim_now();
        }
    };

    int n_done = 0;
    const int seat = blockIdx.x;
    int idx = seat < a.n_static_seats ? seat * kWavesPerWg + wave : claim_unit();
    while (idx >= 0 && idx < a.n_dunits) {
        idx = __builtin_amdgcn_readfirstlane(idx);
        const uint64_t tb = a.evlog ? wall_clock64() : 0;
        const POD_CONST int32_t *w = (const POD_CONST int32_t *)a.dunits + 8 * (int64_t)idx;
        const int kv_head = w[1], t0 = w[2], t1 = w[3], prow0 = w[4], q_start = w[6], cache_row = w[7];
        const elem *kc = (const elem *)a.k_cache + kv_head * a.head_stride;
        const elem *vc = (const elem *)a.v_cache + kv_head * a.head_stride;
        const POD_CONST int32_t *table = (const POD_CONST int32_t *)a.block_table +
                                         (int64_t)cache_row * a.max_blocks_per_seq;
        // element offset (head 0, channel 0) of key t, a multiple of 16: a step lies in one block
        auto base_of = [&](int t) __attribute__((always_inline)) -> int64_t {
            if constexpr (LAYOUT == kLayoutContiguous) {
                return (int64_t)cache_row * a.kv_seq_stride + (int64_t)t * a.tok_stride;
            } else {
                const int blk = table[t >> a.bs_shift];
                return (int64_t)blk * a.block_elems + (int64_t)(t & (a.block_size - 1)) * a.tok_stride;
            }
        };
        // query heads of the group: columns of the products, zero beyond the group
        v8 q[KS];
        {
            const char *qb = (const char *)((const elem *)a.decode_q +
                                            ((int64_t)q_start * a.n_q_heads + kv_head * group) * D);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                u32x4 raw = {0u, 0u, 0u, 0u};
                if (col_ok) raw = load16(qb + (n16 * D + ks * 32 + b4 * 8) * 2);
                q[ks] = __builtin_bit_cast(v8, raw);
            }
        }
        f32x4 o[MB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) o[mb] = f32x4{0.f, 0.f, 0.f, 0.f};
        float m_run = neg_inf(), l_run = 0.f;

        // Requests.  Keys past the unit's end re-read its last key (finite data; masked out of the
        // softmax by index), so every address is inside the unit's rows.
        u32x4 kreg[KS];
        // The lane offsets of a ragged last step are worked out where they are needed, from copies
        // the compiler cannot see through: otherwise it computes them ahead of the loop and holds a
        // dozen registers for a path taken once per unit.
        auto request_k = [&](int t) __attribute__((always_inline)) {
            const char *kb = (const char *)(kc + base_of(t));
            const int n_valid = min(t1 - t, STEP);
            uint32_t off = k_src0;
            if (n_valid < STEP) {
                uint32_t row = (uint32_t)n16, piece = (uint32_t)b4;
                asm volatile("" : "+v"(row), "+v"(piece));
                off = min(row, (uint32_t)(n_valid - 1)) * (uint32_t)tok_bytes + piece * 16u;
            }
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) kreg[ks] = load16_stream(kb + off + ks * 64);
        };
        auto request_v = [&](int t) __attribute__((always_inline)) {
            const char *vb = (const char *)(vc + base_of(t));
            const int n_valid = min(t1 - t, STEP);
            if (n_valid == STEP) {
                uint32_t src = v_src0;
                asm volatile("" : "+v"(src));
#pragma unroll
                for (int g = 0; g < 4; ++g) dma16_stream(lds0 + g * 1024, src ^ (uint32_t)(g << 4), vb + (int64_t)4 * g * tok_bytes);
            } else {
                uint32_t row = (uint32_t)b4, pos = (uint32_t)n16;
                asm volatile("" : "+v"(row), "+v"(pos));
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const uint32_t src_row = min(4u * g + row, (uint32_t)(n_valid - 1));
                    dma16_stream(lds0 + g * 1024, src_row * (uint32_t)tok_bytes + ((pos ^ ((row << 2) | g)) << 4), vb);
                }
            }
        };

        request_k(t0);
        request_v(t0);
        for (int t = t0; t < t1; t += STEP) {
            const bool more = t + STEP < t1;
            // S^T = K Q^T: register r holds key t + 4*b4 + r of query column n16
            f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) s = N::mfma16(__builtin_bit_cast(v8, kreg[ks]), q[ks], s);
            __builtin_amdgcn_sched_barrier(0);
            if (more) request_k(t + STEP);                    // into the registers just consumed
            const int n_valid = min(t1 - t, STEP) - 4 * b4;   // keys of this lane that exist
#pragma unroll
            for (int r = 0; r < 4; ++r) s[r] = (r < n_valid) ? s[r] : neg_inf();
            float mx = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
            mx = max_across_32(max_across_16(mx)) * c;
            const bool grow = mx > m_run + kMaxSlack;         // also true for the first key
            if (__builtin_amdgcn_ballot_w64(grow) != 0) {
                const float alpha = grow ? fast_exp2(m_run - mx) : 1.f;
                m_run = grow ? mx : m_run;
                l_run *= alpha;
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) o[mb] = o[mb] * alpha;
            }
            const float m_use = (m_run == neg_inf()) ? 0.f : m_run;
            typename N::v4 pk;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float p = fast_exp2(__builtin_fmaf(s[r], c, -m_use));
                l_run += p;
                pk[r] = (elem)p;
            }
            // The V rows of this step were requested one step ago; the only requests younger than
            // them are the four K loads just issued.
            if (more) wait_loads_but<KS>();
            else wait_all_loads();
            // O^T += V^T P^T: rows = channels, contraction over the 16 keys in S's register order.
            // The address of block mb is one XOR away from the lane's base (kept opaque so that the
            // eight addresses are not held in registers); reads run two blocks ahead of their use.
            {
                uint32_t v_base = lds0 + v_rd0;           // the region is 4 KB aligned: bits 5-7 are the lane's own
                asm volatile("" : "+v"(v_base));
                constexpr int kAheadV = 2;
                auto v_at = [&](int mb) __attribute__((always_inline)) {
                    return lds_read_tr((const POD_LDS unsigned char *)(uintptr_t)(v_base ^ (uint32_t)(mb << 5)));
                };
                s16x4 vv[MB];
#pragma unroll
                for (int mb = 0; mb < kAheadV; ++mb) vv[mb] = v_at(mb);
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    if (mb + kAheadV < MB) vv[mb + kAheadV] = v_at(mb + kAheadV);
                    o[mb] = N::mfma16k16(vv[mb], pk, o[mb]);
                }
                __builtin_amdgcn_sched_group_barrier(0x100, kAheadV, 0);
#pragma unroll
                for (int mb = 0; mb < MB - kAheadV; ++mb) {
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                }
                __builtin_amdgcn_sched_group_barrier(0x008, kAheadV, 0);
            }
            // the region is free once the reads have returned
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            if (more) request_v(t + STEP);
        }

        // o[mb][r] is channel mb*16 + 4*b4 + r of query column n16
        const float l_tot = sum_across_32(sum_across_16(l_run));
        if (col_ok) {
            if (prow0 < 0) {
                const float inv = 1.f / l_tot;
                elem *op = (elem *)a.out +
                    ((int64_t)(a.n_prefill_rows + q_start) * a.n_q_heads + kv_head * group + n16) * D;
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    typename N::v4 wv;
#pragma unroll
                    for (int e = 0; e < 4; ++e) wv[e] = (elem)(o[mb][e] * inv);
                    *(typename N::v4 *)(op + mb * 16 + 4 * b4) = wv;
                }
            } else {
                const int64_t prow = (int64_t)prow0 + n16;
                float *po = a.part_o + prow * D;
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) *(f32x4 *)(po + mb * 16 + 4 * b4) = o[mb];
                if (b4 == 0) {
                    a.part_ml[prow * 2 + 0] = m_run;
                    a.part_ml[prow * 2 + 1] = l_tot;
                }
            }
        }
        lane_test_done();
        if (a.evlog) {
            if (lane == 0) log_event(a, kDecode, idx, tb);
            lane_test_done();
        }
        ++n_done;
        idx = claim_unit();
    }
    if (a.trace) {
        __syncthreads();
        if (threadIdx.x == 0)
            write_trace(a, a.n_pitems + blockIdx.x, __smid() & (kCuSlots - 1), kDecode, n_done, 0, t_start, wall_clock64());
    }
    finish_and_reset(a.hdr, &flag);
}

// The prefill kernel of that configuration: the stand-alone prefill kernel, held to 208 registers
// (seven values go to scratch memory at head_dim 128; the kernel measures 1-3 % faster, not
// slower) so that two of its workgroups and one light decode workgroup fill a unit's register file.
template <int DT, int D, int LAYOUT>
__global__ __launch_bounds__(kWgThreads, 2) __attribute__((amdgpu_num_vgpr(kHeavyPrefillVgprs / 2))) void prefill_heavy_kernel(KernelArgs a)
{
    __shared__ __attribute__((aligned(16))) unsigned char smem[PrefillLds<D>::kBytes];
    const uint64_t t0 = a.trace ? wall_clock64() : 0;
    prefill_item_run<DT, D, LAYOUT>(a, a.pitems_by_wg[blockIdx.x], smem);
    if (a.trace && threadIdx.x == 0)
        write_trace(a, blockIdx.x, __smid() & (kCuSlots - 1), kPrefill, 1, 0, t0, wall_clock64());
}

// ------------------------------------------------------------------------------------------
// Fused kernel.  One resident round of workgroups (two per compute unit); each binds its first
// operation after it has been placed on a compute unit (Section 4.1): the leader reads the
// hardware unit id, takes a ticket from that unit's counter and chooses the operation that keeps
// the unit's resident mix at the prefill:decode ratio, so that every unit runs both at once.  A
// workgroup then works as a persistent worker (Section 4.4): it claims work of its operation from
// the shared counters until none is left, switches to the other operation (the listing's "switch
// ops" step), and ends when both are exhausted.  As a prefill worker the whole workgroup takes
// one item at a time; as a decode worker each of its wavefronts takes units on its own
// (Section 4.2.3).  No workgroup ever waits for another one.
// ------------------------------------------------------------------------------------------
template <int DT, int D, int LAYOUT>
__global__ __launch_bounds__(kWgThreads, 2) void fused_kernel(KernelArgs a)
{
    __shared__ __attribute__((aligned(16))) unsigned char smem[FusedLds<D>::kBytes];
    __shared__ int bind[6];                                  // role, seat, unit id, last flag, item, queue
    WsHeader *hdr = a.hdr;
    const uint64_t t0 = a.trace ? wall_clock64() : 0;
    if (threadIdx.x == 0) {
        const unsigned cu = __smid() & (kCuSlots - 1);
        const uint32_t ticket = atomicAdd(&hdr->cu_state[cu], 1u);
        bind[0] = role_for_ticket(ticket, a.p_ratio, a.d_ratio, (int)cu);
        bind[2] = (int)cu;
    }
    __syncthreads();
    const int first = bind[0];
    const int xcd = bind[2] >> 6;                            // unit id = xcc << 6 | se << 4 | cu
    int n_first, n_second;
    uint64_t t_switch = 0;
    // A workgroup takes its decode seat when it enters the decode operation, first or second.
    // There are n_dwgs seats, one per compute unit: the decode stream is fastest with four
    // wavefronts per unit (more of them only queue up in the memory system and slow each other
    // down unevenly), so a workgroup that finds every seat taken leaves the decode work to the
    // seated ones.  Every workgroup asks for a seat sooner or later and the grid has at least
    // n_dwgs workgroups, so all seats, and with them all fixed first units, are taken.
    auto take_seat = [&]() {
        __syncthreads();
        if (threadIdx.x == 0) bind[1] = (int)atomicAdd(&hdr->next_item[kDecode], 1u);
        __syncthreads();
        const int seat = bind[1];
        return seat;
    };
    if (first == kPrefill) {
        n_first = prefill_worker_run<DT, D, LAYOUT>(a, smem, &bind[4], xcd);
        if (a.trace) t_switch = wall_clock64();
        const int seat = take_seat();
        n_second = seat < a.n_dwgs ? decode_worker_run<DT, D, LAYOUT>(a, smem, seat, xcd) : 0;
    } else {
        const int seat = take_seat();
        n_first = seat < a.n_dwgs ? decode_worker_run<DT, D, LAYOUT>(a, smem, seat, xcd) : 0;
        if (a.trace) t_switch = wall_clock64();
        n_second = prefill_worker_run<DT, D, LAYOUT>(a, smem, &bind[4], xcd);
    }
    __syncthreads();
    if (threadIdx.x == 0 && a.trace) write_trace(a, blockIdx.x, bind[2], first, n_first, n_second, t0, t_switch);
    finish_and_reset(hdr, &bind[3]);
}

// ------------------------------------------------------------------------------------------
// CTA-parallel fused kernel: the launch of Section 4.1's listing as printed.  One workgroup per
// work item (a prefill item, or a decode workgroup of four one-wavefront units); the hardware
// places workgroups as slots come free.  Each one reads its hardware unit id, takes that unit's
// ticket, picks its operation with the ticket rule, claims the next work id of that operation from
// a global counter, switches operation if that counter has run past its limit, runs the one item
// and leaves.  The persistent kernel above is the variant of Section 4.4; this one exists so that
// the two can be timed against each other on this chip.
// ------------------------------------------------------------------------------------------
template <int DT, int D, int LAYOUT>
__global__ __launch_bounds__(kWgThreads, 2) void fused_cta_kernel(KernelArgs a)
{
    __shared__ __attribute__((aligned(16))) unsigned char smem[FusedLds<D>::kBytes];
    __shared__ int bind[4];                                  // role, work id, unit id, last flag
    WsHeader *hdr = a.hdr;
    const uint64_t t0 = a.trace ? wall_clock64() : 0;
    if (threadIdx.x == 0) {
        const unsigned cu = __smid() & (kCuSlots - 1);
        const uint32_t ticket = atomicAdd(&hdr->cu_state[cu], 1u);
        int role = role_for_ticket(ticket, a.p_ratio, a.d_ratio, (int)cu);
        int id = -1;
        for (int attempt = 0; attempt < 2 && id < 0; ++attempt) {
            const uint32_t limit = (uint32_t)(role == kPrefill ? a.n_pitems : a.n_dctas);
            const uint32_t k = atomicAdd(&hdr->next_item[role], 1u);
            if (k < limit) id = (int)k;
            else role ^= 1;                                  // that operation has no work left: the other one
        }
        bind[0] = id < 0 ? (int)kNone : role;
        bind[1] = id;
        bind[2] = (int)cu;
    }
    __syncthreads();
    const int role = bind[0];
    const int id = __builtin_amdgcn_readfirstlane(bind[1]);
    int n_done = 0;
    if (role == kPrefill) {
        PrefillItem it;
        const POD_CONST int32_t *w = (const POD_CONST int32_t *)a.pitems + 8 * (int64_t)id;
        it.req = w[0]; it.kv_head = w[1]; it.row0 = w[2]; it.n_rows = w[3];
        it.kv_begin = w[4]; it.kv_end = w[5]; it.prow0 = w[6]; it.split = w[7];
        prefill_item_run<DT, D, LAYOUT>(a, it, smem);
        n_done = 1;
    } else if (role == kDecode) {
        n_done = decode_worker_run<DT, D, LAYOUT>(a, smem, id, bind[2] >> 6);
    }
    __syncthreads();
    if (threadIdx.x == 0 && a.trace) write_trace(a, blockIdx.x, bind[2], role, n_done, 0, t0, wall_clock64());
    finish_and_reset(hdr, &bind[3]);
}

// ------------------------------------------------------------------------------------------
// Combine: merge split-KV partials.  With running maxima m_s (log2 domain), weight sums l_s and
// un-normalised outputs O_s:  M = max m_s,  out = sum_s O_s 2^(m_s - M) / sum_s l_s 2^(m_s - M).
// ------------------------------------------------------------------------------------------
template <int DT, int D>
__global__ __launch_bounds__(kWgThreads) void combine_kernel(KernelArgs a)
{
    using N = Num<DT>;
    constexpr int TPR = D / 4;                      // threads per row, 4 channels each
    constexpr int RPP = kWgThreads / TPR;           // rows per pass
    constexpr int U = 8;                            // splits fetched together (independent loads)
    // every group of TPR threads merges one output row; a workgroup takes RPP rows of the list
    const int group = a.group;
    const int sub = threadIdx.x % TPR;
    const int crow = blockIdx.x * RPP + threadIdx.x / TPR;
    if (crow < a.n_crows) {
        const int2 er = *(const int2 *)(a.crows + 2 * (int64_t)crow);
        const CombineEntry e = a.centries[er.x];
        const int r = er.y;
        int64_t out_row;
        int hq;
        if (e.kind == kPrefill) {
            const int R = e.row0 + r;
            const int tok = R / group;
            hq = e.kv_head * group + (R - tok * group);
            out_row = e.q_start + tok;
        } else {
            hq = e.kv_head * group + r;
            out_row = (int64_t)a.n_prefill_rows + e.q_start;
        }
        float M = neg_inf(), lsum = 0.f;
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        for (int s0 = 0; s0 < e.n_splits; s0 += U) {
            float ms[U], ls[U];
            f32x4 v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int s = min(s0 + u, e.n_splits - 1);
                const int64_t prow = (int64_t)e.prow0 + (int64_t)s * e.split_stride + r;
                const float2 ml = *(const float2 *)(a.part_ml + prow * 2);
                ms[u] = (s0 + u < e.n_splits) ? ml.x : neg_inf();
                ls[u] = ml.y;
                v[u] = *(const f32x4 *)(a.part_o + prow * D + sub * 4);
            }
            float Mn = M;
#pragma unroll
            for (int u = 0; u < U; ++u) Mn = fmaxf(Mn, ms[u]);
            if (Mn == neg_inf()) continue;          // no split so far saw a key of this row
            const float keep = fast_exp2(M - Mn);   // 0 while M is still -inf
            lsum *= keep;
            acc = acc * keep;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const float w = fast_exp2(ms[u] - Mn);   // 0 for a split that saw no key
                lsum += ls[u] * w;
                acc += v[u] * w;
            }
            M = Mn;
        }
        const float inv = 1.f / lsum;
        typename N::v4 w4;
#pragma unroll
        for (int i = 0; i < 4; ++i) w4[i] = (typename N::elem)(acc[i] * inv);
        *(typename N::v4 *)((typename N::elem *)a.out + (out_row * a.n_q_heads + hq) * D + sub * 4) = w4;
    }
}

__global__ void clear_header_kernel(WsHeader *hdr)
{
    uint32_t *p = (uint32_t *)hdr;
    for (int i = threadIdx.x + blockIdx.x * blockDim.x; i < (int)(sizeof(WsHeader) / 4);
         i += blockDim.x * gridDim.x)
        p[i] = 0u;
}

// ------------------------------------------------------------------------------------------
// Host-side launchers.
// ------------------------------------------------------------------------------------------
template <int DT, int D, int LAYOUT>
static hipError_t launch_variant(int which, const KernelArgs &a, hipStream_t stream)
{
    switch (which) {
    case kLaunchPrefill:
        if (a.n_pitems > 0)
            prefill_kernel<DT, D, LAYOUT><<<dim3(a.n_pitems), dim3(kWgThreads), 0, stream>>>(a);
        break;
    case kLaunchDecode:
        if (a.n_dwgs > 0)
            decode_kernel<DT, D, LAYOUT><<<dim3(a.n_dwgs), dim3(kWgThreads), 0, stream>>>(a);
        break;
    case kLaunchFused:
        if (a.fused_grid > 0)
            fused_kernel<DT, D, LAYOUT><<<dim3(a.fused_grid), dim3(kWgThreads), 0, stream>>>(a);
        break;
    case kLaunchFusedCta:
        if (a.n_pitems + a.n_dctas > 0)
            fused_cta_kernel<DT, D, LAYOUT><<<dim3(a.n_pitems + a.n_dctas), dim3(kWgThreads), 0, stream>>>(a);
        break;
    case kLaunchPrefillHeavy:
        if constexpr (D == 128 && LAYOUT != kLayoutPagedAny) {
            if (a.n_pitems > 0)
                prefill_heavy_kernel<DT, D, LAYOUT><<<dim3(a.n_pitems), dim3(kWgThreads), 0, stream>>>(a);
        } else {
            return hipErrorInvalidValue;
        }
        break;
    case kLaunchDecodeLite:
        if constexpr (D == 128 && LAYOUT != kLayoutPagedAny) {
            if (a.n_dwgs > 0)
                decode_lite_kernel<DT, LAYOUT><<<dim3(a.n_dwgs), dim3(kWgThreads), 0, stream>>>(a);
        } else {
            return hipErrorInvalidValue;
        }
        break;
    case kLaunchCombine:
        if (a.n_crows > 0) {
            constexpr int kRowsPerWg = kWgThreads / (D / 4);
            combine_kernel<DT, D><<<dim3((a.n_crows + kRowsPerWg - 1) / kRowsPerWg), dim3(kWgThreads), 0, stream>>>(a);
        }
        break;
    default:
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <int DT, int D>
static hipError_t launch_layout(int which, const KernelArgs &a, int layout, hipStream_t stream)
{
    switch (layout) {
    case kLayoutContiguous: return launch_variant<DT, D, kLayoutContiguous>(which, a, stream);
    case kLayoutPaged16: return launch_variant<DT, D, kLayoutPaged16>(which, a, stream);
    case kLayoutPagedAny: return launch_variant<DT, D, kLayoutPagedAny>(which, a, stream);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch(int which, const KernelArgs &a, int dtype, int head_dim, bool paged, hipStream_t stream)
{
    // The block-wise paths want power-of-two blocks of at least 16 keys whose byte size fits 32 bits.
    const bool block_wise = a.bs_shift >= 4 && a.block_elems * 2 < (1ll << 32);
    const int layout = !paged ? kLayoutContiguous : (block_wise ? kLayoutPaged16 : kLayoutPagedAny);
    if (dtype == 0 && head_dim == 128) return launch_layout<0, 128>(which, a, layout, stream);
    if (dtype == 0 && head_dim == 64) return launch_layout<0, 64>(which, a, layout, stream);
    if (dtype == 1 && head_dim == 128) return launch_layout<1, 128>(which, a, layout, stream);
    if (dtype == 1 && head_dim == 64) return launch_layout<1, 64>(which, a, layout, stream);
    if (dtype == 0 && head_dim == 256) return launch_layout<0, 256>(which, a, layout, stream);
    if (dtype == 1 && head_dim == 256) return launch_layout<1, 256>(which, a, layout, stream);
    return hipErrorInvalidValue;
}

hipError_t clear_header(WsHeader *hdr, hipStream_t stream)
{
    clear_header_kernel<<<dim3(1), dim3(256), 0, stream>>>(hdr);
    return hipGetLastError();
}

// Workspace of the entry point that allocates nothing.  In host code the name below is only a
// handle for the symbol, not a device address: the address of each GPU's copy comes from
// hipGetSymbolAddress, once per device with that device current, and only that address is ever
// handed to kernels and copies.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

hipError_t static_scratch(void **ptr)
{
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void *per_device[kMaxDevices] = {nullptr};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!per_device[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        per_device[dev] = p;
    }
    *ptr = per_device[dev];
    return hipSuccess;
}

}  // namespace pod
