// Shared declarations of the gfx950 Stream kernels (device + host side of the library).
// Nothing in here is used by the CPU oracle.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "stream.h"

namespace stream {

constexpr int kMaxBatch = 64;   // sequence descriptors travel as kernel arguments (2 KB of the 4 KB a launch may pass)
constexpr int kMaxTopk = 64;    // one node per lane of a 64-wide wavefront (narrow kernels)
constexpr int kMaxTopkWide = 512;   // stream_prune / stream_prune_variable / stream_sparse_attn: lists of up to 512 blocks
constexpr int kXcds = 8;        // MI355X: 8 XCDs, workgroups are dealt to them round-robin

// One sequence of the packed batch.
struct SeqDesc {
    long long tok0;  // first token in the packed token axis
    int len;         // L_s real tokens
    int nblk;        // query blocks T_p / b_q, T_p = L_s rounded up to a multiple of lcm(b_q, b_k)
    int blk0;        // first global block id
    int k;           // k_s
    int levels;      // refinement levels to run: max(1, ceil(log2(ceil(N_k / k_s)))), N_k = T_p / b_k
    int pad_;
};

struct SeqTable {
    int n;
    int pad_[3];
    SeqDesc d[kMaxBatch];
};

// Workgroup -> (kv head, slot) mapping that keeps each XCD's L2 on as few key heads as it can.
enum MapMode { kMapPlain = 0, kMapKvMultipleOfXcd = 1, kMapKvDividesXcd = 2 };

struct WgMap {
    int mode;
    int per_kv;   // work items (workgroups) per kv head
    int kv_heads;
    int grid;     // workgroups to launch
};

inline WgMap make_wg_map(int kv_heads, int per_kv)
{
    WgMap m;
    m.kv_heads = kv_heads;
    m.per_kv = per_kv;
    if (kv_heads % kXcds == 0) {
        m.mode = kMapKvMultipleOfXcd;
        m.grid = kv_heads * per_kv;
    } else if (kXcds % kv_heads == 0) {
        m.mode = kMapKvDividesXcd;
        int r = kXcds / kv_heads;
        m.grid = kXcds * ((per_kv + r - 1) / r);
    } else {
        m.mode = kMapPlain;
        m.grid = kv_heads * per_kv;
    }
    return m;
}

// Returns false when this workgroup has no work.
__device__ __forceinline__ bool wg_decode(const WgMap &m, int wg, int &kvh, int &slot)
{
    if (m.mode == kMapKvMultipleOfXcd) {
        int x = wg % kXcds, i = wg / kXcds;
        kvh = x + kXcds * (i / m.per_kv);
        slot = i % m.per_kv;
        return true;
    }
    if (m.mode == kMapKvDividesXcd) {
        int x = wg % kXcds, i = wg / kXcds;
        int r = kXcds / m.kv_heads;
        kvh = x % m.kv_heads;
        slot = i * r + x / m.kv_heads;
        return slot < m.per_kv;
    }
    kvh = wg / m.per_kv;
    slot = wg % m.per_kv;
    return true;
}

// Sequence that owns global block gb (linear scan: the table is tiny and the scan is scalar).
__device__ __forceinline__ int seq_of_block(const SeqTable &t, int gb)
{
    int s = 0;
    while (s + 1 < t.n && gb >= t.d[s + 1].blk0) ++s;
    return s;
}

// Mask rule C (stream_mask) at token and at block level.  Blocks: key block r is valid for
// query block q when one of its keys is visible to one of q's queries; the valid blocks of a
// row are the contiguous range [mask_rmin, mask_rmax].
__host__ __device__ __forceinline__ bool mask_token(int mask, int window, int tq, int tk)
{
    // branch-free on purpose (| and & on bools): this sits in per-element code of the kernels
    const bool causal_ok = tk <= tq;
    const bool window_ok = (mask != STREAM_MASK_SLIDING) | (tq - tk < window);
    return (mask == STREAM_MASK_FULL) | (causal_ok & window_ok);
}

// Blocks: queries come in blocks of bq tokens, keys in blocks of bk tokens (b_q, b_k of Alg. 2).
__host__ __device__ __forceinline__ int mask_rmin(int mask, int window, int q, int bq, int bk)
{
    if (mask != STREAM_MASK_SLIDING) return 0;
    // the first query of the block, q*bq, sees keys > q*bq - window
    const long long lo = (long long)q * bq - window + 1;           // first visible key (may be < 0)
    if (lo <= 0) return 0;
    return (int)(lo / bk);                                          // key block that contains it
}

// -1 for a query block that holds no real token (padding up to lcm(bq, bk))
__host__ __device__ __forceinline__ int mask_rmax(int mask, int q, int bq, int bk, int L)
{
    const long long first = (long long)q * bq;
    if (first >= L) return -1;
    // the last real query of the block sees keys up to itself (no mask: up to the last key)
    const long long last = mask == STREAM_MASK_FULL || first + bq > L ? (long long)L - 1 : first + bq - 1;
    return (int)(last / bk);
}

#if defined(__HIPCC__)
// Packed K/V tiles are read with raw buffer loads: a scalar resource (base + size, so a read
// past the region returns zeros instead of faulting), a scalar byte offset that selects the tile
// and a per-lane offset.  One fragment = 64 lanes x 16 bytes = 1 KiB; fragment j of a tile sits
// at byte j * 1024.  The split below keeps the per-lane part inside the 12-bit immediate.
typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_tile_rsrc(const void *base, unsigned bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}

__device__ __forceinline__ uint4 load_frag(__amdgpu_buffer_rsrc_t rs, unsigned lane_off,
                                           unsigned tile_off, int j)
{
    const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(rs, lane_off + (j & 3) * 1024,
                                                            tile_off + (j >> 2) * 4096, 0);
    return make_uint4(v[0], v[1], v[2], v[3]);
}
#endif

// Host-side validated problem description shared by both entry points.
struct Problem {
    int H, Hkv, g, d, b, bk, dtype, esize, batch, kmax;   // b = b_q (query block), bk = b_k
    int mask, window;         // stream_mask rule; window in tokens (sliding window only)
    const unsigned *cbits;    // STREAM_MASK_ARRAY: the T x T bit array (device) and its row pitch in words
    long long cpitch;
    long long T;
    int NB;
    SeqTable seqs;
    int max_levels;
};

stream_status make_problem(const stream_shape *s, int topk, const int *topk_per_seq, int topk_max,
                           Problem *out);

size_t align_up(size_t x, size_t a);

// Packs a [kv_heads, T, d] tensor into block tiles whose 16-byte chunks are ordered the way the
// 32x32 MFMA operand fragments are read: see pack_kernel in stream_pack.hip.
// STREAM_MASK_ARRAY: block-level summaries of the bit array C for query blocks of b_q and key
// blocks of b_k tokens, one bit per (query block, key block), rows of block_bitmap_words(pb)
// words: any = C^blk of Alg. 2 (some real pair of the block is visible), all = every pair of
// the block is real and visible (no token-level test needed).
int block_bitmap_words(const Problem &pb);
stream_status launch_block_bitmaps(const Problem &pb, unsigned *any_bits, unsigned *all_bits, hipStream_t st);

// Fragment shape of the packed copy: kPackFrag32 - a fragment is 32 rows x 32 bytes (operands of the
// 32x32 MFMAs), kPackFrag16 - 16 rows x 64 bytes (operands of the 16x16x32 bf16 MFMA).
enum PackLayout { kPackFrag32 = 0, kPackFrag16 = 1 };

stream_status launch_pack(const void *src, long long stride_h, long long stride_t, void *dst,
                          const Problem &pb, hipStream_t st, PackLayout layout = kPackFrag32);

}  // namespace stream
