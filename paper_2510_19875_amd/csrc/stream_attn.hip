// stream_sparse_attn: Eq. (2) of the paper on the retained key blocks, gfx950.
//
// A wavefront owns up to 64 query tokens of one (head, query block) and walks the block's
// retained key blocks in ascending order with a running softmax.  K tiles come from the same
// packed layout the pruning kernels use; V tiles are packed transposed so that a lane's 16
// bytes hold one feature of the 8 (bf16) or 4 (fp32) keys its MFMA contraction slots cover.
//
// Pass 1 computes S^T = K Q^T with 32x32 MFMAs: a lane then owns one query column and 16 key
// rows per accumulator, so the softmax statistics are per lane (plus one exchange between the
// two lane halves) and the probabilities already sit in B-operand order for O^T += V^T P^T.
// Pass 2 (only when the received mass is requested) recomputes S = Q K^T, where a lane owns one
// key column, turns it into probabilities with the final row normalisers and adds the column
// sums to mass[] with atomics.
#include "stream_mfma.h"

#include <math.h>

namespace stream {


// ---------------------------------------------------------------------------------------------
// V packing.  Per 32-key group and per 32-feature block db, fragment vf holds for lane
// (mrow = lane % 32, gh = lane / 32) the values V[key][db*32 + mrow] of the keys
//     bf16: element e of fragment vf (2 per group): key = (2*vf + e/4)*8 + gh*4 + e%4
//     fp32: element e of fragment vf (4 per group): key = vf*8 + gh*4 + e
// which are exactly the key rows a lane's S^T accumulator elements cover, in order.
// Layout: [kv_head][global block][group][db][vf][lane] x 16 bytes.
// ---------------------------------------------------------------------------------------------
struct PackVParams {
    const char *src;
    char *dst;
    long long stride_h_bytes, stride_t_bytes;
    int d, esize, b, NB;
    SeqTable seqs;
};

__global__ void __launch_bounds__(256) pack_v_kernel(PackVParams p)
{
    const int groups = p.b / 32;
    const int ndb = p.d / 32;
    const int nvf = p.esize == 2 ? 2 : 4;
    const long long grp = blockIdx.x;
    const int gi = (int)(grp % groups);
    const long long t = grp / groups;
    const int gb = (int)(t % p.NB);
    const int kvh = (int)(t / p.NB);
    const int s = seq_of_block(p.seqs, gb);
    const SeqDesc sd = p.seqs.d[s];
    const int tok0 = (gb - sd.blk0) * p.b + gi * 32;
    char *dst = p.dst + grp * (32LL * p.d * p.esize);
    const char *src = p.src + kvh * p.stride_h_bytes;
    for (int c = threadIdx.x; c < ndb * nvf * 64; c += blockDim.x) {
        const int lane = c & 63, vf = (c >> 6) % nvf, db = (c >> 6) / nvf;
        const int mrow = lane & 31, gh = lane >> 5;
        uint4 out = make_uint4(0, 0, 0, 0);
        if (p.esize == 2) {
            unsigned short v[8];
            for (int e = 0; e < 8; ++e) {
                const int key = (2 * vf + (e >> 2)) * 8 + gh * 4 + (e & 3);
                const int tok = tok0 + key;
                v[e] = tok < sd.len ? *reinterpret_cast<const unsigned short *>(
                                          src + (sd.tok0 + tok) * p.stride_t_bytes + (db * 32 + mrow) * 2)
                                    : (unsigned short)0;
            }
            out.x = v[0] | ((unsigned)v[1] << 16); out.y = v[2] | ((unsigned)v[3] << 16);
            out.z = v[4] | ((unsigned)v[5] << 16); out.w = v[6] | ((unsigned)v[7] << 16);
        } else {
            unsigned v[4];
            for (int e = 0; e < 4; ++e) {
                const int key = vf * 8 + gh * 4 + e;
                const int tok = tok0 + key;
                v[e] = tok < sd.len ? *reinterpret_cast<const unsigned *>(
                                          src + (sd.tok0 + tok) * p.stride_t_bytes + (db * 32 + mrow) * 4)
                                    : 0u;
            }
            out = make_uint4(v[0], v[1], v[2], v[3]);
        }
        *reinterpret_cast<uint4 *>(dst + (long long)c * 16) = out;
    }
}

struct AttnParams {
    const char *Q;
    const char *Kp, *Vp;
    char *O;
    long long q_sh_b, q_st_b, o_sh_b, o_st_b;
    const int *idx, *cnt;
    float *lse, *mass;           // nullable
    float *lse2;                 // workspace [H, T]: base-2 log-sum-exp, written by pass 1 for pass 2
    long long T;
    int H, g, NB, kmax;
    float scale_log2e;           // scale * log2(e): softmax runs in base 2
    int mask, window;            // the mask rule C (stream_mask) and its window
    // STREAM_MASK_ARRAY (ARB kernels): the bit array C, its "wholly visible" block summary
    // [NB, cw] and the words per row of the summary
    const unsigned *cbits, *call;
    long long cpitch;
    int cw;
    WgMap map;
    SeqTable seqs;
};
static_assert(sizeof(AttnParams) <= 4096, "kernel arguments are limited to 4 KB");

typedef float floatx8 __attribute__((ext_vector_type(8)));

template <bool BF16>
__device__ __forceinline__ floatx16 mfma16(const uint4 &a, const uint4 &b, floatx16 c)
{
    if constexpr (BF16) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                       __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    } else {
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_bit_cast(float, a.x), __builtin_bit_cast(float, b.x), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_bit_cast(float, a.y), __builtin_bit_cast(float, b.y), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_bit_cast(float, a.z), __builtin_bit_cast(float, b.z), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_bit_cast(float, a.w), __builtin_bit_cast(float, b.w), c, 0, 0, 0);
        return c;
    }
}

// Bit pattern of a float taken BY VALUE.  (__builtin_bit_cast applied directly to an element of
// an ext_vector_type lvalue reads element 0 whatever the index, with this compiler.)
__device__ __forceinline__ unsigned f2u(float v) { return __builtin_bit_cast(unsigned, v); }

// Eight probabilities -> one bf16 B-operand fragment (round to nearest even, v_cvt_pk_bf16_f32).
__device__ __forceinline__ uint4 to_bf16_frag(float a, float b, float c, float d, float e, float f,
                                               float g, float h)
{
    floatx8 t = {a, b, c, d, e, f, g, h};
    return __builtin_bit_cast(uint4, __builtin_convertvector(t, bf16x8));
}

__device__ __forceinline__ unsigned pack_bf16x2(float lo, float hi)
{
    typedef float floatx2 __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    floatx2 t = {lo, hi};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(t, bf16x2));
}

// S^T += K-fragment x Q-fragment with the result in ordinary vector registers.  The compiler
// keeps every MFMA result of a one-wave-per-SIMD kernel in the accumulation registers, from
// where the softmax would have to copy each score out again; the scores are consumed by vector
// instructions only, so the pipelined loop issues these MFMAs itself.  Callers keep two MFMAs
// or more between the last of these and the first read of its result (the wait the hardware
// does not enforce); accumulation onto the same registers back to back is interlocked.
__device__ __forceinline__ void qk_mfma_bf16(floatx16 &c, const uint4 &a, const u32x4_t &bv, bool first)
{
    const u32x4_t av = {a.x, a.y, a.z, a.w};
    if (first)
        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(c) : "v"(av), "a"(bv));
    else
        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(c) : "v"(av), "a"(bv));
}

// acc + lo + hi of a packed bf16 pair (v_dot2c_f32_bf16 against (1, 1)).
__device__ __forceinline__ float dot2_ones(unsigned pair, float acc)
{
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, pair),
                                           __builtin_bit_cast(bf16x2_t, 0x3f803f80u), acc, false);
}

// Compile-time loop: f(integral_constant<int, I>) for I = 0 .. N-1.
template <int I> struct IntC { static constexpr int value = I; };
template <int I, int N, class F>
__device__ __forceinline__ void static_for(F &f)
{
    if constexpr (I < N) {
        f(IntC<I>{});
        static_for<I + 1, N>(f);
    }
}

// NQ: 32-query groups per wavefront, NK: 32-key groups per key sub-tile, BQ / BK: query / key
// block size.
//
// Pass 1 handles a key sub-tile in one of two ways.  Plain order (sub-tiles the mask cuts, the
// sub-tile that sets the softmax reference, the fallback): the K fragments of t are already in
// registers; issue the V fragment loads of t -> S^T = K Q^T, refilling each K fragment's
// registers with sub-tile t+1 as soon as its last MFMA is issued -> running-maximum softmax
// update -> O^T += V^T P^T.  Pipelined order (the unmasked middle of the list): see the comment
// at the loop.  Loads return in issue order, so each wait is a count of younger loads still
// allowed in flight.
// PASS 1: outputs O, lse (and the base-2 normalisers for pass 2).  PASS 2: received mass, a
// separate launch with two wavefronts per SIMD so that one's exponentials overlap the other's MFMAs.
// ARB: the mask C is an explicit bit array (STREAM_MASK_ARRAY): every sub-tile of a block that is
// not wholly visible takes the token-level test against the array, in the plain order; the
// pipelined loop takes the longest run of wholly visible sub-tiles of the list.
// WIDE: block lists of more than 64 entries (up to kMaxTopkWide): the list sits in LDS instead of
// one register (a scalar read of LDS per sub-tile in place of a lane select); the loops are the same.
template <bool BF16, int D, int NQ, int NK, int BQ, int BK, int PASS, int OCC, bool ARB = false, bool WIDE = false>
__global__ void __launch_bounds__(256, OCC) attn_kernel(const AttnParams p)
{
    constexpr int ES = BF16 ? 2 : 4;
    constexpr int FR = D * ES / 32;            // K/Q fragments per 32-token group
    constexpr int NDB = D / 32;                // 32-feature blocks of the output
    constexpr int NVF = BF16 ? 2 : 4;          // V fragments per (group, feature block)
    constexpr int QT = 32 * NQ;                // queries per wavefront
    constexpr int KT = 32 * NK;                // keys per sub-tile
    constexpr int QSUB = BQ / QT;              // wavefronts per row
    constexpr int KSUB = BK / KT;              // key sub-tiles per block
    constexpr long long TILE_BYTES = (long long)BK * D * ES;
    constexpr long long QBLK_BYTES = (long long)BQ * D * ES;   // packed bytes of one query block's span
    constexpr int GROUP_BYTES = 32 * D * ES;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform: keep it scalar
    const int col = lane & 31, gh = lane >> 5;
    // The arguments a wavefront needs before its first tile, fetched together: left to itself the
    // compiler loads each where it is first used and waits for it there - a dozen round trips to
    // the scalar cache one after the other, at the start of every row, with nothing to hide them
    // behind when a SIMD holds one wavefront.  (The empty asm makes them live here.)
    WgMap a_map = p.map;
    int a_NB = p.NB, a_g = p.g, a_kmax = p.kmax, a_nseq = p.seqs.n, a_mask = p.mask, a_window = p.window;
    float a_scale = p.scale_log2e;
    long long a_qsh = p.q_sh_b, a_qst = p.q_st_b;
    const char *a_Q = p.Q, *a_Kp = p.Kp, *a_Vp = p.Vp;
    unsigned long long u_idx = (unsigned long long)p.idx, u_cnt = (unsigned long long)p.cnt;
    asm volatile("" : "+s"(a_map.mode), "+s"(a_map.per_kv), "+s"(a_map.kv_heads), "+s"(a_NB), "+s"(a_g),
                      "+s"(a_kmax), "+s"(a_nseq), "+s"(a_qsh), "+s"(a_qst), "+s"(a_Q), "+s"(a_Kp), "+s"(a_Vp),
                      "+s"(u_idx), "+s"(u_cnt), "+s"(a_mask), "+s"(a_window), "+s"(a_scale));
    // (the two pointers that are dereferenced come back as pointers to global memory: through
    // the asm the compiler no longer knows where they point and would use flat loads, whose
    // completion it can only wait for together with every other load in flight)
    typedef const int __attribute__((address_space(1))) *global_int_ptr;
    const int *a_idx = (const int *)(global_int_ptr)u_idx, *a_cnt = (const int *)(global_int_ptr)u_cnt;
    int kvh, slot;
    if (!wg_decode(a_map, blockIdx.x, kvh, slot)) return;
    const long long items_per_kv = (long long)a_NB * a_g * QSUB;
    const long long it = (long long)slot * 4 + wave;
    if (it >= items_per_kv) return;
    int qs, rk_blk, rk_head;
    if (items_per_kv <= 0x7fffffffLL) {           // (a 64-bit division is ~100 instructions)
        const unsigned rk = (unsigned)it / (unsigned)QSUB;
        qs = (int)((unsigned)it % (unsigned)QSUB);
        rk_blk = (int)(rk / (unsigned)a_g);
        rk_head = (int)(rk - (unsigned)rk_blk * (unsigned)a_g);
    } else {
        const long long rk = it / QSUB;
        qs = (int)(it % QSUB);
        rk_blk = (int)(rk / a_g);
        rk_head = (int)(rk % a_g);
    }
    const int gb = a_NB - 1 - rk_blk;
    const int h = kvh * a_g + rk_head;
    int sq = 0;
    while (sq + 1 < a_nseq && gb >= p.seqs.d[sq + 1].blk0) ++sq;
    const SeqDesc sd = p.seqs.d[sq];
    const int q = gb - sd.blk0, L = sd.len;
    const long long row = (long long)h * a_NB + gb;
    const int qtok0 = q * BQ + qs * QT;         // first query token (sequence-local) of this wavefront
    if (qtok0 >= L) return;
    const int *my_idx = a_idx + row * a_kmax;
    // (the list is fetched for every slot of the row, whatever its count, so that the load does
    // not wait for the count)
    const int my_raw = !WIDE && lane < a_kmax ? my_idx[lane] : 0;
    int n_blk = a_cnt[row];
    n_blk = n_blk < 0 ? 0 : (n_blk > a_kmax ? a_kmax : n_blk);   // never read past the row's list

    // key sub-tiles to visit: all of every listed block, except that under a causal rule the
    // sub-tiles of the diagonal block lying entirely after this wavefront's queries are dropped
    // (lists are ascending, so the diagonal block, if present, is the last one); the count is
    // fixed further down, once the list has been looked at
    int n_tiles = n_blk * KSUB;

    // Q fragments (usable as A or B operand): lane (col, gh), fragment fr -> chunk 2*fr+gh of row col
    // (through a resource that starts at the wavefront's first query and spans its real rows:
    // rows past the end of the sequence read as zeros, no branch around any load)
    uint4 qf[NQ][FR];
    {
        const int qrows = L - qtok0 < QT ? L - qtok0 : QT;
        const __amdgpu_buffer_rsrc_t qrs = make_tile_rsrc(
            a_Q + (long long)h * a_qsh + (sd.tok0 + qtok0) * a_qst, (unsigned)((long long)(qrows - 1) * a_qst + D * ES));
#pragma unroll
        for (int cq = 0; cq < NQ; ++cq) {
            const unsigned voff = (unsigned)(cq * 32 + col) * (unsigned)a_qst + gh * 16;
#pragma unroll
            for (int fr = 0; fr < FR; ++fr) {
                const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(qrs, voff + fr * 32, 0, 0);
                qf[cq][fr] = make_uint4(v[0], v[1], v[2], v[3]);
            }
        }
    }
    // packed K and V tiles of this (kv head, sequence)
    const unsigned region_bytes = (unsigned)((long long)sd.nblk * QBLK_BYTES);
    const __amdgpu_buffer_rsrc_t krs =
        make_tile_rsrc(a_Kp + ((long long)kvh * a_NB + sd.blk0) * QBLK_BYTES, region_bytes);
    const __amdgpu_buffer_rsrc_t vrs =
        make_tile_rsrc(a_Vp + ((long long)kvh * a_NB + sd.blk0) * QBLK_BYTES, region_bytes);
    const unsigned lane_off = lane * 16;
    // the row's block list lives in one register (lane j holds entry j; lists have <= 64 entries)
    // and is read with a scalar lane select: no memory access inside the tile loops
    const int my_blk = lane < n_blk ? my_raw : 0;
    __shared__ int s_blk[WIDE ? 4 : 1][WIDE ? kMaxTopkWide : 1];
    // pass 1: staging of the output tile, 32 query rows of at most 256 bytes at a time (the pad
    // of 16 bytes per row spreads the rows over the banks)
    constexpr int O_NDBU = NDB < 256 / (32 * ES) ? NDB : 256 / (32 * ES);   // feature blocks per staged unit
    constexpr int O_URB = O_NDBU * 32 * ES, O_URS = O_URB + 16;
    __shared__ __align__(16) char s_o[PASS == 1 ? 4 * 32 * O_URS : 16];
    // ARB: "every pair of this query block and that key block is real and set in C", per key block
    const unsigned *allrow = ARB ? p.call + (long long)gb * p.cw : nullptr;
    auto all_bit = [&](int r) -> bool {          // (an entry outside the block range reads as "cut")
        return (unsigned)r < (unsigned)p.cw * 32u && ((allrow[r >> 5] >> (r & 31)) & 1u);
    };
    // The loops below assume what stream_prune writes: strictly ascending ids of key blocks of the
    // sequence.  A list that is anything else (not ascending, a repeated id, an id outside the
    // sequence) is still handled safely: `plain_list` sends every sub-tile through the plain order
    // with the token-level mask (so no key after a query, and no key outside the sequence, ever
    // counts), and the trimming of the last block is skipped.
    const int nkb = (int)((long long)sd.nblk * BQ / BK);          // key blocks of the sequence
    bool entry_bad = false;
    if constexpr (WIDE) {
        for (int i = lane; i < n_blk; i += 64) {
            int v = my_idx[i];
            const int before = i > 0 ? my_idx[i - 1] : -1;
            entry_bad = entry_bad | ((unsigned)v >= (unsigned)nkb) | (v <= before);
            // (with a mask array the top bit of an entry says that C cuts through the block)
            if constexpr (ARB) v |= all_bit(v) ? 0 : (int)0x80000000;
            s_blk[wave][i] = v;
        }
        wave_sync();
    } else {
        const int before = __shfl_up(my_blk, 1);
        entry_bad = (lane < n_blk) & (((unsigned)my_blk >= (unsigned)nkb) | ((lane > 0) & (my_blk <= before)));
    }
    const bool plain_list = __ballot(entry_bad) != 0ull;          // wave-uniform
    if (!ARB && !plain_list && n_blk > 0 && a_mask != STREAM_MASK_FULL) {
        const int last_r = WIDE ? my_idx[n_blk - 1] : __builtin_amdgcn_readlane(my_blk, n_blk - 1);
        if (last_r * BK + (KSUB - 1) * KT > qtok0 + QT - 1) {
            int vis = (qtok0 + QT - 1 - last_r * BK) / KT + 1;
            vis = vis < 0 ? 0 : (vis > KSUB ? KSUB : vis);
            n_tiles = (n_blk - 1) * KSUB + vis;
        }
    }
    n_tiles = __builtin_amdgcn_readfirstlane(n_tiles);
    auto list_entry = [&](int i) -> int {        // i is wave-uniform
        if constexpr (WIDE)
            return __builtin_amdgcn_readfirstlane(s_blk[wave][i]) & 0x7fffffff;
        else
            return __builtin_amdgcn_readlane(my_blk, i);
    };
    auto tile_off = [&](int t) -> unsigned {
        const int ts = __builtin_amdgcn_readfirstlane(t);
        const int r = list_entry(ts / KSUB);
        return (unsigned)r * (unsigned)TILE_BYTES + (unsigned)(ts % KSUB) * NK * GROUP_BYTES;
    };
    auto tile_ktok0 = [&](int t) -> int {
        const int ts = __builtin_amdgcn_readfirstlane(t);
        const int r = list_entry(ts / KSUB);
        return r * BK + (ts % KSUB) * KT;
    };
    // does the mask C (or the end of the sequence) cut through the sub-tile that starts at key k0?
    auto needs_mask = [&](int k0) -> bool {
        bool m = k0 + KT > L;
        if (a_mask != STREAM_MASK_FULL) m = m || (k0 + KT - 1 > qtok0);                       // keys after a query
        if (a_mask == STREAM_MASK_SLIDING) m = m || (k0 <= qtok0 + QT - 1 - a_window);         // keys before a window
        return m;
    };
    // ARB: bit j = list entry j is wholly visible to this query block (every pair real and set in
    // C); one lane per entry looks it up once, the loops then test a scalar bit per sub-tile
    unsigned long long allmask = 0;
    if constexpr (ARB && !WIDE)
        allmask = __ballot(lane < n_blk && all_bit(my_blk));
    auto tile_masked = [&](int t) -> bool {      // t is wave-uniform
        if (plain_list) return true;
        if constexpr (ARB && WIDE)
            return __builtin_amdgcn_readfirstlane(s_blk[wave][__builtin_amdgcn_readfirstlane(t) / KSUB]) < 0;
        else if constexpr (ARB)
            return !((allmask >> (__builtin_amdgcn_readfirstlane(t) / KSUB)) & 1ull);
        else
            return needs_mask(tile_ktok0(t));
    };

    if constexpr (PASS == 1) {
    floatx16 acc_o[NDB][NQ];
    float m_run[NQ], l_run[NQ];
    // bf16: the PV product uses the probabilities rounded to bf16, so O is normalised by the sum
    // of those same rounded values (lr_run): a row dominated by one key then gets that key's V
    // exactly, whatever the rounding of its probability.  lse uses the unrounded sum (l_run).
    float lr_run[NQ];
    const float c2 = a_scale;
    // (fp32 at d = 128 does not fit the double buffers in the register file: plain loop only)
    constexpr bool PIPE = NK == 1 && (BF16 || D == 64);
    // The pipelined loop reads the Q fragments from the accumulation registers (an MFMA takes
    // its B operand from either file), which leaves the vector registers to the scores.
    u32x4_t qacc[NQ][FR];
    if constexpr (PIPE && BF16) {
#pragma unroll
        for (int cq = 0; cq < NQ; ++cq)
#pragma unroll
            for (int fr = 0; fr < FR; ++fr) {
                u32x4_t v = {qf[cq][fr].x, qf[cq][fr].y, qf[cq][fr].z, qf[cq][fr].w};
                asm volatile("" : "+a"(v));
                qacc[cq][fr] = v;
                qf[cq][fr] = make_uint4(v[0], v[1], v[2], v[3]);
            }
    }

    uint4 kreg[NK][FR];
    // ------------------------------------------------------------------ pass 1: O and lse
    // Leading sub-tiles that need no mask run in a software pipeline that keeps the matrix
    // pipe busy while the vector ALUs do the softmax: iteration t issues, as one interleaved
    // stream,  O^T += V(t-1)^T P(t-1)^T  and  S(t+1)^T = K(t+1) Q^T  (MFMA groups), the loads
    // that refill each V / K fragment right after its last use, and between the MFMA groups
    // the exponentials and conversions of S(t) cut into small chunks.  S is double buffered by parity.
    // Iteration 0 multiplies a zero P, the last one computes an S nobody reads: one loop body
    // serves all iterations.  Sub-tiles the mask cuts (diagonal block, sequence tail, edge of a
    // sliding window) go through the plain order, before and after.
    // Lists are ascending, so the sub-tiles the mask cuts are a prefix (keys before the window
    // of a sliding mask) and a suffix (diagonal block, end of the sequence): [tb, t_end) is the
    // unmasked middle, n_fast its length.
    int tb = 0, t_end = 0;
    if constexpr (PIPE) {
        t_end = n_tiles;
        while (t_end > 0 && tile_masked(t_end - 1)) --t_end;
        if (a_mask == STREAM_MASK_SLIDING)
            while (tb < t_end && tile_masked(tb)) ++tb;
        if constexpr (ARB) {
            // an array can cut any entry of the list: the pipeline takes the longest run of
            // wholly visible sub-tiles (after the first sub-tile), the plain order the rest
            int run_b = -1;
            tb = t_end = n_tiles;
            for (int t = 1; t <= n_tiles; ++t) {
                const bool m = t == n_tiles || tile_masked(t);
                if (!m && run_b < 0) run_b = t;
                if (m && run_b >= 0) {
                    if (t - run_b > t_end - tb) { tb = run_b; t_end = t; }
                    run_b = -1;
                }
            }
        }
        // the pipelined loop keeps the softmax reference fixed (see below): the sub-tile before
        // it always goes through the plain order, which sets the reference
        tb = tb < 1 ? 1 : tb;
        tb = __builtin_amdgcn_readfirstlane(tb < n_tiles ? tb : n_tiles);
        t_end = __builtin_amdgcn_readfirstlane(t_end > tb ? t_end : tb);
    }
    const int n_fast = t_end - tb;

    // One sub-tile in the plain order: loads, S, mask, softmax update, PV.
    auto serial_tile = [&](const int t) {
        const unsigned off = tile_off(t);
        const int ktok0 = tile_ktok0(t);
        const unsigned knext = tile_off(t + 1 < n_tiles ? t + 1 : t);
        uint4 vreg[NK][NDB * NVF];
#pragma unroll
        for (int rb = 0; rb < NK; ++rb)
#pragma unroll
            for (int j = 0; j < NDB * NVF; ++j)
                vreg[rb][j] = load_frag(vrs, lane_off, off, rb * NDB * NVF + j);
        __builtin_amdgcn_sched_barrier(0);

        floatx16 acc_s[NK][NQ];
#pragma unroll
        for (int rb = 0; rb < NK; ++rb)
#pragma unroll
            for (int cq = 0; cq < NQ; ++cq)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc_s[rb][cq][i] = 0.f;
#pragma unroll
        for (int fr = 0; fr < FR; ++fr)
#pragma unroll
            for (int rb = 0; rb < NK; ++rb) {
#pragma unroll
                for (int cq = 0; cq < NQ; ++cq)
                    acc_s[rb][cq] = mfma16<BF16>(kreg[rb][fr], qf[cq][fr], acc_s[rb][cq]);
                __builtin_amdgcn_sched_barrier(0);
                kreg[rb][fr] = load_frag(krs, lane_off, knext, rb * FR + fr);
                __builtin_amdgcn_sched_barrier(0);
            }
        // mask (raw scores): the rule C inside the tile, padded keys
        if (tile_masked(t)) {
#pragma unroll
            for (int rb = 0; rb < NK; ++rb)
#pragma unroll
                for (int cq = 0; cq < NQ; ++cq)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int tk = ktok0 + rb * 32 + (i >> 2) * 8 + gh * 4 + (i & 3);
                        const int tq = qtok0 + cq * 32 + col;
                        // (a select, not a conditional store: `if (!visible) acc_s[..][i] = -inf` on a
                        // vector element was dropped by this compiler inside the lambda)
                        bool visible = (unsigned)tk < (unsigned)L;
                        if constexpr (ARB) {
                            // the word of this lane's query row that holds keys ktok0 + rb*32 .. +31
                            // (a word wholly past the end of the row is not read)
                            const unsigned cwd = ((tq < L) & ((unsigned)(ktok0 + rb * 32) < (unsigned)L)) ? p.cbits[(long long)tq * p.cpitch + ((ktok0 >> 5) + rb)] : 0u;
                            visible = visible & ((cwd >> ((i >> 2) * 8 + gh * 4 + (i & 3))) & 1u);
                        } else {
                            visible = visible & mask_token(a_mask, a_window, tq, tk);
                        }
                        acc_s[rb][cq][i] = visible ? acc_s[rb][cq][i] : -INFINITY;
                    }
        }
        // running softmax per query column, in base 2: logit = raw * c2
        float alpha[NQ];
        bool grew = false;
#pragma unroll
        for (int cq = 0; cq < NQ; ++cq) {
            float mx = -INFINITY;
#pragma unroll
            for (int rb = 0; rb < NK; ++rb)
#pragma unroll
                for (int i = 0; i < 16; ++i) mx = fmaxf(mx, acc_s[rb][cq][i]);
            mx = fmaxf(mx, __shfl_xor(mx, 32)) * c2;
            // the reference exponent follows the running maximum lazily: it moves only when the
            // maximum has grown by more than 2^8, so probabilities stay <= 256 (harmless in fp32
            // and bf16) and the output accumulators are rescaled a handful of times per row
            const float m_new = mx > m_run[cq] + 8.f ? mx : m_run[cq];
            const float m_use = m_new == -INFINITY ? 0.f : m_new;
            grew = grew || (m_new > m_run[cq] && m_run[cq] != -INFINITY);
            alpha[cq] = __builtin_amdgcn_exp2f(m_run[cq] - m_use);
            m_run[cq] = m_new;
            float sum = 0.f;
#pragma unroll
            for (int rb = 0; rb < NK; ++rb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const float pr = __builtin_amdgcn_exp2f(fmaf(acc_s[rb][cq][i], c2, -m_use));
                    acc_s[rb][cq][i] = pr;
                    sum += pr;
                }
            l_run[cq] = l_run[cq] * alpha[cq] + sum;   // per-lane partial; halves are added at the end
            if constexpr (BF16) lr_run[cq] *= alpha[cq];
        }
        // rescale the output accumulators only when some column's maximum moved
        if (__any(grew)) {
#pragma unroll
            for (int cq = 0; cq < NQ; ++cq)
#pragma unroll
                for (int db = 0; db < NDB; ++db)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        // The accumulators live in the accumulation registers, where the MFMAs
                        // update them; scale them there (read, multiply, write back) so that this
                        // rare path does not drag all 128 of them through the vector registers
                        // on every iteration.
                        float t = acc_o[db][cq][i], tmp;
                        asm volatile("v_accvgpr_read_b32 %1, %0\n\t"
                                     "v_mul_f32 %1, %1, %2\n\t"
                                     "v_accvgpr_write_b32 %0, %1"
                                     : "+a"(t), "=&v"(tmp)
                                     : "v"(alpha[cq]));
                        acc_o[db][cq][i] = t;
                    }
            asm volatile("s_nop 7");
        }
        // O^T += V^T P^T
#pragma unroll
        for (int rb = 0; rb < NK; ++rb)
#pragma unroll
            for (int vf = 0; vf < NVF; ++vf) {
                uint4 pf[NQ];
#pragma unroll
                for (int cq = 0; cq < NQ; ++cq) {
                    if constexpr (BF16) {
                        const int o = vf * 8;
                        pf[cq] = to_bf16_frag(acc_s[rb][cq][o + 0], acc_s[rb][cq][o + 1],
                                              acc_s[rb][cq][o + 2], acc_s[rb][cq][o + 3],
                                              acc_s[rb][cq][o + 4], acc_s[rb][cq][o + 5],
                                              acc_s[rb][cq][o + 6], acc_s[rb][cq][o + 7]);
                        lr_run[cq] = dot2_ones(pf[cq].w, dot2_ones(pf[cq].z, dot2_ones(pf[cq].y, dot2_ones(pf[cq].x, lr_run[cq]))));
                    } else {
                        const int o = vf * 4;
                        pf[cq].x = f2u(acc_s[rb][cq][o + 0]);
                        pf[cq].y = f2u(acc_s[rb][cq][o + 1]);
                        pf[cq].z = f2u(acc_s[rb][cq][o + 2]);
                        pf[cq].w = f2u(acc_s[rb][cq][o + 3]);
                    }
                }
#pragma unroll
                for (int db = 0; db < NDB; ++db)
#pragma unroll
                    for (int cq = 0; cq < NQ; ++cq)
                        acc_o[db][cq] = mfma16<BF16>(vreg[rb][db * NVF + vf], pf[cq], acc_o[db][cq]);
            }
    };
    // The pipelined loop does not follow the running maximum: it keeps the reference exponent
    // the plain order has set so far (probabilities are then 2^(s - m_ref), any magnitude fp32
    // and bf16 represent; the final normalisation makes the choice of reference immaterial).
    // That saves the maximum, the reference update and the accumulator rescale of every
    // pipelined sub-tile.  It cannot be wrong silently: a probability beyond 2^127 or a row sum
    // that vanished shows as a non-finite or zero normaliser / output, and then the row is
    // computed again entirely in the plain order (`safe`), which tracks the maximum.
    float lse2[NQ];   // log2-domain log-sum-exp of each query column
    float inv[NQ];
    bool safe = !PIPE;
    for (;;) {
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int cq = 0; cq < NQ; ++cq)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc_o[db][cq][i] = 0.f;
#pragma unroll
    for (int cq = 0; cq < NQ; ++cq) { m_run[cq] = -INFINITY; l_run[cq] = 0.f; lr_run[cq] = 0.f; }
    if (n_tiles > 0) {
        const unsigned off0 = tile_off(0);
        // same order as the refills inside the loops: waits count loads in issue order
#pragma unroll
        for (int fr = 0; fr < FR; ++fr)
#pragma unroll
            for (int rb = 0; rb < NK; ++rb) {
                kreg[rb][fr] = load_frag(krs, lane_off, off0, rb * FR + fr);
                __builtin_amdgcn_sched_barrier(0);
            }
    }
    const int t_plain = safe ? n_tiles : tb;      // plain order up to here ...
    const int t_resume = safe ? n_tiles : t_end;  // ... and again from here
    for (int t = 0; t < t_plain; ++t) serial_tile(t);

    if constexpr (PIPE) {
    if (!safe && n_fast > 0) {
        constexpr int GPV = NVF * NDB;          // MFMA groups of the PV product
        constexpr int G = GPV + FR;             // + groups of the QK product
        constexpr int C = 5 * NQ;               // softmax chunks: per column 4 x four exponentials, 1 convert
        // P has one buffer: the first chunk that writes P (index 4) must not run before the
        // MFMAs of the last PV group (chunks of group g follow the group's MFMAs)
        static_assert((GPV - 1) * C / G <= 4, "P would be overwritten while PV still reads it");
        float m_fix[NQ];                        // the reference exponent, fixed for the loop
#pragma unroll
        for (int cq = 0; cq < NQ; ++cq) {
            // a column that has seen no key yet takes 0: from here on that is its reference, also
            // for the plain order that follows (sums and accumulators are relative to m_run)
            m_fix[cq] = m_run[cq] == -INFINITY ? 0.f : m_run[cq];
            m_run[cq] = m_fix[cq];
        }
        floatx16 S[2][NQ];
        uint4 Pf[NVF][NQ];
        // V and K fragments are double buffered by parity as well: what iteration t loads is
        // consumed by iteration t + 2, so a load has two iterations to arrive.
        //   iteration t (parity sb): vr[sb] holds V(t-1), refilled with V(t+1);
        //                            kb(sb) holds K(t+1), refilled with K(t+3).
        uint4 vr[2][GPV];
        uint4 k1r[FR];                          // parity 1 of the K buffer; parity 0 is kreg[0]
        // the pipeline counts its sub-tiles from 0; list position = tb + that
        auto clampk = [&](int x) {              // K tile to prefetch: never past the first masked tile
            x = tb + (x < n_fast ? x : n_fast);
            return x < n_tiles ? x : n_tiles - 1;
        };
#pragma unroll
        for (int vf = 0; vf < NVF; ++vf)
#pragma unroll
            for (int cq = 0; cq < NQ; ++cq) Pf[vf][cq] = make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int j = 0; j < GPV; ++j) vr[0][j] = make_uint4(0, 0, 0, 0);   // iteration 0: 0 x 0
        {   // S(0), then the fragments of iterations 0 and 1 in the order they are consumed
            const unsigned k1 = tile_off(clampk(1));
#pragma unroll
            for (int fr = 0; fr < FR; ++fr) {
#pragma unroll
                for (int cq = 0; cq < NQ; ++cq) {
                    if constexpr (BF16) {
                        qk_mfma_bf16(S[0][cq], kreg[0][fr], qacc[cq][fr], fr == 0);
                    } else {
                        floatx16 z;
#pragma unroll
                        for (int i = 0; i < 16; ++i) z[i] = 0.f;
                        S[0][cq] = mfma16<BF16>(kreg[0][fr], qf[cq][fr], fr == 0 ? z : S[0][cq]);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
                kreg[0][fr] = load_frag(krs, lane_off, k1, fr);
                __builtin_amdgcn_sched_barrier(0);
            }
            const unsigned off0 = tile_off(tb);
#pragma unroll
            for (int g = 0; g < GPV; ++g) {
                const int vf = g / NDB, db = g % NDB;
                vr[1][db * NVF + vf] = load_frag(vrs, lane_off, off0, db * NVF + vf);
                __builtin_amdgcn_sched_barrier(0);
            }
            const unsigned k2 = tile_off(clampk(2));
#pragma unroll
            for (int fr = 0; fr < FR; ++fr) {
                k1r[fr] = load_frag(krs, lane_off, k2, fr);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        auto iter = [&](const int t, auto SBc) {
            constexpr int sb = decltype(SBc)::value, ob = sb ^ 1;
            const unsigned voff = tile_off(tb + (t + 1 < n_fast ? t + 1 : n_fast - 1));
            const unsigned knext = tile_off(clampk(t + 3));
            float sv[NQ][16], sum[NQ];
            auto chunk = [&](auto Cc) {
                constexpr int c = decltype(Cc)::value;
                {
                    constexpr int cq = c / 5, part = c % 5;
                    if constexpr (part == 0) sum[cq] = 0.f;
                    if constexpr (part < 4) {
#pragma unroll
                        for (int i = part * 4; i < part * 4 + 4; ++i) {
                            sv[cq][i] = __builtin_amdgcn_exp2f(fmaf(S[sb][cq][i], c2, -m_fix[cq]));
                            sum[cq] += sv[cq][i];
                            // keeps the chunk where it is written (in the shadow of this
                            // group's MFMAs): its results are first used much later
                            asm volatile("" : "+v"(sv[cq][i]));
                        }
                        asm volatile("" : "+v"(sum[cq]));
                    } else {
#pragma unroll
                        for (int vf = 0; vf < NVF; ++vf) {
                            if constexpr (BF16) {
                                const int o = vf * 8;
                                Pf[vf][cq] = to_bf16_frag(sv[cq][o + 0], sv[cq][o + 1], sv[cq][o + 2],
                                                              sv[cq][o + 3], sv[cq][o + 4], sv[cq][o + 5],
                                                              sv[cq][o + 6], sv[cq][o + 7]);
                            } else {
                                const int o = vf * 4;
                                Pf[vf][cq] = make_uint4(f2u(sv[cq][o + 0]), f2u(sv[cq][o + 1]),
                                                            f2u(sv[cq][o + 2]), f2u(sv[cq][o + 3]));
                            }
                            asm volatile("" : "+v"(Pf[vf][cq].x), "+v"(Pf[vf][cq].y),
                                             "+v"(Pf[vf][cq].z), "+v"(Pf[vf][cq].w));
                            if constexpr (BF16)
                                lr_run[cq] = dot2_ones(Pf[vf][cq].w, dot2_ones(Pf[vf][cq].z,
                                             dot2_ones(Pf[vf][cq].y, dot2_ones(Pf[vf][cq].x, lr_run[cq]))));
                        }
                        l_run[cq] += sum[cq];
                        asm volatile("" : "+v"(l_run[cq]));
                        if constexpr (BF16) asm volatile("" : "+v"(lr_run[cq]));
                    }
                }
            };
            auto group = [&](auto Gc) {
                constexpr int g = decltype(Gc)::value;
                if constexpr (g < GPV) {
                    constexpr int vf = g / NDB, db = g % NDB;
#pragma unroll
                    for (int cq = 0; cq < NQ; ++cq)
                        acc_o[db][cq] = mfma16<BF16>(vr[sb][db * NVF + vf], Pf[vf][cq], acc_o[db][cq]);
                    __builtin_amdgcn_sched_barrier(0);
                    vr[sb][db * NVF + vf] = load_frag(vrs, lane_off, voff, db * NVF + vf);
                } else {
                    constexpr int fr = g - GPV;
                    uint4 &kb = sb == 0 ? kreg[0][fr] : k1r[fr];
#pragma unroll
                    for (int cq = 0; cq < NQ; ++cq) {
                        if constexpr (BF16) {
                            qk_mfma_bf16(S[ob][cq], kb, qacc[cq][fr], fr == 0);
                        } else {
                            floatx16 z;
#pragma unroll
                            for (int i = 0; i < 16; ++i) z[i] = 0.f;
                            S[ob][cq] = mfma16<BF16>(kb, qf[cq][fr], fr == 0 ? z : S[ob][cq]);
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    kb = load_frag(krs, lane_off, knext, fr);
                }
                __builtin_amdgcn_sched_barrier(0);
                // this group's share of the softmax chunks
                constexpr int c0 = g * C / G, c1 = (g + 1) * C / G;
                auto run = [&](auto Ic) { chunk(IntC<c0 + decltype(Ic)::value>{}); };
                static_for<0, c1 - c0>(run);
                __builtin_amdgcn_sched_barrier(0);
            };
            static_for<0, G>(group);
        };
        auto drain = [&](auto SBc) {   // O^T += V(n_fast-1)^T P(n_fast-1)^T
            constexpr int sb = decltype(SBc)::value;
#pragma unroll
            for (int vf = 0; vf < NVF; ++vf)
#pragma unroll
                for (int db = 0; db < NDB; ++db)
#pragma unroll
                    for (int cq = 0; cq < NQ; ++cq)
                        acc_o[db][cq] = mfma16<BF16>(vr[sb][db * NVF + vf], Pf[vf][cq], acc_o[db][cq]);
        };
        int t = 0;
        for (; t + 1 < n_fast; t += 2) {
            iter(t, IntC<0>{});
            iter(t + 1, IntC<1>{});
        }
        // V(n_fast - 1) sits in the buffer of parity n_fast & 1; both K buffers hold K(n_fast)
        if (t < n_fast) {
            iter(t, IntC<0>{});
            drain(IntC<1>{});
        } else {
            drain(IntC<0>{});
        }
    }
    }
    for (int t = t_resume; t < n_tiles; ++t) serial_tile(t);

    // normalisers; in the first attempt also the check that nothing overflowed or vanished
    bool bad = false;
#pragma unroll
    for (int cq = 0; cq < NQ; ++cq) {
        const float l_tot = l_run[cq] + __shfl_xor(l_run[cq], 32);
        const float lr_tot = BF16 ? lr_run[cq] + __shfl_xor(lr_run[cq], 32) : l_tot;
        inv[cq] = lr_tot > 0.f ? 1.f / lr_tot : 0.f;
        lse2[cq] = l_tot > 0.f ? m_run[cq] + log2f(l_tot) : -INFINITY;
        if (!safe) {
            bad = bad | !(l_tot > 1e-30f) | !(l_tot < 3e38f) | !(lr_tot > 1e-30f) | !(lr_tot < 3e38f);
            // (0 * x summed over the accumulators is NaN as soon as one of them is not finite)
            float chk = 0.f;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int i = 0; i < 16; ++i) chk = fmaf(acc_o[db][cq][i], 0.f, chk);
            bad = bad | !(chk == 0.f);
        }
    }
    if (safe || !__any(bad)) break;
    safe = true;
    }

    // ------------------------------------------------------------------ store O, lse
    // O^T accumulator: lane holds query `col`; element i of block db is feature
    // db*32 + 8*(i/4) + 4*gh + (i%4): four consecutive features per group of 4.  Written from
    // here a store instruction would touch 32 rows with 8 or 16 bytes each; the normalised tile
    // goes through LDS instead, 32 rows at a time, and leaves as whole rows (16 bytes per lane).
    {
        char *so = s_o + wave * 32 * O_URS;
        constexpr int LPR = O_URB / 16, RPI = 64 / LPR;        // lanes per staged row, rows per store
#pragma unroll
        for (int cq = 0; cq < NQ; ++cq)
#pragma unroll
            for (int u = 0; u < NDB / O_NDBU; ++u) {
#pragma unroll
                for (int dbu = 0; dbu < O_NDBU; ++dbu)
#pragma unroll
                    for (int i4 = 0; i4 < 4; ++i4) {
                        const int db = u * O_NDBU + dbu;
                        const int feat = dbu * 32 + i4 * 8 + gh * 4;      // within the unit
                        const float a = acc_o[db][cq][i4 * 4 + 0] * inv[cq], b = acc_o[db][cq][i4 * 4 + 1] * inv[cq];
                        const float c = acc_o[db][cq][i4 * 4 + 2] * inv[cq], d = acc_o[db][cq][i4 * 4 + 3] * inv[cq];
                        if constexpr (BF16) {
                            uint2 v;
                            v.x = pack_bf16x2(a, b);
                            v.y = pack_bf16x2(c, d);
                            *reinterpret_cast<uint2 *>(so + col * O_URS + feat * 2) = v;
                        } else {
                            *reinterpret_cast<float4 *>(so + col * O_URS + feat * 4) = make_float4(a, b, c, d);
                        }
                    }
                // (LDS serves a wavefront's instructions in order: the reads below see these writes,
                // and the next unit's writes come after these reads; the barrier only keeps the
                // compiler from moving them across each other)
                __builtin_amdgcn_wave_barrier();
                // (all reads of the unit first, then its stores: one LDS latency per unit, not per store)
                uint4 ov[32 / RPI];
#pragma unroll
                for (int j = 0; j < 32 / RPI; ++j)
                    ov[j] = *reinterpret_cast<const uint4 *>(so + (j * RPI + lane / LPR) * O_URS + (lane % LPR) * 16);
#pragma unroll
                for (int j = 0; j < 32 / RPI; ++j) {
                    const int r = j * RPI + lane / LPR, ch = lane % LPR;
                    const int tok = qtok0 + cq * 32 + r;
                    if (tok < L)
                        *reinterpret_cast<uint4 *>(p.O + (long long)h * p.o_sh_b + (sd.tok0 + tok) * p.o_st_b +
                                                   u * O_URB + ch * 16) = ov[j];
                }
                __builtin_amdgcn_wave_barrier();
            }
    }
#pragma unroll
    for (int cq = 0; cq < NQ; ++cq) {
        const int tok = qtok0 + cq * 32 + col;
        if (tok < L && gh == 0) {
            if (p.lse) p.lse[(long long)h * p.T + sd.tok0 + tok] = lse2[cq] * 0.6931471805599453f;
            if (p.lse2) p.lse2[(long long)h * p.T + sd.tok0 + tok] = lse2[cq];
        }
    }
    } else {
    uint4 kreg[NK][FR];
    const float c2 = a_scale;
    // ------------------------------------------------------------------ pass 2: received mass
    // S = Q K^T: a lane owns key column `col`; element i of row block rq is query
    // rq*32 + 8*(i/4) + 4*gh + (i%4).  Its normaliser:
    // (through a resource over the wavefront's real queries: rows past the end of the sequence
    // read as zeros, and no load sits behind a branch)
    float lq[NQ][16];
    {
        const int qrows = L - qtok0 < QT ? L - qtok0 : QT;
        const __amdgpu_buffer_rsrc_t lrs =
            make_tile_rsrc(p.lse2 + (long long)h * p.T + sd.tok0 + qtok0, (unsigned)qrows * 4u);
#pragma unroll
        for (int rq = 0; rq < NQ; ++rq)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const unsigned voff = (unsigned)(rq * 32 + (i >> 2) * 8 + gh * 4 + (i & 3)) * 4u;
                lq[rq][i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(lrs, voff, 0, 0));
            }
    }
    float *mass_h = p.mass + (long long)h * p.T + sd.tok0;
    if (n_tiles > 0) {
        const unsigned off0 = tile_off(0);
        // same order as the refills inside the loop: waits count loads in issue order
#pragma unroll
        for (int fr = 0; fr < FR; ++fr)
#pragma unroll
            for (int rb = 0; rb < NK; ++rb) {
                kreg[rb][fr] = load_frag(krs, lane_off, off0, rb * FR + fr);
                __builtin_amdgcn_sched_barrier(0);
            }
    }
    for (int t = 0; t < n_tiles; ++t) {
        const int ktok0 = tile_ktok0(t);
        const unsigned knext = tile_off(t + 1 < n_tiles ? t + 1 : t);
        floatx16 acc_s[NQ][NK];
#pragma unroll
        for (int rq = 0; rq < NQ; ++rq)
#pragma unroll
            for (int ck = 0; ck < NK; ++ck)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc_s[rq][ck][i] = 0.f;
#pragma unroll
        for (int fr = 0; fr < FR; ++fr)
#pragma unroll
            for (int ck = 0; ck < NK; ++ck) {
#pragma unroll
                for (int rq = 0; rq < NQ; ++rq)
                    acc_s[rq][ck] = mfma16<BF16>(qf[rq][fr], kreg[ck][fr], acc_s[rq][ck]);
                __builtin_amdgcn_sched_barrier(0);
                kreg[ck][fr] = load_frag(krs, lane_off, knext, ck * FR + fr);
                __builtin_amdgcn_sched_barrier(0);
            }
        const bool need_mask = tile_masked(t) || (qtok0 + QT > L);
#pragma unroll
        for (int ck = 0; ck < NK; ++ck) {
            const int tk = ktok0 + ck * 32 + col;
            float colsum = 0.f;
            if (!need_mask) {   // wave-uniform: most sub-tiles are fully visible
#pragma unroll
                for (int rq = 0; rq < NQ; ++rq)
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        colsum += __builtin_amdgcn_exp2f(fmaf(acc_s[rq][ck][i], c2, -lq[rq][i]));
            } else {
                // (the empty asm keeps this a real branch: merged into the path above, the mask
                // arithmetic would run on every sub-tile)
                asm volatile("" ::: "memory");
                // ARB: lane j fetches the mask word of query row j for this 32-key group; an
                // element takes its row's word from the lane that fetched it
                unsigned rowword = 0u;
                if constexpr (ARB) {
                    const int tqr = qtok0 + lane;
                    if (lane < QT && tqr < L && (unsigned)(ktok0 + ck * 32) < (unsigned)L)     // (no read of a word wholly past the end of the row)
                        rowword = p.cbits[(long long)tqr * p.cpitch + ((ktok0 >> 5) + ck)];
                }
#pragma unroll
                for (int rq = 0; rq < NQ; ++rq)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int tq = qtok0 + rq * 32 + (i >> 2) * 8 + gh * 4 + (i & 3);
                        const float e = __builtin_amdgcn_exp2f(fmaf(acc_s[rq][ck][i], c2, -lq[rq][i]));
                        bool visible = tq < L;
                        if constexpr (ARB) {
                            const unsigned cwd = (unsigned)__shfl((int)rowword, rq * 32 + (i >> 2) * 8 + gh * 4 + (i & 3));
                            visible = visible & ((cwd >> col) & 1u);
                        } else {
                            visible = visible & mask_token(a_mask, a_window, tq, tk);
                        }
                        colsum += visible ? e : 0.f;
                    }
            }
            colsum += __shfl_xor(colsum, 32);
            if (gh == 0 && (unsigned)tk < (unsigned)L && colsum != 0.f) atomicAdd(mass_h + tk, colsum);
        }
    }
    }
}

typedef void (*attn_fn)(const AttnParams);

// 64 queries per wavefront (32 for query block 32) against 32-key sub-tiles: with one 32-key
// group in flight the scores, the K/V fragments and the Q tile fit the 256 architectural VGPRs
// and the output accumulators live in the accumulation registers.
template <int PASS, int OCC, bool BF16, int D, int NQ, int BQ>
static attn_fn pick_attn_kernel_bk(int bk, bool arb, bool wide)
{
    if (wide && arb) {
        if (bk == 32) return attn_kernel<BF16, D, NQ, 1, BQ, 32, PASS, OCC, true, true>;
        if (bk == 64) return attn_kernel<BF16, D, NQ, 1, BQ, 64, PASS, OCC, true, true>;
        return attn_kernel<BF16, D, NQ, 1, BQ, 128, PASS, OCC, true, true>;
    }
    if (wide) {
        if (bk == 32) return attn_kernel<BF16, D, NQ, 1, BQ, 32, PASS, OCC, false, true>;
        if (bk == 64) return attn_kernel<BF16, D, NQ, 1, BQ, 64, PASS, OCC, false, true>;
        return attn_kernel<BF16, D, NQ, 1, BQ, 128, PASS, OCC, false, true>;
    }
    if (arb) {
        if (bk == 32) return attn_kernel<BF16, D, NQ, 1, BQ, 32, PASS, OCC, true>;
        if (bk == 64) return attn_kernel<BF16, D, NQ, 1, BQ, 64, PASS, OCC, true>;
        return attn_kernel<BF16, D, NQ, 1, BQ, 128, PASS, OCC, true>;
    }
    if (bk == 32) return attn_kernel<BF16, D, NQ, 1, BQ, 32, PASS, OCC>;
    if (bk == 64) return attn_kernel<BF16, D, NQ, 1, BQ, 64, PASS, OCC>;
    return attn_kernel<BF16, D, NQ, 1, BQ, 128, PASS, OCC>;
}

template <int PASS, int OCC, bool BF16, int D>
static attn_fn pick_attn_kernel_d(int bq, int bk, bool arb, bool wide)
{
    constexpr int OCC2 = (BF16 || D == 64) ? OCC : 1;
    if (bq == 32) return pick_attn_kernel_bk<PASS, OCC, BF16, D, 1, 32>(bk, arb, wide);
    if (bq == 64) return pick_attn_kernel_bk<PASS, OCC2, BF16, D, 2, 64>(bk, arb, wide);
    return pick_attn_kernel_bk<PASS, OCC2, BF16, D, 2, 128>(bk, arb, wide);
}

template <int PASS, int OCC>
static attn_fn pick_attn_kernel(const Problem &pb, int &qsub)
{
    qsub = pb.b == 128 ? 2 : 1;
    const bool arb = pb.mask == STREAM_MASK_ARRAY;
    const bool wide = pb.kmax > kMaxTopk;              // lists longer than one register of entries
    if (pb.dtype == STREAM_BF16)
        return pb.d == 128 ? pick_attn_kernel_d<PASS, OCC, true, 128>(pb.b, pb.bk, arb, wide)
                           : pick_attn_kernel_d<PASS, OCC, true, 64>(pb.b, pb.bk, arb, wide);
    return pb.d == 128 ? pick_attn_kernel_d<PASS, OCC, false, 128>(pb.b, pb.bk, arb, wide)
                       : pick_attn_kernel_d<PASS, OCC, false, 64>(pb.b, pb.bk, arb, wide);
}

struct AttnWorkspace {
    size_t kp, vp, lse2, cany, call, total;
};

static AttnWorkspace attn_layout(const Problem &pb)
{
    AttnWorkspace w;
    const size_t tile = align_up((size_t)pb.Hkv * pb.NB * pb.b * pb.d * pb.esize, 256);
    w.kp = 0;
    w.vp = tile;
    w.lse2 = 2 * tile;
    size_t off = 2 * tile + align_up((size_t)pb.H * pb.T * 4, 256);
    // block-level summaries of an explicit mask array
    const size_t bm = pb.mask == STREAM_MASK_ARRAY ? align_up((size_t)pb.NB * block_bitmap_words(pb) * 4, 256) : 0;
    w.cany = off; off += bm;
    w.call = off; off += bm;
    w.total = off;
    return w;
}

__global__ void __launch_bounds__(256) zero_kernel(float *p, long long n)
{
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0.f;
}

}  // namespace stream

using namespace stream;

extern "C" {

size_t stream_sparse_attn_workspace_bytes(const stream_shape *shape, int topk_max)
{
    Problem pb;
    if (topk_max < 1) return 0;
    if (make_problem(shape, 0, nullptr, 0, &pb) != STREAM_OK) return 0;
    return attn_layout(pb).total;
}

stream_status stream_sparse_attn(const void *Q, const void *K, const void *V,
                                 const stream_shape *shape,
                                 const int *idx, const int *cnt, int topk_max, float scale,
                                 void *O, float *lse, float *mass,
                                 void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!Q || !K || !V || !shape || !idx || !cnt || !O) return STREAM_EINVAL;
    if (topk_max < 1 || !(scale > 0.f) || !isfinite(scale)) return STREAM_EINVAL;
    Problem pb;
    stream_status rc = make_problem(shape, 0, nullptr, 0, &pb);
    if (rc != STREAM_OK) return rc;
    pb.kmax = topk_max;
    if (topk_max > kMaxTopkWide) return STREAM_EUNSUPPORTED;
    {
        int qsub_probe = 1;
        if (!pick_attn_kernel<1, 1>(pb, qsub_probe)) return STREAM_EUNSUPPORTED;   // long lists with a mask array
    }
    const long long dflt_h = pb.T * pb.d;
    const long long q_sh = shape->q_stride_h ? shape->q_stride_h : dflt_h;
    const long long q_st = shape->q_stride_t ? shape->q_stride_t : pb.d;
    const long long k_sh = shape->k_stride_h ? shape->k_stride_h : dflt_h;
    const long long k_st = shape->k_stride_t ? shape->k_stride_t : pb.d;
    const long long v_sh = shape->v_stride_h ? shape->v_stride_h : dflt_h;
    const long long v_st = shape->v_stride_t ? shape->v_stride_t : pb.d;
    const long long o_sh = shape->o_stride_h ? shape->o_stride_h : dflt_h;
    const long long o_st = shape->o_stride_t ? shape->o_stride_t : pb.d;
    if (q_st < pb.d || k_st < pb.d || v_st < pb.d || o_st < pb.d) return STREAM_EINVAL;
    if (((uintptr_t)Q | (uintptr_t)K | (uintptr_t)V | (uintptr_t)O) & 15) return STREAM_EINVAL;
    if (((q_sh | q_st | k_sh | k_st | v_sh | v_st | o_sh | o_st) * pb.esize) & 15) return STREAM_EINVAL;
    // the kernels address a wavefront's query rows with 32-bit offsets from its first row
    if (q_st * pb.esize * 128 >= (1LL << 31)) return STREAM_EUNSUPPORTED;
    const AttnWorkspace w = attn_layout(pb);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < w.total) return STREAM_EWORKSPACE;
    hipStream_t st = (hipStream_t)hip_stream;
    char *ws = (char *)workspace;

    rc = launch_pack(K, k_sh, k_st, ws + w.kp, pb, st);
    if (rc != STREAM_OK) return rc;
    {
        PackVParams pv;
        pv.src = (const char *)V;
        pv.dst = ws + w.vp;
        pv.stride_h_bytes = v_sh * pb.esize;
        pv.stride_t_bytes = v_st * pb.esize;
        pv.d = pb.d; pv.esize = pb.esize; pv.b = pb.b; pv.NB = pb.NB;
        pv.seqs = pb.seqs;
        const long long grid = (long long)pb.Hkv * pb.NB * (pb.b / 32);
        if (grid > 0x7fffffffLL) return STREAM_EUNSUPPORTED;
        hipLaunchKernelGGL(pack_v_kernel, dim3((unsigned)grid), dim3(256), 0, st, pv);
        if (hipGetLastError() != hipSuccess) return STREAM_EDEVICE;
    }
    if (mass) {
        const long long n = (long long)pb.H * pb.T;
        hipLaunchKernelGGL(zero_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, mass, n);
        if (hipGetLastError() != hipSuccess) return STREAM_EDEVICE;
    }
    AttnParams p;
    p.Q = (const char *)Q;
    p.Kp = ws + w.kp;
    p.Vp = ws + w.vp;
    p.O = (char *)O;
    p.q_sh_b = q_sh * pb.esize; p.q_st_b = q_st * pb.esize;
    p.o_sh_b = o_sh * pb.esize; p.o_st_b = o_st * pb.esize;
    p.idx = idx; p.cnt = cnt; p.lse = lse; p.mass = mass;
    p.T = pb.T; p.H = pb.H; p.g = pb.g; p.NB = pb.NB; p.kmax = topk_max;
    p.scale_log2e = scale * 1.4426950408889634f;
    p.mask = pb.mask; p.window = pb.window;
    p.cbits = pb.cbits; p.cpitch = pb.cpitch;
    p.call = (const unsigned *)(ws + w.call);
    p.cw = pb.mask == STREAM_MASK_ARRAY ? block_bitmap_words(pb) : 0;
    if (pb.mask == STREAM_MASK_ARRAY) {
        rc = launch_block_bitmaps(pb, (unsigned *)(ws + w.cany), (unsigned *)(ws + w.call), st);
        if (rc != STREAM_OK) return rc;
    }
    p.seqs = pb.seqs;
    p.lse2 = mass ? (float *)(ws + w.lse2) : nullptr;
    for (int pass = 1; pass <= (mass ? 2 : 1); ++pass) {
        int qsub = 1;
        attn_fn fn = pass == 1 ? pick_attn_kernel<1, 1>(pb, qsub) : pick_attn_kernel<2, 2>(pb, qsub);
        const long long items_per_kv = (long long)pb.NB * pb.g * qsub;
        const long long per_kv = (items_per_kv + 3) / 4;
        if (per_kv * pb.Hkv + 64 > 0x7fffffffLL) return STREAM_EUNSUPPORTED;
        p.map = make_wg_map(pb.Hkv, (int)per_kv);
        hipLaunchKernelGGL(fn, dim3((unsigned)p.map.grid), dim3(256), 0, st, p);
        if (hipGetLastError() != hipSuccess) return STREAM_EDEVICE;
    }
    return STREAM_OK;
}

}  // extern "C"
