// stream_prune: Algorithm 2 ("Stream", Appendix C) on gfx950.
//
// A wavefront owns one (query head, query block) row (four wavefronts share a row when
// block = 128) and runs the row's refinement levels back to back, all of them in one launch by
// default: it holds the row's Q tile in registers as MFMA operand fragments and, per level,
// gathers the packed K tiles of the branches that need a new score, reduces each 32x32
// accumulator set to the masked maximum (score line of Alg. 2 / Eq. (4)), selects the k best of
// the 2k branch scores across its lanes and hands the surviving nodes, in positional order, to
// the next level through LDS (through the node lists [heads, NB, k] in the workspace when the
// caller splits a row's levels over several launches): O(T) memory either way.
// Variants of the same kernel: a sweep over several k with a per-row cache of block scores
// (stream_prune_multi) and a sparsity constant per row (stream_prune_variable).
#include "stream_prune.h"

#include <math.h>

#include <mutex>

namespace stream {

// Template parameters: element type, head dim, 32-row groups of Q per wavefront (MB), 32-key
// groups of K per wavefront (NG), wavefronts per row (WPR: 1, or 4 = 2 query halves x 2 key
// halves for block 128), occupancy hint, k sweep with the block-score cache (MULTI).
// ARB: the mask C is an explicit bit array (STREAM_MASK_ARRAY) instead of a rule: a branch's
// representative is found by scanning the row's C^blk bits, and every block that is not wholly
// visible takes the token-level test against the array.
// KS: a key block is scored as KS sub-tiles of 32 * NG keys one after the other (its score is the
// maximum over them): half the K registers and accumulators of the whole-block form (no register
// spills, and a level's first MFMAs start after half as many bytes have arrived).  Used for short
// lists, where a level has a handful of tiles: measured 3-5 % faster there, 3-4 % slower on long
// lists.  (A third wavefront per SIMD would fit only with ~30 spilled registers: slower.)
template <bool BF16, int D, int MB, int NG, int WPR, int OCC, bool MULTI, bool ARB = false, int KS = 1>
__global__ void __launch_bounds__(256, OCC) level_kernel(const PruneParams p)
{
    static_assert(KS == 1 || WPR == 1, "sub-tiles only in the one-wavefront-per-row form");
    constexpr int ES = BF16 ? 2 : 4;
    constexpr int FR = D * ES / 32;                       // fragments per 32-token group
    // bf16 tiles are multiplied with 16x16x32 MFMAs (S16): under the power limit that governs a
    // kernel made of back-to-back MFMAs this shape sustains ~10 % more FLOP/s than 32x32x16 on
    // the same data.  An operand fragment (64 lanes x 16 bytes) then covers 16 rows x 32
    // contraction indices instead of 32 x 16: lane l supplies row l % 16, 16-byte chunk l / 16 of
    // the fragment's 64-byte slice of the row.  fp32 keeps 32x32x2.
    constexpr bool S16 = BF16;
    constexpr int RG = S16 ? 2 * MB : MB;                 // row groups of the Q tile (16 or 32 rows each)
    constexpr int CG = S16 ? 2 * NG : NG;                 // key groups of the K tile
    constexpr int KF = S16 ? D / 32 : FR;                 // fragments of a group along the contraction axis
    constexpr int GR = S16 ? 16 : 32;                     // rows / keys per group
    constexpr int AE = S16 ? 4 : 16;                      // accumulator elements per lane and group pair
    typedef float acc_t __attribute__((ext_vector_type(AE)));
    static_assert(RG * KF == MB * FR && CG * KF == NG * FR, "same number of fragments either way");
    constexpr int BQ = 32 * MB * (WPR == 4 ? 2 : 1);      // query block b_q
    constexpr int BK = 32 * NG * KS * (WPR == 4 ? 2 : 1); // key block b_k
    constexpr long long TILE_BYTES = (long long)BK * D * ES;
    constexpr int GROUP_BYTES = 32 * D * ES;
    __shared__ int s_rep[4][2 * kMaxTopk];
    __shared__ float s_sc[4][2 * kMaxTopk];
    __shared__ int s_nf[4][kMaxTopk], s_nl[4][kMaxTopk];   // survivors on their way to the next level
    __shared__ float s_ns[4][kMaxTopk];
    // k sweep: block scores this row has computed so far, whatever k they were computed for
    // (entry = block id << 32 | score bits, direct mapped; a miss only costs a recomputation)
    __shared__ unsigned long long s_cache[MULTI ? 4 : 1][MULTI ? kScoreCache : 1];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform: keep it scalar
    int kvh, slot;
    if (!wg_decode(p.map, blockIdx.x, kvh, slot)) return;
    const long long rows_per_kv = (long long)p.NB * p.g;
    const long long rk = WPR == 1 ? (long long)slot * 4 + wave : (long long)slot;
    if (rk >= rows_per_kv) return;
    const int gb = p.NB - 1 - (int)(rk / p.g);            // long rows first
    const int h = kvh * p.g + (int)(rk % p.g);
    const int sq = seq_of_block(p.seqs, gb);
    const SeqDesc sd = p.seqs.d[sq];
    const int q = gb - sd.blk0, L = sd.len;
    const int N = sd.nblk * BQ / BK;                      // key blocks of the sequence: the nodes range over these
    int row_k = sd.k, row_levels = sd.levels;
    if (!MULTI && p.vk_den > 0) {
        int valid = mask_rmax(p.mask, q, BQ, BK, L) - mask_rmin(p.mask, p.window, q, BQ, BK) + 1;
        if constexpr (ARB) {
            valid = 0;
            for (int w = 0; w < p.cw; ++w) valid += __popc(p.cany[(long long)gb * p.cw + w]);
        }
        row_k = variable_k(valid, p.vk_num, p.vk_den, p.vk_min, p.kmax);
        row_levels = levels_for(N, row_k);
    }
    if (!MULTI && p.level_begin > row_levels) return;
    const int qh = WPR == 4 ? (wave >> 1) : 0;            // query half / key half of this wavefront
    const int kh = WPR == 4 ? (wave & 1) : 0;

    // ---- Q tile of this wavefront as A-operand fragments: lane (mrow = lane % 32, gh = lane / 32)
    //      holds, for fragment fr, the 16 bytes at chunk 2*fr + gh of row mrow.  Issued first so
    //      that the loads overlap the node-state loads below; rows past the end of the sequence
    //      fall outside the buffer resource and read as zeros.
    uint4 qf[RG][KF];
    {
        // the resource starts at this wavefront's first query row (64-bit arithmetic) and spans
        // its real rows only, so per-lane offsets stay below 128 token strides whatever the
        // length of the sequence and the layout of Q
        const int qrow0 = q * BQ + qh * 32 * MB;
        const int qrows = L - qrow0 < 32 * MB ? L - qrow0 : 32 * MB;
        const __amdgpu_buffer_rsrc_t qrs = make_tile_rsrc(
            p.Q + (long long)h * p.q_sh_b + (sd.tok0 + qrow0) * p.q_st_b,
            qrows > 0 ? (unsigned)((long long)(qrows - 1) * p.q_st_b + D * ES) : 0u);
        // S16: lane (row l % 16, chunk l / 16 of the 64-byte slice); else (row l % 32, chunk l / 32
        // of the 32-byte slice)
        const int mrow = S16 ? (lane & 15) : (lane & 31), gh = S16 ? (lane >> 4) : (lane >> 5);
        constexpr int SLICE = S16 ? 64 : 32;
#pragma unroll
        for (int rb = 0; rb < RG; ++rb) {
            const unsigned voff = (unsigned)(rb * GR + mrow) * (unsigned)p.q_st_b + gh * 16;
#pragma unroll
            for (int fr = 0; fr < KF; ++fr) {
                const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(qrs, voff + fr * SLICE, 0, 0);
                qf[rb][fr] = make_uint4(v[0], v[1], v[2], v[3]);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }

    if constexpr (MULTI) {
        for (int i = lane; i < kScoreCache; i += 64) s_cache[wave][i] = ~0ull;
        wave_sync();
    }
    unsigned long long tiles_done = 0;
    const int n_k = MULTI ? p.n_k : 1;
    for (int ki = 0; ki < n_k; ++ki) {
    // this pass's k, its number of levels and its output row
    int k = row_k, levels = row_levels;
    long long row = (long long)h * p.NB + gb;
    if constexpr (MULTI) {
        k = p.klist[ki];
        levels = levels_for(N, k);
        row = ((long long)h * n_k + ki) * p.NB + gb;
    }
    const int level_begin = MULTI ? 1 : p.level_begin;
    const int level_last = MULTI ? levels : (p.level_end < levels ? p.level_end : levels);

    // ---- node of this lane (node init line of Alg. 2 at the first level)
    int f = 0, l = -1;
    float sc = -INFINITY;
    bool live = false;
    if (level_begin == 1) {
        if (lane < k) {
            f = (int)(((long long)lane * N) / k);
            l = (int)(((long long)(lane + 1) * N) / k) - 1;
            live = f <= l;
        }
    } else {
        // all four loads are independent (slots past the live count hold stale but allocated data)
        const int c = p.ncnt[row];
        if (lane < p.kmax) {
            f = p.nf[row * p.kmax + lane];
            l = p.nl[row * p.kmax + lane];
            sc = p.ns[row * p.kmax + lane];
        }
        live = lane < c;
        if (!live) { f = 0; l = -1; sc = -INFINITY; }
    }

    // K tiles of this (kv head, sequence), from this wavefront's key half on
    const char *kbase = p.Kp + ((long long)kvh * p.NB + sd.blk0) * BQ * D * ES + (long long)kh * NG * GROUP_BYTES;
    const unsigned kbytes = (unsigned)((long long)N * TILE_BYTES - (long long)kh * NG * GROUP_BYTES);
    const __amdgpu_buffer_rsrc_t krs = make_tile_rsrc(kbase, kbytes);
    const unsigned lane_off = lane * 16;
    const bool tail_row = (q + 1) * BQ > L;               // the query block has padded rows
    const int qtok0 = q * BQ + qh * 32 * MB;
    // valid key blocks of this row under the mask C: rmin .. rmax (a branch's representative is
    // its first valid block); blocks the mask cuts through need the token-level test
    const int rmin = mask_rmin(p.mask, p.window, q, BQ, BK), rmax = mask_rmax(p.mask, q, BQ, BK, L);
    // blocks <= edge_hi hold a key that lies outside the window of the block's last query
    const int edge_num = q * BQ + BQ - 1 - p.window;
    const int edge_hi = p.mask == STREAM_MASK_SLIDING && edge_num >= 0 ? edge_num / BK : -1;
    // ... and so do the blocks from cut_lo on: those that reach past the row's first query (causal
    // rules: (r + 1) b_k - 1 > q b_q) or past the end of the sequence ((r + 1) b_k > L); every block
    // when the query block itself has padded rows
    int cut_lo = L / BK;
    if (p.mask != STREAM_MASK_FULL && (q * BQ + 1) / BK < cut_lo) cut_lo = (q * BQ + 1) / BK;
    if (tail_row) cut_lo = 0;
    const long long o = row * p.kmax;
    // ARB: first key block of [a, b] that C^blk leaves to this row, or -1
    const unsigned *anyrow = ARB ? p.cany + (long long)gb * p.cw : nullptr;
    const unsigned *allrow = ARB ? p.call + (long long)gb * p.cw : nullptr;
    auto first_valid = [&](int a, int b) -> int {
        if (a > b) return -1;
        for (int w = a >> 5; w <= (b >> 5); ++w) {
            unsigned x = anyrow[w];
            if (w == (a >> 5)) x &= ~0u << (a & 31);
            if (w == (b >> 5) && (b & 31) != 31) x &= (1u << ((b & 31) + 1)) - 1u;
            if (x) return w * 32 + __builtin_ctz(x);
        }
        return -1;
    };

    // The Q tile has to be there before the first MFMA anyway; waiting for it here, once, lets
    // the waits inside the tile loop count K fragments only (vmcnt(0), other counters untouched).
    __builtin_amdgcn_s_waitcnt(0x0F70);

    // A row runs its levels level_begin .. level_last back to back: the Q tile stays in
    // registers and the node list moves from one level to the next through LDS.
    for (int level = level_begin; level <= level_last; ++level) {
        const bool first = level == 1;
        // ---- split at the midpoint; causal validity: a branch is valid iff it is non-empty and
        //      starts at or before the query block; its representative is its first block.
        const int m = (f + l + 1) >> 1;
        int rep_p = f > rmin ? f : rmin;                      // the node's own representative
        int rep0 = rep_p;                                     // left child [f, m-1]
        int rep1 = m > rmin ? m : rmin;                       // right child [m, l] (never empty)
        bool v0 = live && m > f && rep0 <= (m - 1 < rmax ? m - 1 : rmax);
        bool v1 = live && rep1 <= (l < rmax ? l : rmax);
        if constexpr (ARB) {
            rep0 = live ? first_valid(f, m - 1) : -1;
            rep1 = live ? first_valid(m, l) : -1;
            v0 = rep0 >= 0;
            v1 = rep1 >= 0;
            rep_p = v0 ? rep0 : rep1;                         // the node's first valid block
        }
        // a child whose representative is the node's own inherits the node's score
        bool need0 = v0 && first;
        bool need1 = v1 && (first || rep1 != rep_p);
        float c0 = 0.f, c1 = 0.f;
        bool hit0 = false, hit1 = false;
        if constexpr (MULTI) {
            // a score of the same block computed earlier for this row (another k, another level)
            if (need0) {
                const unsigned long long e = s_cache[wave][rep0 & (kScoreCache - 1)];
                hit0 = (int)(e >> 32) == rep0;
                c0 = __builtin_bit_cast(float, (unsigned)e);
            }
            if (need1) {
                const unsigned long long e = s_cache[wave][rep1 & (kScoreCache - 1)];
                hit1 = (int)(e >> 32) == rep1;
                c1 = __builtin_bit_cast(float, (unsigned)e);
            }
            need0 = need0 && !hit0;
            need1 = need1 && !hit1;
        }

        const unsigned long long b0 = __ballot(need0), b1 = __ballot(need1);
        const int n0 = __popcll(b0), nt = n0 + __popcll(b1);
        const int pos0 = lanes_below(b0), pos1 = n0 + lanes_below(b1);
        if (need0) s_rep[wave][pos0] = rep0;
        if (need1) s_rep[wave][pos1] = rep1;
        wave_sync();

        uint4 kf[CG][KF];
        if (nt > 0) {
            const int r0 = __builtin_amdgcn_readfirstlane(s_rep[wave][0]);
            // same order as the refills in the loop below: waits count loads in issue order
#pragma unroll
            for (int fr = 0; fr < KF; ++fr)
#pragma unroll
                for (int cb = 0; cb < CG; ++cb) {
                    kf[cb][fr] = load_frag(krs, lane_off, (unsigned)r0 * (unsigned)TILE_BYTES, cb * KF + fr);
                    __builtin_amdgcn_sched_barrier(0);
                }
        }
        float mx = -INFINITY;
        for (int u = 0; u < nt * KS; ++u) {
            // sub-tile sk of the t-th block to score; the one after it (the last repeats itself)
            const int t = u / KS, sk = u % KS;
            const bool more = u + 1 < nt * KS;
            const int un = more ? u + 1 : u;
            const int r = __builtin_amdgcn_readfirstlane(s_rep[wave][t]);
            const unsigned nxt = (unsigned)__builtin_amdgcn_readfirstlane(s_rep[wave][un / KS]) * (unsigned)TILE_BYTES +
                                 (unsigned)(un % KS) * (unsigned)(NG * GROUP_BYTES);
            // after the level's last tile there is nothing to fetch ahead: the refills then go
            // through a resource of zero bytes, which answers every load with zeros without a
            // memory access (loads return in order: real ones would hold up the next level's first tile)
            const __amdgpu_buffer_rsrc_t krs_next = make_tile_rsrc(kbase, more ? kbytes : 0u);
            acc_t acc[RG][CG];
#pragma unroll
            for (int rb = 0; rb < RG; ++rb)
#pragma unroll
                for (int cb = 0; cb < CG; ++cb)
#pragma unroll
                    for (int i = 0; i < AE; ++i) acc[rb][cb][i] = 0.f;
#pragma unroll
            for (int fr = 0; fr < KF; ++fr) {
#pragma unroll
                for (int cb = 0; cb < CG; ++cb) {
#pragma unroll
                    for (int rb = 0; rb < RG; ++rb) {
                        if constexpr (S16)
                            acc[rb][cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                                __builtin_bit_cast(bf16x8, qf[rb][fr]), __builtin_bit_cast(bf16x8, kf[cb][fr]),
                                acc[rb][cb], 0, 0, 0);
                        else
                            acc[rb][cb] = mfma_frag<BF16>(qf[rb][fr], kf[cb][fr], acc[rb][cb]);
                    }
                    // the fragment is consumed: refill its registers from the next tile right here,
                    // so that every fragment of the next tile has a whole tile of MFMA time to arrive
                    // (the scheduling barriers stop the compiler from sinking the loads to the end)
                    __builtin_amdgcn_sched_barrier(0);
                    kf[cb][fr] = load_frag(krs_next, lane_off, nxt, cb * KF + fr);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            // the block reaches past the row's first query (causal rules) or past the sequence
            bool cut = (r <= edge_hi) | (r >= cut_lo);
            if constexpr (ARB) cut = !((allrow[r >> 5] >> (r & 31)) & 1u);
            if (!cut) {
#pragma unroll
                for (int rb = 0; rb < RG; ++rb)
#pragma unroll
                    for (int cb = 0; cb < CG; ++cb)
#pragma unroll
                        for (int i = 0; i < AE; ++i) mx = fmaxf(mx, acc[rb][cb][i]);
            } else {
                // a block the mask cuts through (diagonal, window edge) or with padded rows/cols:
                // token-level test.  Accumulator layouts: 32x32 - lane holds column lane % 32, element
                // i is row 8*(i/4) + 4*(lane/32) + (i%4); 16x16 - column lane % 16, row 4*(lane/16) + i.
                const int ktok0 = r * BK + (kh + sk) * 32 * NG;
                // ARB: lane j fetches the mask words of query row j (and j + 64) of this tile, one per
                // 32-key group; an element then takes its row's word from the lane that fetched it
                constexpr int RS = (32 * MB + 63) / 64;
                unsigned rowword[RS][NG];
                if constexpr (ARB) {
#pragma unroll
                    for (int sl = 0; sl < RS; ++sl) {
                        const int tq = qtok0 + sl * 64 + lane;
                        const bool ok = (sl * 64 + lane < 32 * MB) & (tq < L);
#pragma unroll
                        for (int cb = 0; cb < NG; ++cb)
                            rowword[sl][cb] = (ok & (ktok0 + cb * 32 < L))       // (not a word wholly past the end of the row)
                                                  ? p.cbits[(long long)tq * p.cpitch + ((ktok0 >> 5) + cb)] : 0u;
                    }
                }
#pragma unroll
                for (int rb = 0; rb < RG; ++rb)
#pragma unroll
                    for (int cb = 0; cb < CG; ++cb)
#pragma unroll
                        for (int i = 0; i < AE; ++i) {
                            // row of the wavefront's Q tile and key of its K tile this element belongs to
                            const int qr = S16 ? rb * 16 + (lane >> 4) * 4 + i
                                               : rb * 32 + (i >> 2) * 8 + (lane >> 5) * 4 + (i & 3);
                            const int kc = S16 ? cb * 16 + (lane & 15) : cb * 32 + (lane & 31);
                            const int tq = qtok0 + qr;
                            const int tk = ktok0 + kc;
                            bool visible = (tq < L) & (tk < L);
                            if constexpr (ARB) {
                                const unsigned cwd = (unsigned)__shfl((int)rowword[qr >> 6][kc >> 5], qr & 63);
                                visible = visible & ((cwd >> (kc & 31)) & 1u);
                            } else {
                                visible = visible & mask_token(p.mask, p.window, tq, tk);
                            }
                            mx = visible ? fmaxf(mx, acc[rb][cb][i]) : mx;
                        }
            }
            if (sk == KS - 1) {
                mx = wave_max(mx);
                if (lane == 0) s_sc[wave][t] = mx;
                mx = -INFINITY;
            }
        }
        tiles_done += (unsigned long long)nt;
        wave_sync();
        if constexpr (WPR == 4) __syncthreads();

        auto tile_score = [&](int t) -> float {
            if constexpr (WPR == 4)
                return fmaxf(fmaxf(s_sc[0][t], s_sc[1][t]), fmaxf(s_sc[2][t], s_sc[3][t]));
            else
                return s_sc[wave][t];
        };
        float s0 = -INFINITY, s1 = -INFINITY;
        if (v0) s0 = need0 ? tile_score(pos0) : (hit0 ? c0 : sc);
        if (v1) s1 = need1 ? tile_score(pos1) : (hit1 ? c1 : sc);
        if constexpr (MULTI) {
            if (need0) s_cache[wave][rep0 & (kScoreCache - 1)] = ((unsigned long long)(unsigned)rep0 << 32) | __builtin_bit_cast(unsigned, s0);
            if (need1) s_cache[wave][rep1 & (kScoreCache - 1)] = ((unsigned long long)(unsigned)rep1 << 32) | __builtin_bit_cast(unsigned, s1);
        }
        // the four wavefronts of a row must all have read this level's tile scores before any of
        // them writes the next level's
        if constexpr (WPR == 4) __syncthreads();

        // ---- top-k of the 2k branch scores (ties to the lower position): see select_topk_wave
        const float sel_s[2] = {s0, s1};
        const bool sel_v[2] = {v0, v1};
        bool sel_keep[2];
        select_topk_wave<2>(sel_s, sel_v, k, lane, sel_keep);
        const bool keep0 = sel_keep[0], keep1 = sel_keep[1];
        const unsigned long long kb0 = __ballot(keep0), kb1 = __ballot(keep1);
        const int before = lanes_below(kb0) + lanes_below(kb1);
        const int p0 = before, p1 = before + (keep0 ? 1 : 0);
        const int newcnt = __popcll(kb0) + __popcll(kb1);
        const bool writer = WPR == 1 || wave == 0;

        if (p.trace && writer) {
            int *tr = p.trace + (((long long)(level - 1) * p.H * n_k * p.NB + row) * p.kmax) * 2;
            if (keep0) { tr[2 * p0] = f; tr[2 * p0 + 1] = m - 1; }
            if (keep1) { tr[2 * p1] = m; tr[2 * p1 + 1] = l; }
            if (lane >= newcnt && lane < p.kmax) { tr[2 * lane] = -1; tr[2 * lane + 1] = -1; }
        }
        if (level == levels) {
            // every node is now a single block: emit I (ascending), pad, count
            if (writer) {
                if (keep0) { p.idx[o + p0] = rep0; if (p.score) p.score[o + p0] = s0; }
                if (keep1) { p.idx[o + p1] = rep1; if (p.score) p.score[o + p1] = s1; }
                if (lane >= newcnt && lane < p.kmax) {
                    p.idx[o + lane] = -1;
                    if (p.score) p.score[o + lane] = -INFINITY;
                }
                if (lane == 0) p.cnt[row] = newcnt;
                // rows that finish before the deepest one: their node list stays as it is
                if (p.trace)
                    for (int lv = level + 1; lv <= p.max_levels; ++lv) {
                        int *tr = p.trace + (((long long)(lv - 1) * p.H * n_k * p.NB + row) * p.kmax) * 2;
                        if (keep0) { tr[2 * p0] = f; tr[2 * p0 + 1] = m - 1; }
                        if (keep1) { tr[2 * p1] = m; tr[2 * p1 + 1] = l; }
                        if (lane >= newcnt && lane < p.kmax) { tr[2 * lane] = -1; tr[2 * lane + 1] = -1; }
                    }
            }
        } else if (level == level_last) {
            // update: survivors overwrite the row's node list in memory, in positional order,
            // for the launch that runs the next levels
            if (writer) {
                if (keep0) { p.nf[o + p0] = f; p.nl[o + p0] = m - 1; p.ns[o + p0] = s0; }
                if (keep1) { p.nf[o + p1] = m; p.nl[o + p1] = l;     p.ns[o + p1] = s1; }
                if (lane == 0) p.ncnt[row] = newcnt;
            }
        } else {
            // update: survivors become the nodes of the next level, node j on lane j
            if (keep0) { s_nf[wave][p0] = f; s_nl[wave][p0] = m - 1; s_ns[wave][p0] = s0; }
            if (keep1) { s_nf[wave][p1] = m; s_nl[wave][p1] = l;     s_ns[wave][p1] = s1; }
            wave_sync();
            live = lane < newcnt;
            // (the lane's LDS address is formed here, from an opaque copy of the lane number: hoisted
            // out of the level loop it does not fit the registers and comes back from scratch, a
            // memory round trip per level)
            int ln = lane;
            asm volatile("" : "+v"(ln));
            f = live ? s_nf[wave][ln] : 0;
            l = live ? s_nl[wave][ln] : -1;
            sc = live ? s_ns[wave][ln] : -INFINITY;
            wave_sync();
        }
    }
    if constexpr (MULTI) wave_sync();     // the last level's cache entries, before the next k reads them
    }
    if (p.tiles && (WPR == 1 || wave == 0) && lane == 0) atomicAdd(p.tiles, tiles_done);
}

struct PruneWorkspace {
    size_t kp, nf, nl, ns, ncnt, cany, call, total;
};

static PruneWorkspace prune_layout(const Problem &pb)
{
    PruneWorkspace w;
    size_t off = 0;
    const size_t rows = (size_t)pb.H * pb.NB;
    w.kp = off;   off += align_up((size_t)pb.Hkv * pb.NB * pb.b * pb.d * pb.esize, 256);
    // node lists: used only when a row's levels are split over several launches (never by the
    // wide kernel, whose lists live in LDS)
    const size_t kk = pb.kmax > kMaxTopk ? 0 : (size_t)pb.kmax;
    w.nf = off;   off += align_up(rows * kk * 4, 256);
    w.nl = off;   off += align_up(rows * kk * 4, 256);
    w.ns = off;   off += align_up(rows * kk * 4, 256);
    w.ncnt = off; off += align_up(rows * 4, 256);
    // block-level summaries of an explicit mask array
    const size_t bm = pb.mask == STREAM_MASK_ARRAY ? align_up((size_t)pb.NB * block_bitmap_words(pb) * 4, 256) : 0;
    w.cany = off; off += bm;
    w.call = off; off += bm;
    w.total = off;
    return w;
}

// Levels a row runs inside one launch unless the caller asks otherwise (all of them).
constexpr int kDefaultLevelsPerLaunch = 64;

typedef void (*level_fn)(const PruneParams);

// One wavefront per row holds MB x NG accumulator tiles; beyond 2 x 2 only one wavefront fits a
// SIMD's registers.  fp32 fragments are twice as many: with d = 128 the 4 x 2 and 2 x 4 shapes do
// not fit at all.
// Lists this short take the two-sub-tile form (KS = 2) of the 64 x 64 bf16 kernel.
constexpr int kShortListTopk = 8;

template <bool MULTI, bool BF16, int D, bool ARB>
static level_fn pick_level_kernel_d(int bq, int bk, int kmax, int &wpr)
{
    constexpr int OCC2 = (BF16 || D == 64) ? 2 : 1;
    constexpr bool BIG = BF16 || D == 64;           // 6 fragment groups + 8 accumulator tiles fit
    wpr = 1;
    const int mb = bq / 32, ng = bk / 32;
    if (mb == 4 && ng == 4) { wpr = 4; return level_kernel<BF16, D, 2, 2, 4, OCC2, MULTI, ARB>; }
    if (mb == 1 && ng == 1) return level_kernel<BF16, D, 1, 1, 1, 2, MULTI, ARB>;
    if constexpr (BF16 && !MULTI && !ARB)
        if (mb == 2 && ng == 2 && kmax <= kShortListTopk) return level_kernel<BF16, D, 2, 1, 1, 2, MULTI, ARB, 2>;
    if (mb == 2 && ng == 2) return level_kernel<BF16, D, 2, 2, 1, OCC2, MULTI, ARB>;
    if (mb == 1 && ng == 2) return level_kernel<BF16, D, 1, 2, 1, OCC2, MULTI, ARB>;
    if (mb == 2 && ng == 1) return level_kernel<BF16, D, 2, 1, 1, OCC2, MULTI, ARB>;
    constexpr int OCC41 = (BF16 && D == 64) ? 2 : 1;   // 5 fragment groups of 8 or 16 registers + 4 tiles
    if (mb == 1 && ng == 4) return level_kernel<BF16, D, 1, 4, 1, OCC41, MULTI, ARB>;
    if (mb == 4 && ng == 1) return level_kernel<BF16, D, 4, 1, 1, OCC41, MULTI, ARB>;
    if constexpr (BIG) {
        if (mb == 2 && ng == 4) return level_kernel<BF16, D, 2, 4, 1, 1, MULTI, ARB>;
        if (mb == 4 && ng == 2) return level_kernel<BF16, D, 4, 2, 1, 1, MULTI, ARB>;
    }
    return nullptr;
}

template <bool MULTI, bool ARB>
static level_fn pick_level_kernel_t(const Problem &pb, int &wpr)
{
    if (pb.dtype == STREAM_BF16)
        return pb.d == 128 ? pick_level_kernel_d<MULTI, true, 128, ARB>(pb.b, pb.bk, pb.kmax, wpr)
                           : pick_level_kernel_d<MULTI, true, 64, ARB>(pb.b, pb.bk, pb.kmax, wpr);
    return pb.d == 128 ? pick_level_kernel_d<MULTI, false, 128, ARB>(pb.b, pb.bk, pb.kmax, wpr)
                       : pick_level_kernel_d<MULTI, false, 64, ARB>(pb.b, pb.bk, pb.kmax, wpr);
}

static level_fn pick_level_kernel(const Problem &pb, bool multi, int &wpr)
{
    if (pb.mask == STREAM_MASK_ARRAY)
        return multi ? pick_level_kernel_t<true, true>(pb, wpr) : pick_level_kernel_t<false, true>(pb, wpr);
    return multi ? pick_level_kernel_t<true, false>(pb, wpr) : pick_level_kernel_t<false, false>(pb, wpr);
}

}  // namespace stream

using namespace stream;

// ---------------------------------------------------------------------------------------------
// Scratch of stream_prune_static: the workspace of stream_prune (packed K tiles, node lists,
// block bitmaps of a mask array) in a device array that belongs to the library, for callers that
// cannot allocate.  Every GPU the library runs on holds its own copy at its own address; host
// code never uses the array's name as an address, only the pointer hipGetSymbolAddress returns
// for the device that is current.
// ---------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[STREAM_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void *g_scratch_ptr[kMaxDevices];      // per device, set on the first call there

// Device address of `scratch` on the current device (looked up once per device), or nullptr.
static void *scratch_of_current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return nullptr;
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

// Packs K and runs the refinement kernel: once per group of levels, or (topk_list != nullptr)
// once for a whole sweep over k, every row then running all its levels for every k in turn.
struct VariableK { int num, den, kmin; };   // den == 0: off

static stream_status run_prune(const void *Q, const void *K, const stream_shape *shape, const Problem &pb,
                               const int *topk_list, int n_k, VariableK vk, int *idx, int *cnt, float *score,
                               const stream_prune_diag *diag, void *workspace, size_t workspace_bytes,
                               void *hip_stream)
{
    const bool multi = topk_list != nullptr;
    const long long q_sh = shape->q_stride_h ? shape->q_stride_h : pb.T * pb.d;
    const long long q_st = shape->q_stride_t ? shape->q_stride_t : pb.d;
    const long long k_sh = shape->k_stride_h ? shape->k_stride_h : pb.T * pb.d;
    const long long k_st = shape->k_stride_t ? shape->k_stride_t : pb.d;
    if (q_st < pb.d || k_st < pb.d || q_sh < 0 || k_sh < 0) return STREAM_EINVAL;
    // 16-byte vector loads: base pointers and strides must keep rows 16-byte aligned
    if (((uintptr_t)Q | (uintptr_t)K) & 15) return STREAM_EINVAL;
    if ((q_sh * pb.esize | q_st * pb.esize | k_sh * pb.esize | k_st * pb.esize) & 15) return STREAM_EINVAL;
    // the kernels address a query block's rows with 32-bit offsets from the block's first row
    if (q_st * pb.esize * 128 >= (1LL << 31)) return STREAM_EUNSUPPORTED;
    const bool wide = pb.kmax > kMaxTopk;       // more than one node per lane: the LDS-list kernel
    if (wide && !level_wide_supported(pb)) return STREAM_EUNSUPPORTED;
    int wpr = 1;
    level_fn fn = wide ? nullptr : pick_level_kernel(pb, multi, wpr);
    if (!wide && !fn) return STREAM_EUNSUPPORTED;
    const PruneWorkspace w = prune_layout(pb);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < w.total) return STREAM_EWORKSPACE;
    hipStream_t st = (hipStream_t)hip_stream;
    char *ws = (char *)workspace;

    // the refinement kernels multiply bf16 tiles with 16x16x32 MFMAs and read K fragments of 16 keys
    stream_status rc = launch_pack(K, k_sh, k_st, ws + w.kp, pb, st,
                                   pb.dtype == STREAM_BF16 ? kPackFrag16 : kPackFrag32);
    if (rc != STREAM_OK) return rc;
    if (pb.mask == STREAM_MASK_ARRAY) {
        rc = launch_block_bitmaps(pb, (unsigned *)(ws + w.cany), (unsigned *)(ws + w.call), st);
        if (rc != STREAM_OK) return rc;
    }

    PruneParams p;
    p.Q = (const char *)Q;
    p.Kp = ws + w.kp;
    p.q_sh_b = q_sh * pb.esize;
    p.q_st_b = q_st * pb.esize;
    p.H = pb.H; p.g = pb.g; p.NB = pb.NB; p.kmax = pb.kmax;
    p.nf = (int *)(ws + w.nf); p.nl = (int *)(ws + w.nl);
    p.ns = (float *)(ws + w.ns); p.ncnt = (int *)(ws + w.ncnt);
    p.idx = idx; p.cnt = cnt; p.score = score;
    p.tiles = diag ? diag->tiles_scored : nullptr;
    p.trace = diag ? diag->trace : nullptr;
    p.seqs = pb.seqs;
    p.mask = pb.mask; p.window = pb.window;
    p.cbits = pb.cbits; p.cpitch = pb.cpitch;
    p.cany = (const unsigned *)(ws + w.cany); p.call = (const unsigned *)(ws + w.call);
    p.cw = pb.mask == STREAM_MASK_ARRAY ? block_bitmap_words(pb) : 0;
    p.max_levels = pb.max_levels;
    p.vk_num = vk.num; p.vk_den = vk.den; p.vk_min = vk.kmin;
    p.n_k = multi ? n_k : 1;
    for (int i = 0; i < kMaxSweep; ++i) p.klist[i] = multi && i < n_k ? topk_list[i] : 0;
    p.wide_ki = 0;
    if (wide) {
        // every row runs all its levels in one launch (levels_per_launch does not apply); a sweep
        // runs one launch per value of k, every sequence with that k
        void *const *evw = diag ? diag->level_events : nullptr;
        p.level_begin = 1;
        if (evw && hipEventRecord((hipEvent_t)evw[0], st) != hipSuccess) return STREAM_EDEVICE;
        for (int ki = 0; ki < p.n_k; ++ki) {
            p.wide_ki = ki;
            if (multi)
                for (int sidx = 0; sidx < p.seqs.n; ++sidx) {
                    SeqDesc &sd = p.seqs.d[sidx];
                    sd.k = topk_list[ki];
                    sd.levels = levels_for((int)((long long)sd.nblk * pb.b / pb.bk), sd.k);
                }
            p.level_end = pb.max_levels;
            rc = launch_level_wide(pb, p, st);
            if (rc != STREAM_OK) return rc;
        }
        if (evw && hipEventRecord((hipEvent_t)evw[1], st) != hipSuccess) return STREAM_EDEVICE;
        return STREAM_OK;
    }
    const long long rows_per_kv = (long long)pb.NB * pb.g;
    const long long per_kv = wpr == 1 ? (rows_per_kv + 3) / 4 : rows_per_kv;
    if (per_kv * pb.Hkv + 64 > 0x7fffffffLL) return STREAM_EUNSUPPORTED;
    p.map = make_wg_map(pb.Hkv, (int)per_kv);
    // levels per launch: every row runs that many of its levels back to back inside one kernel
    // (a sweep always runs whole rows)
    int per_launch = !multi && diag && diag->levels_per_launch > 0 ? diag->levels_per_launch : kDefaultLevelsPerLaunch;
    void *const *ev = diag ? diag->level_events : nullptr;
    int launch = 0;
    for (int level = 1; level <= pb.max_levels; level += per_launch, ++launch) {
        p.level_begin = level;
        p.level_end = level + per_launch - 1 < pb.max_levels ? level + per_launch - 1 : pb.max_levels;
        if (ev && hipEventRecord((hipEvent_t)ev[2 * launch], st) != hipSuccess) return STREAM_EDEVICE;
        hipLaunchKernelGGL(fn, dim3((unsigned)p.map.grid), dim3(256), 0, st, p);
        if (hipGetLastError() != hipSuccess) return STREAM_EDEVICE;
        if (ev && hipEventRecord((hipEvent_t)ev[2 * launch + 1], st) != hipSuccess) return STREAM_EDEVICE;
    }
    return STREAM_OK;
}

extern "C" {

size_t stream_prune_workspace_bytes(const stream_shape *shape, int topk_max)
{
    Problem pb;
    if (topk_max < 1) return 0;
    if (make_problem(shape, topk_max, nullptr, topk_max, &pb) != STREAM_OK) return 0;
    return prune_layout(pb).total;
}

stream_status stream_prune(const void *Q, const void *K, const stream_shape *shape,
                           int topk, const int *topk_per_seq, int topk_max,
                           int *idx, int *cnt, float *score, const stream_prune_diag *diag,
                           void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!Q || !K || !shape || !idx || !cnt) return STREAM_EINVAL;
    if (topk_max < 1) return STREAM_EINVAL;
    Problem pb;
    stream_status rc = make_problem(shape, topk, topk_per_seq, topk_max, &pb);
    if (rc != STREAM_OK) return rc;
    return run_prune(Q, K, shape, pb, nullptr, 0, VariableK{0, 0, 0}, idx, cnt, score, diag, workspace,
                     workspace_bytes, hip_stream);
}

stream_status stream_prune_static(const void *Q, const void *K, const stream_shape *shape,
                                  int topk, const int *topk_per_seq, int topk_max,
                                  int *idx, int *cnt, float *score, const stream_prune_diag *diag,
                                  void *hip_stream)
{
    if (!Q || !K || !shape || !idx || !cnt) return STREAM_EINVAL;
    if (topk_max < 1) return STREAM_EINVAL;
    Problem pb;
    stream_status rc = make_problem(shape, topk, topk_per_seq, topk_max, &pb);
    if (rc != STREAM_OK) return rc;
    if (prune_layout(pb).total > (size_t)STREAM_STATIC_SCRATCH_BYTES) return STREAM_EWORKSPACE;
    void *ws = scratch_of_current_device();
    if (!ws) return STREAM_EDEVICE;
    // (nothing in the scratch has to start at zero: the packer rewrites every tile the kernels
    // read, node lists and bitmaps are written before they are read)
    return run_prune(Q, K, shape, pb, nullptr, 0, VariableK{0, 0, 0}, idx, cnt, score, diag, ws,
                     (size_t)STREAM_STATIC_SCRATCH_BYTES, hip_stream);
}

size_t stream_prune_multi_workspace_bytes(const stream_shape *shape, int n_k, int topk_max)
{
    if (n_k < 1 || n_k > kMaxSweep) return 0;
    return stream_prune_workspace_bytes(shape, topk_max);
}

stream_status stream_prune_multi(const void *Q, const void *K, const stream_shape *shape,
                                 const int *topk_list, int n_k, int topk_max,
                                 int *idx, int *cnt, float *score, const stream_prune_diag *diag,
                                 void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!Q || !K || !shape || !idx || !cnt || !topk_list) return STREAM_EINVAL;
    if (topk_max < 1 || n_k < 1) return STREAM_EINVAL;
    if (n_k > kMaxSweep) return STREAM_EUNSUPPORTED;
    int kmin = topk_list[0];
    for (int i = 0; i < n_k; ++i) {
        if (topk_list[i] < 1 || topk_list[i] > topk_max) return STREAM_EINVAL;
        if (topk_list[i] < kmin) kmin = topk_list[i];
    }
    // the smallest k has the deepest rows: it fixes the number of levels (and the trace length)
    Problem pb;
    stream_status rc = make_problem(shape, kmin, nullptr, topk_max, &pb);
    if (rc != STREAM_OK) return rc;
    return run_prune(Q, K, shape, pb, topk_list, n_k, VariableK{0, 0, 0}, idx, cnt, score, diag, workspace,
                     workspace_bytes, hip_stream);
}

stream_status stream_prune_variable(const void *Q, const void *K, const stream_shape *shape,
                                    int keep_num, int keep_den, int topk_min, int topk_max,
                                    int *idx, int *cnt, float *score, const stream_prune_diag *diag,
                                    void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!Q || !K || !shape || !idx || !cnt) return STREAM_EINVAL;
    if (keep_num < 1 || keep_den < 1 || keep_num > keep_den) return STREAM_EINVAL;
    if (topk_min < 1 || topk_max < topk_min) return STREAM_EINVAL;
    // the rows with the smallest k are the deepest: they fix the number of levels
    Problem pb;
    stream_status rc = make_problem(shape, topk_min, nullptr, topk_max, &pb);
    if (rc != STREAM_OK) return rc;
    return run_prune(Q, K, shape, pb, nullptr, 0, VariableK{keep_num, keep_den, topk_min}, idx, cnt, score,
                     diag, workspace, workspace_bytes, hip_stream);
}

}  // extern "C"
