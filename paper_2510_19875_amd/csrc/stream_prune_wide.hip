// stream_prune for more than 64 blocks kept per row (up to 512): Algorithm 2 ("Stream",
// Appendix C) with the row's node list in LDS instead of one node per lane.
//
// A wavefront owns one (query head, query block) row and runs all its levels in one launch, as
// the narrow kernel does; every step that the narrow kernel does once across the 64 lanes is done
// here in chunks of 64 nodes (split, list of blocks to score) or 64 branch positions (scores,
// threshold search, compaction).  The tile loop is the narrow kernel's.  Large k means few levels
// and hundreds of tiles per level, so the chunked bookkeeping is a small part of a row.
// ARB: the mask C is an explicit bit array, handled as in the narrow kernel (representatives from
// the block-level summary, token-level test against the array where a block is not wholly
// visible).  A sweep over k runs one launch per value (no score cache).
#include "stream_prune.h"

namespace stream {

// LDS per wavefront, in 4-byte words per kept block: two node lists (first, last, score) that
// swap roles at every level, the blocks to score and their scores, and per branch position the
// score's source / sort key and the representative block.
constexpr int kWideWordsPerK = 6 + 2 + 2 + 2 + 2;

__device__ __forceinline__ float key_to_score(unsigned u)
{
    // inverse of sortable_bits
    return __builtin_bit_cast(float, (u & 0x80000000u) ? (u & 0x7fffffffu) : ~u);
}

// KH: a key block is scored in KH pieces of 32 * NG keys each (128 x 128 blocks: two pieces of 64
// keys, the accumulators of a 128 x 128 tile do not fit one wavefront), the block's score being the
// maximum over the pieces.
template <bool BF16, int D, int MB, int NG, int KH, int OCC, bool ARB>
__global__ void __launch_bounds__(128, OCC) level_wide_kernel(const PruneParams p)
{
    constexpr int ES = BF16 ? 2 : 4;
    constexpr int FR = D * ES / 32;
    constexpr int BQ = 32 * MB, BK = 32 * NG * KH;
    constexpr long long TILE_BYTES = (long long)BK * D * ES;
    // bf16: 16x16x32 MFMAs on fragments of 16 rows x 64 bytes, as in the narrow kernel
    constexpr bool S16 = BF16;
    constexpr int RG = S16 ? 2 * MB : MB;                 // row groups of the Q tile (16 or 32 rows each)
    constexpr int CG = S16 ? 2 * NG : NG;                 // key groups of a piece of the K tile
    constexpr int KF = S16 ? D / 32 : FR;                 // fragments of a group along the contraction axis
    constexpr int GR = S16 ? 16 : 32;
    constexpr int AE = S16 ? 4 : 16;
    typedef float acc_t __attribute__((ext_vector_type(AE)));
    extern __shared__ __align__(16) int smem[];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    int kvh, slot;
    if (!wg_decode(p.map, blockIdx.x, kvh, slot)) return;
    const long long rows_per_kv = (long long)p.NB * p.g;
    const long long rk = (long long)slot * 2 + wave;
    if (rk >= rows_per_kv) return;
    const int gb = p.NB - 1 - (int)(rk / p.g);            // long rows first
    const int h = kvh * p.g + (int)(rk % p.g);
    const SeqDesc sd = p.seqs.d[seq_of_block(p.seqs, gb)];
    const int q = gb - sd.blk0, L = sd.len;
    const int N = sd.nblk * BQ / BK;                      // key blocks of the sequence
    const int KM = p.kmax;
    int k = sd.k, levels = sd.levels;
    const int rmin = mask_rmin(p.mask, p.window, q, BQ, BK), rmax = mask_rmax(p.mask, q, BQ, BK, L);
    // ARB: the block-level summaries of this query block (any pair visible / every pair visible)
    const unsigned *anyrow = ARB ? p.cany + (long long)gb * p.cw : nullptr;
    const unsigned *allrow = ARB ? p.call + (long long)gb * p.cw : nullptr;
    if (p.vk_den > 0) {
        int valid = rmax - rmin + 1;
        if constexpr (ARB) {
            valid = 0;
            for (int w = 0; w < p.cw; ++w) valid += __popc(anyrow[w]);
        }
        k = variable_k(valid, p.vk_num, p.vk_den, p.vk_min, p.kmax);
        levels = levels_for(N, k);
    }
    // ARB: first key block of [a, b] that C^blk leaves to this row, or -1
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

    // this wavefront's LDS arrays
    int *base = smem + wave * (kWideWordsPerK * KM);
    int *nfb[2] = {base, base + KM};
    int *nlb[2] = {base + 2 * KM, base + 3 * KM};
    float *nsb[2] = {(float *)(base + 4 * KM), (float *)(base + 5 * KM)};
    int *s_rep = base + 6 * KM;                           // [2 KM] blocks to score
    float *s_sc = (float *)(base + 8 * KM);               // [2 KM] their scores
    unsigned *s_key = (unsigned *)(base + 10 * KM);       // [2 KM] per branch position: source, then sort key
    int *s_brep = base + 12 * KM;                         // [2 KM] per branch position: representative

    // ---- Q tile of this row as A-operand fragments (as in the narrow kernel)
    uint4 qf[RG][KF];
    {
        const int mrow = S16 ? (lane & 15) : (lane & 31), gh = S16 ? (lane >> 4) : (lane >> 5);
        constexpr int SLICE = S16 ? 64 : 32;
        // (resource from the row's first query on, 64-bit base: see the narrow kernel)
        const int qrow0 = q * BQ;
        const int qrows = L - qrow0 < 32 * MB ? L - qrow0 : 32 * MB;
        const __amdgpu_buffer_rsrc_t qrs = make_tile_rsrc(
            p.Q + (long long)h * p.q_sh_b + (sd.tok0 + qrow0) * p.q_st_b,
            qrows > 0 ? (unsigned)((long long)(qrows - 1) * p.q_st_b + D * ES) : 0u);
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
    const __amdgpu_buffer_rsrc_t krs = make_tile_rsrc(
        p.Kp + ((long long)kvh * p.NB + sd.blk0) * BQ * D * ES, (unsigned)((long long)N * TILE_BYTES));
    const unsigned lane_off = lane * 16;
    const bool tail_row = (q + 1) * BQ > L;
    const int qtok0 = q * BQ;
    const int edge_num = q * BQ + BQ - 1 - p.window;
    const int edge_hi = p.mask == STREAM_MASK_SLIDING && edge_num >= 0 ? edge_num / BK : -1;
    const unsigned long long lt = (1ull << lane) - 1ull;
    const long long row = ((long long)h * p.n_k + p.wide_ki) * p.NB + gb;   // n_k > 1: one launch per k of a sweep
    const long long o = row * p.kmax;

    // ---- node init line of Alg. 2: the non-empty ranges of the equal split, in order
    int cnt = 0;
    for (int c0 = 0; c0 < k; c0 += 64) {
        const int j = c0 + lane;
        const int f = (int)(((long long)j * N) / k);
        const int l = (int)(((long long)(j + 1) * N) / k) - 1;
        const bool live = j < k && f <= l;
        const unsigned long long b = __ballot(live);
        const int pos = cnt + __popcll(b & lt);
        if (live) { nfb[0][pos] = f; nlb[0][pos] = l; nsb[0][pos] = -INFINITY; }
        cnt += __popcll(b);
    }
    wave_sync();

    // The Q tile has to be there before the first MFMA anyway; waiting for it here, once, lets
    // the waits inside the tile loop count K fragments only (vmcnt(0), other counters untouched).
    __builtin_amdgcn_s_waitcnt(0x0F70);
    unsigned long long tiles_done = 0;
    for (int level = 1; level <= levels; ++level) {
        const bool first = level == 1;
        const int cur = (level - 1) & 1, nxt_buf = cur ^ 1;
        const int *nf = nfb[cur], *nl = nlb[cur];
        const float *ns = nsb[cur];

        // ---- split every node, find the children's representatives, list the blocks to score.
        //      Per branch position: -2 = not valid, -1 = inherits the node's score, >= 0 = index
        //      of its block in the list.
        int nt = 0;
        for (int c0 = 0; c0 < cnt; c0 += 64) {
            const int j = c0 + lane;
            const bool live = j < cnt;
            const int f = live ? nf[j] : 0, l = live ? nl[j] : -1;
            const int m = (f + l + 1) >> 1;
            int rep_p = f > rmin ? f : rmin;
            int rep0 = rep_p;
            int rep1 = m > rmin ? m : rmin;
            bool v0 = live && m > f && rep0 <= (m - 1 < rmax ? m - 1 : rmax);
            bool v1 = live && rep1 <= (l < rmax ? l : rmax);
            if constexpr (ARB) {
                rep0 = live ? first_valid(f, m - 1) : -1;
                rep1 = live ? first_valid(m, l) : -1;
                v0 = rep0 >= 0;
                v1 = rep1 >= 0;
                rep_p = v0 ? rep0 : rep1;                     // the node's first valid block
            }
            const bool need0 = v0 && first;
            const bool need1 = v1 && (first || rep1 != rep_p);
            const unsigned long long b0 = __ballot(need0), b1 = __ballot(need1);
            const int pos0 = nt + __popcll(b0 & lt), pos1 = nt + __popcll(b0) + __popcll(b1 & lt);
            if (need0) s_rep[pos0] = rep0;
            if (need1) s_rep[pos1] = rep1;
            if (live) {
                s_key[2 * j] = (unsigned)(v0 ? (need0 ? pos0 : -1) : -2);
                s_key[2 * j + 1] = (unsigned)(v1 ? (need1 ? pos1 : -1) : -2);
                s_brep[2 * j] = rep0;
                s_brep[2 * j + 1] = rep1;
            }
            nt += __popcll(b0) + __popcll(b1);
        }
        wave_sync();

        // ---- score the listed blocks (the narrow kernel's tile loop)
        uint4 kf[CG][KF];
        if (nt > 0) {
            const int r0 = __builtin_amdgcn_readfirstlane(s_rep[0]);
#pragma unroll
            for (int fr = 0; fr < KF; ++fr)
#pragma unroll
                for (int cb = 0; cb < CG; ++cb) {
                    kf[cb][fr] = load_frag(krs, lane_off, (unsigned)r0 * (unsigned)TILE_BYTES, cb * KF + fr);
                    __builtin_amdgcn_sched_barrier(0);
                }
        }
        float mx_block = -INFINITY;
        for (int u = 0; u < nt * KH; ++u) {
            const int t = u / KH, piece = u % KH;
            const int r = __builtin_amdgcn_readfirstlane(s_rep[t]);
            const int un = u + 1 < nt * KH ? u + 1 : u;
            const unsigned nxt = (unsigned)__builtin_amdgcn_readfirstlane(s_rep[un / KH]) * (unsigned)TILE_BYTES;
            const int nxt_frag = (un % KH) * NG * FR;
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
                    __builtin_amdgcn_sched_barrier(0);
                    kf[cb][fr] = load_frag(krs, lane_off, nxt, nxt_frag + cb * KF + fr);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            float mx = -INFINITY;
            bool cut = tail_row || (p.mask != STREAM_MASK_FULL && (r + 1) * BK - 1 > q * BQ) ||
                       r <= edge_hi || (r + 1) * BK > L;
            if constexpr (ARB) cut = !((allrow[r >> 5] >> (r & 31)) & 1u);
            if (!cut) {
#pragma unroll
                for (int rb = 0; rb < RG; ++rb)
#pragma unroll
                    for (int cb = 0; cb < CG; ++cb)
#pragma unroll
                        for (int i = 0; i < AE; ++i) mx = fmaxf(mx, acc[rb][cb][i]);
            } else {
                const int ktok0 = r * BK + piece * 32 * NG;
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
                            // row of the Q tile and key of the piece this accumulator element belongs to
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
            mx = wave_max(mx);
            mx_block = piece == 0 ? mx : fmaxf(mx_block, mx);
            if (lane == 0 && piece == KH - 1) s_sc[t] = mx_block;
        }
        tiles_done += (unsigned long long)nt;
        wave_sync();

        // ---- per branch position: its score as an order-preserving integer key (0 = not a candidate)
        const int npos = 2 * cnt;
        int n_valid = 0;
        for (int c0 = 0; c0 < npos; c0 += 64) {
            const int pp = c0 + lane;
            unsigned key = 0;
            if (pp < npos) {
                const int src = (int)s_key[pp];
                if (src != -2) {
                    const float s = src >= 0 ? s_sc[src] : ns[pp >> 1];
                    const unsigned bts = sortable_bits(s);
                    key = bts ? bts : 1u;
                }
                s_key[pp] = key;
            }
            n_valid += __popcll(__ballot(key != 0));
        }
        wave_sync();

        // ---- the k-th largest key: threshold search over the bits, counts summed over the chunks
        unsigned thr = 1;            // n_valid <= k: every candidate is kept (keys are >= 1)
        int need_eq = 0x7fffffff;    // candidates equal to the threshold that are kept (in position order)
        bool strict_only = false;    // keep only key > thr plus need_eq of the equal ones
        if (n_valid > k) {
            thr = 0;
            bool exact = false;
            for (int bit = 31; bit >= 0 && !exact; --bit) {
                const unsigned t = thr | (1u << bit);
                int ge = 0;
                for (int c0 = 0; c0 < npos; c0 += 64) {
                    const int pp = c0 + lane;
                    const unsigned key = pp < npos ? s_key[pp] : 0u;
                    ge += __popcll(__ballot(key >= t));
                }
                if (ge >= k) {
                    thr = t;
                    exact = ge == k;
                }
            }
            if (!exact) {
                int n_gt = 0;
                for (int c0 = 0; c0 < npos; c0 += 64) {
                    const int pp = c0 + lane;
                    const unsigned key = pp < npos ? s_key[pp] : 0u;
                    n_gt += __popcll(__ballot(key > thr));
                }
                need_eq = k - n_gt;
                strict_only = true;
            }
        }

        // ---- update: survivors, in position order, become the next level's nodes
        int *nfo = nfb[nxt_buf], *nlo = nlb[nxt_buf];
        float *nso = nsb[nxt_buf];
        int out_base = 0, eq_seen = 0;
        const bool last = level == levels;
        int *tr = p.trace ? p.trace + (((long long)(level - 1) * p.H * p.n_k * p.NB + row) * p.kmax) * 2 : nullptr;
        for (int c0 = 0; c0 < npos; c0 += 64) {
            const int pp = c0 + lane;
            const unsigned key = pp < npos ? s_key[pp] : 0u;
            bool keep;
            if (strict_only) {
                const bool eq = key == thr;
                const unsigned long long be = __ballot(eq);
                keep = key > thr || (eq && eq_seen + __popcll(be & lt) < need_eq);
                eq_seen += __popcll(be);
            } else {
                keep = key >= thr;
            }
            const unsigned long long bk = __ballot(keep);
            const int out = out_base + __popcll(bk & lt);
            if (keep) {
                const int j = pp >> 1;
                const int f = nf[j], l = nl[j];
                const int m = (f + l + 1) >> 1;
                const int cf = (pp & 1) ? m : f, cl = (pp & 1) ? l : m - 1;
                const float s = key_to_score(key);
                nfo[out] = cf; nlo[out] = cl; nso[out] = s;
                if (tr) { tr[2 * out] = cf; tr[2 * out + 1] = cl; }
                if (last) {
                    p.idx[o + out] = s_brep[pp];
                    if (p.score) p.score[o + out] = s;
                }
            }
            out_base += __popcll(bk);
        }
        const int newcnt = out_base;
        if (tr)
            for (int j = newcnt + lane; j < p.kmax; j += 64) { tr[2 * j] = -1; tr[2 * j + 1] = -1; }
        if (last) {
            for (int j = newcnt + lane; j < p.kmax; j += 64) {
                p.idx[o + j] = -1;
                if (p.score) p.score[o + j] = -INFINITY;
            }
            if (lane == 0) p.cnt[row] = newcnt;
        }
        wave_sync();
        cnt = newcnt;
        // rows that finish before the deepest one: their node list stays as it is
        if (last && p.trace)
            for (int lv = level + 1; lv <= p.max_levels; ++lv) {
                int *t2 = p.trace + (((long long)(lv - 1) * p.H * p.n_k * p.NB + row) * p.kmax) * 2;
                for (int j = lane; j < p.kmax; j += 64) {
                    const bool lv_live = j < cnt;
                    t2[2 * j] = lv_live ? nfb[nxt_buf][j] : -1;
                    t2[2 * j + 1] = lv_live ? nlb[nxt_buf][j] : -1;
                }
            }
    }
    if (p.tiles && lane == 0) atomicAdd(p.tiles, tiles_done);
}

typedef void (*wide_fn)(const PruneParams);

template <bool BF16, int D, bool ARB>
static wide_fn pick_wide(int bq, int bk)
{
    constexpr int OCC2 = (BF16 || D == 64) ? 2 : 1;
    constexpr bool BIG = BF16 || D == 64;
    const int mb = bq / 32, ng = bk / 32;
    if (mb == 1 && ng == 1) return level_wide_kernel<BF16, D, 1, 1, 1, 2, ARB>;
    if (mb == 2 && ng == 2) return level_wide_kernel<BF16, D, 2, 2, 1, OCC2, ARB>;
    if (mb == 1 && ng == 2) return level_wide_kernel<BF16, D, 1, 2, 1, OCC2, ARB>;
    if (mb == 2 && ng == 1) return level_wide_kernel<BF16, D, 2, 1, 1, OCC2, ARB>;
    if (mb == 1 && ng == 4) return level_wide_kernel<BF16, D, 1, 4, 1, 1, ARB>;
    if (mb == 4 && ng == 1) return level_wide_kernel<BF16, D, 4, 1, 1, 1, ARB>;
    if constexpr (BIG) {
        if (mb == 2 && ng == 4) return level_wide_kernel<BF16, D, 2, 4, 1, 1, ARB>;
        if (mb == 4 && ng == 2) return level_wide_kernel<BF16, D, 4, 2, 1, 1, ARB>;
        if (mb == 4 && ng == 4) return level_wide_kernel<BF16, D, 4, 2, 2, 1, ARB>;   // two pieces of 64 keys
    }
    return nullptr;     // fp32 with d = 128: the 128-row tiles do not fit
}

template <bool ARB>
static wide_fn pick_wide_mask(const Problem &pb)
{
    return pb.dtype == STREAM_BF16
               ? (pb.d == 128 ? pick_wide<true, 128, ARB>(pb.b, pb.bk) : pick_wide<true, 64, ARB>(pb.b, pb.bk))
               : (pb.d == 128 ? pick_wide<false, 128, ARB>(pb.b, pb.bk) : pick_wide<false, 64, ARB>(pb.b, pb.bk));
}

static wide_fn pick_wide_kernel(const Problem &pb)
{
    if (pb.kmax > kWideTopk) return nullptr;
    return pb.mask == STREAM_MASK_ARRAY ? pick_wide_mask<true>(pb) : pick_wide_mask<false>(pb);
}

bool level_wide_supported(const Problem &pb) { return pick_wide_kernel(pb) != nullptr; }

stream_status launch_level_wide(const Problem &pb, const PruneParams &p_in, hipStream_t st)
{
    wide_fn fn = pick_wide_kernel(pb);
    if (!fn) return STREAM_EUNSUPPORTED;
    PruneParams p = p_in;
    const long long rows_per_kv = (long long)pb.NB * pb.g;
    const long long per_kv = (rows_per_kv + 1) / 2;                  // two rows (wavefronts) per workgroup
    if (per_kv * pb.Hkv + 64 > 0x7fffffffLL) return STREAM_EUNSUPPORTED;
    p.map = make_wg_map(pb.Hkv, (int)per_kv);
    const size_t lds = (size_t)2 * kWideWordsPerK * pb.kmax * 4;     // <= 57,344 bytes at k = 512
    hipLaunchKernelGGL(fn, dim3((unsigned)p.map.grid), dim3(128), lds, st, p);
    return hipGetLastError() == hipSuccess ? STREAM_OK : STREAM_EDEVICE;
}

}  // namespace stream
