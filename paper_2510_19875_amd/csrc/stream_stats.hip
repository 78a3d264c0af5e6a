// stream_receiver_stats: block means of a head's dense attention pattern and their vertical
// kurtosis (Section 4.1, "Thought Anchors": receiver heads) on gfx950.
//
// The T x T probability matrix is never stored.  Two passes over 32x32 MFMA tiles S^T = K Q^T
// (a lane owns a query column), both on operands packed into 1 KiB MFMA fragments:
//   rows     a wavefront owns up to 64 queries, keeps their Q fragments in registers, streams
//            the visible 64-key tiles and keeps a running (max, sum) per query: the
//            log-sum-exp of every row of the pattern;
//   columns  a wavefront owns one key block, keeps its K fragments in registers, streams the
//            query tiles that can see it, turns scores into probabilities with the rows'
//            log-sum-exp, reduces each b x b span to its mean and adds the means' powers, in fp64
//            and shifted by the column's first value, to the column's four power sums.
// A third, tiny kernel reduces the column statistics to the two numbers per (head, sequence).
#include "stream_mfma.h"

#include <math.h>

namespace stream {

struct StatsParams {
    const char *Qp, *Kp;        // packed fragments: [heads | kv_heads][global block][b * d]
    float *lse2;                // [heads, NB * b]: log2-domain log-sum-exp per (padded) query
    float *block_mean;          // nullable [heads, NB, NBk]
    float *col_mean, *col_kurt; // [heads, NBk]
    float *head_stats;          // [heads, batch, 2]
    float c;                    // scale * log2(e)
    int H, g, NB, b;            // NB query blocks of b = b_q tokens
    int NBk, bk;                // NBk key blocks of b_k tokens (NB * b = NBk * bk padded tokens)
    int mask, window;
    // STREAM_MASK_ARRAY (ARB kernels): the bit array C, the "some pair visible" summary per (query
    // block, key block), and the number of query blocks every column is defined on
    const unsigned *cbits, *cany;
    long long cpitch;
    int cw;
    int *col_n;                 // [heads, NBk]
    WgMap map;
    SeqTable seqs;
};
static_assert(sizeof(StatsParams) <= 4096, "kernel arguments are limited to 4 KB");

// Query blocks (of bq tokens) that can see key block j (of bk tokens) of a sequence of L tokens:
// imin .. imax, contiguous for all three mask rules (the counterpart of mask_rmin / mask_rmax);
// imin > imax for a key block of padding only.
__host__ __device__ __forceinline__ void mask_irange(int mask, int window, int j, int bq, int bk, int L,
                                                     int &imin, int &imax)
{
    const long long k_first = (long long)j * bk;
    if (k_first >= L) { imin = 0; imax = -1; return; }
    // causal rules: the first query block whose last query is at or after the block's first key
    imin = mask == STREAM_MASK_FULL ? 0 : (int)(k_first / bq);
    long long hi = ((long long)L - 1) / bq;                       // last query block with a real token
    if (mask == STREAM_MASK_SLIDING) {
        // the block's last key, j*bk + bk - 1, is seen by queries < j*bk + bk - 1 + window
        const long long w = (k_first + bk + window - 2) / bq;
        hi = w < hi ? w : hi;
    }
    imax = (int)hi;
}

// Sequence that owns global key block gk (key blocks are counted like query blocks, per sequence).
__device__ __forceinline__ int seq_of_key_block(const SeqTable &t, int gk, int bq, int bk)
{
    int s = 0;
    while (s + 1 < t.n && gk >= (int)((long long)t.d[s + 1].blk0 * bq / bk)) ++s;
    return s;
}

// ---------------------------------------------------------------------------------------------
// rows: log-sum-exp of every query.  NS = 32-query groups per wavefront (1 for block 32).
// ---------------------------------------------------------------------------------------------
// ARB: the mask is an explicit bit array: every 64-key tile of the sequence is visited and every
// element takes its bit (a lane owns a query: one mask word per 32 keys).  A query that sees no key
// gets lse = -inf, and with it a zero row of probabilities in the column pass.
template <bool BF16, int D, int NS, int OCC, bool ARB>
__global__ void __launch_bounds__(256, OCC) stats_rows_kernel(const StatsParams p)
{
    constexpr int ES = BF16 ? 2 : 4;
    constexpr int FR = D * ES / 32;                 // fragments per 32-token group
    constexpr int GROUP_BYTES = 32 * D * ES;
    constexpr int QT = 32 * NS;                     // queries of this wavefront
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    int kvh, slot;
    if (!wg_decode(p.map, blockIdx.x, kvh, slot)) return;
    const int subs = p.b / QT;                      // query tiles per block
    const long long items_per_kv = (long long)p.NB * subs * p.g;
    const long long rk = (long long)slot * 4 + wave;
    if (rk >= items_per_kv) return;
    const long long tile_id = (long long)p.NB * subs - 1 - rk / p.g;    // long rows first
    const int h = kvh * p.g + (int)(rk % p.g);
    const int gb = (int)(tile_id / subs), sub = (int)(tile_id % subs);
    const SeqDesc sd = p.seqs.d[seq_of_block(p.seqs, gb)];
    const int L = sd.len;
    const int tq0 = (gb - sd.blk0) * p.b + sub * QT;
    float *out = p.lse2 + (long long)h * p.NB * p.b + (long long)sd.blk0 * p.b + tq0;
    if (tq0 >= L) {                                 // a tile of padding only
        if (lane < QT) out[lane] = 0.f;
        return;
    }
    const unsigned lane_off = lane * 16;
    const long long seq_bytes = (long long)sd.nblk * p.b * D * ES;
    const __amdgpu_buffer_rsrc_t qrs = make_tile_rsrc(
        p.Qp + ((long long)h * p.NB + sd.blk0) * p.b * D * ES, (unsigned)seq_bytes);
    const __amdgpu_buffer_rsrc_t krs = make_tile_rsrc(
        p.Kp + ((long long)kvh * p.NB + sd.blk0) * p.b * D * ES, (unsigned)seq_bytes);

    uint4 qf[NS][FR];
#pragma unroll
    for (int qs = 0; qs < NS; ++qs)
#pragma unroll
        for (int fr = 0; fr < FR; ++fr)
            qf[qs][fr] = load_frag(qrs, lane_off, (unsigned)(tq0 / 32 + qs) * GROUP_BYTES, fr);

    // visible 64-key tiles of these queries
    const int last_q = tq0 + QT - 1 < L - 1 ? tq0 + QT - 1 : L - 1;
    const int hi_tok = p.mask == STREAM_MASK_FULL ? L - 1 : last_q;
    const int lo_tok = p.mask == STREAM_MASK_SLIDING && tq0 - p.window + 1 > 0 ? tq0 - p.window + 1 : 0;
    int kt_lo = lo_tok / 64, kt_hi = hi_tok / 64;
    if constexpr (ARB) {
        // from the first to the last key block some query of this block sees (the block summary of
        // the array): a causal or a document mask then costs its triangle, not the square
        const unsigned *anyrow = p.cany + (long long)gb * p.cw;
        const int nkb = (int)(((long long)sd.nblk * p.b) / p.bk);      // key blocks of the sequence
        int r_first = 0x7fffffff, r_last = -1;
        for (int w0 = 0; w0 * 32 < nkb; w0 += 64) {
            const int wi = w0 + lane;
            const unsigned x = wi * 32 < nkb ? anyrow[wi] : 0u;
            const unsigned long long nz = __ballot(x != 0u);
            if (nz) {
                const int wf = w0 + __builtin_ctzll(nz), wl = w0 + 63 - __builtin_clzll(nz);
                if (r_last < 0) r_first = wf * 32 + __builtin_ctz(__builtin_amdgcn_readlane(x, wf - w0));
                r_last = wl * 32 + 31 - __builtin_clz(__builtin_amdgcn_readlane(x, wl - w0));
            }
        }
        kt_lo = r_last < 0 ? 1 : (int)((long long)r_first * p.bk / 64);
        kt_hi = r_last < 0 ? 0 : (int)((((long long)r_last + 1) * p.bk - 1) / 64);
        if (kt_hi > (L - 1) / 64) kt_hi = (L - 1) / 64;
    }

    float m[NS], l[NS];
#pragma unroll
    for (int qs = 0; qs < NS; ++qs) { m[qs] = -INFINITY; l[qs] = 0.f; }

    uint4 kf[2][FR];
#pragma unroll
    for (int fr = 0; fr < FR; ++fr)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            kf[kb][fr] = load_frag(krs, lane_off, (unsigned)kt_lo * 2u * GROUP_BYTES, kb * FR + fr);
            __builtin_amdgcn_sched_barrier(0);
        }
    for (int kt = kt_lo; kt <= kt_hi; ++kt) {
        const unsigned nxt = (unsigned)(kt < kt_hi ? kt + 1 : kt) * 2u * GROUP_BYTES;
        floatx16 acc[2][NS];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int qs = 0; qs < NS; ++qs)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[kb][qs][i] = 0.f;
#pragma unroll
        for (int fr = 0; fr < FR; ++fr) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
                for (int qs = 0; qs < NS; ++qs)
                    acc[kb][qs] = mfma_frag<BF16>(kf[kb][fr], qf[qs][fr], acc[kb][qs]);
                // consumed: refill from the next tile so that it has a whole tile of MFMA time
                __builtin_amdgcn_sched_barrier(0);
                kf[kb][fr] = load_frag(krs, lane_off, nxt, kb * FR + fr);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        const int tk0 = kt * 64;
        const bool cut = ARB | (tq0 + QT > L) | (tk0 + 64 > L) |
                         ((p.mask != STREAM_MASK_FULL) & (tk0 + 63 > tq0)) |
                         ((p.mask == STREAM_MASK_SLIDING) & (tq0 + QT - 1 - tk0 >= p.window));
        // accumulator layout: lane holds query column (lane % 32); element i is key row
        // 8*(i/4) + 4*(lane/32) + (i%4)
#pragma unroll
        for (int qs = 0; qs < NS; ++qs) {
            unsigned cwd[2] = {0u, 0u};              // ARB: this lane's query against the tile's two key groups
            if constexpr (ARB) {
                const int tq = tq0 + qs * 32 + (lane & 31);
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
                    if (tq < L && tk0 + kb * 32 < L) cwd[kb] = p.cbits[(long long)tq * p.cpitch + (tk0 >> 5) + kb];
            }
            // m[] is kept on the raw products (c > 0, so the maximum commutes with the scaling):
            // per element one max, one fused multiply-add, one exp2, one add
            float x[2][16];
            float tmax = -INFINITY;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    float v = acc[kb][qs][i];
                    if (cut) {
                        const int tq = tq0 + qs * 32 + (lane & 31);
                        const int tk = tk0 + kb * 32 + (i >> 2) * 8 + (lane >> 5) * 4 + (i & 3);
                        bool vis = (tq < L) & (tk < L);
                        if constexpr (ARB) vis = vis & ((cwd[kb] >> ((i >> 2) * 8 + (lane >> 5) * 4 + (i & 3))) & 1u);
                        else vis = vis & mask_token(p.mask, p.window, tq, tk);
                        v = vis ? v : -INFINITY;
                    }
                    x[kb][i] = v;
                    tmax = fmaxf(tmax, v);
                }
            const float m_new = fmaxf(m[qs], tmax);
            const float m_ref = m_new == -INFINITY ? 0.f : m_new;
            const float mc = m_ref * p.c;
            float sum = 0.f;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int i = 0; i < 16; ++i) sum += __builtin_amdgcn_exp2f(fmaf(x[kb][i], p.c, -mc));
            l[qs] = l[qs] * __builtin_amdgcn_exp2f((m[qs] - m_ref) * p.c) + sum;
            m[qs] = m_new;
        }
    }
    // the two lane halves hold different key rows of the same query: merge them
#pragma unroll
    for (int qs = 0; qs < NS; ++qs) {
        const float m2 = __shfl_xor(m[qs], 32), l2 = __shfl_xor(l[qs], 32);
        const float mm = fmaxf(m[qs], m2);
        const float m_ref = mm == -INFINITY ? 0.f : mm;
        const float lt = l[qs] * __builtin_amdgcn_exp2f((m[qs] - m_ref) * p.c) +
                         l2 * __builtin_amdgcn_exp2f((m2 - m_ref) * p.c);
        const int tq = tq0 + qs * 32 + (lane & 31);
        if (lane < 32) out[qs * 32 + lane] = tq < L ? m_ref * p.c + log2f(lt) : 0.f;
    }
}

// ---------------------------------------------------------------------------------------------
// columns: block means and the moments of every column.  NG = 32-key groups of a key block,
// NS = 32-query groups per streamed tile, TPB = streamed tiles per query block.
// ---------------------------------------------------------------------------------------------
// ARB: the query blocks a column is defined on come from the block summary of the array (they need
// not be contiguous: the tiles between the first and the last are all streamed, spans the array
// hides from the column are left out of its moments), and every element takes its bit.
template <bool BF16, int D, int NG, int NS, int TPB, int OCC, bool ARB>
__global__ void __launch_bounds__(256, OCC) stats_cols_kernel(const StatsParams p)
{
    constexpr int ES = BF16 ? 2 : 4;
    constexpr int FR = D * ES / 32;
    constexpr int GROUP_BYTES = 32 * D * ES;
    constexpr int BK = 32 * NG;                     // key block b_k
    constexpr int QT = 32 * NS;
    constexpr int BQ = QT * TPB;                    // query block b_q = TPB streamed tiles
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    int kvh, slot;
    if (!wg_decode(p.map, blockIdx.x, kvh, slot)) return;
    const long long items_per_kv = (long long)p.NBk * p.g;
    const long long rk = (long long)slot * 4 + wave;
    if (rk >= items_per_kv) return;
    const int gbj = (int)(rk / p.g);                // global key block; causal: early columns are the long ones
    const int h = kvh * p.g + (int)(rk % p.g);
    const SeqDesc sd = p.seqs.d[seq_of_key_block(p.seqs, gbj, BQ, BK)];
    const int L = sd.len;
    const int kblk0 = (int)((long long)sd.blk0 * BQ / BK);
    const int j = gbj - kblk0;
    const int tk0 = j * BK;
    const unsigned lane_off = lane * 16;
    const long long seq_bytes = (long long)sd.nblk * BQ * D * ES;
    const __amdgpu_buffer_rsrc_t qrs = make_tile_rsrc(
        p.Qp + ((long long)h * p.NB + sd.blk0) * BQ * D * ES, (unsigned)seq_bytes);
    const __amdgpu_buffer_rsrc_t krs = make_tile_rsrc(
        p.Kp + ((long long)kvh * p.NB + sd.blk0) * BQ * D * ES, (unsigned)seq_bytes);
    const float *lse_seq = p.lse2 + (long long)h * p.NB * BQ + (long long)sd.blk0 * BQ;

    uint4 kf[NG][FR];
#pragma unroll
    for (int kg = 0; kg < NG; ++kg)
#pragma unroll
        for (int fr = 0; fr < FR; ++fr)
            kf[kg][fr] = load_frag(krs, lane_off, (unsigned)(j * NG + kg) * GROUP_BYTES, fr);

    int imin, imax;
    mask_irange(p.mask, p.window, j, BQ, BK, L, imin, imax);
    auto span_valid = [&](int i) -> bool {          // ARB: does query block i see key block j at all?
        return (p.cany[(long long)(sd.blk0 + i) * p.cw + (gbj >> 5)] >> (gbj & 31)) & 1u;
    };
    if constexpr (ARB) {
        imin = 0x7fffffff; imax = -1;
        for (int i0 = 0; i0 < sd.nblk; i0 += 64) {
            const unsigned long long b = __ballot(i0 + lane < sd.nblk && span_valid(i0 + lane));
            if (b) {
                if (imax < 0) imin = i0 + __builtin_ctzll(b);
                imax = i0 + 63 - __builtin_clzll(b);
            }
        }
    }
    if (imin > imax) {                              // a key block of padding only (or hidden from everyone): no column
        if (lane == 0) {
            p.col_mean[(long long)h * p.NBk + gbj] = 0.f; p.col_kurt[(long long)h * p.NBk + gbj] = 0.f;
            if constexpr (ARB) p.col_n[(long long)h * p.NBk + gbj] = 0;
        }
        return;
    }
    const int nk = L - tk0 < BK ? L - tk0 : BK;     // real keys of the block
    float *bm = p.block_mean ? p.block_mean + ((long long)h * p.NB + sd.blk0) * p.NBk + gbj : nullptr;

    // power sums of the column's means, in fp64, shifted by the column's first value (the
    // diagonal block) so that the central moments formed from them at the end lose nothing that
    // matters: four short independent chains per span instead of a long dependent update
    double x0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0, s4 = 0.0;
    int n_spans = 0;                                // spans the column is defined on

    uint4 qf[NS][FR];
    float lq[NS];
    {
        const int tq0 = imin * BQ;
#pragma unroll
        for (int fr = 0; fr < FR; ++fr)
#pragma unroll
            for (int qs = 0; qs < NS; ++qs) {
                qf[qs][fr] = load_frag(qrs, lane_off, (unsigned)(tq0 / 32 + qs) * GROUP_BYTES, fr);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
        for (int qs = 0; qs < NS; ++qs) lq[qs] = lse_seq[tq0 + qs * 32 + (lane & 31)];
    }
    const int n_tiles = (imax - imin + 1) * TPB;
    float psum = 0.f;
    for (int t = 0; t < n_tiles; ++t) {
        const int tq0 = imin * BQ + t * QT;
        const int tqn = t + 1 < n_tiles ? tq0 + QT : tq0;
        const unsigned nxt = (unsigned)(tqn / 32) * GROUP_BYTES;
        floatx16 acc[NG][NS];
#pragma unroll
        for (int kg = 0; kg < NG; ++kg)
#pragma unroll
            for (int qs = 0; qs < NS; ++qs)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[kg][qs][i] = 0.f;
#pragma unroll
        for (int fr = 0; fr < FR; ++fr) {
#pragma unroll
            for (int qs = 0; qs < NS; ++qs) {
#pragma unroll
                for (int kg = 0; kg < NG; ++kg)
                    acc[kg][qs] = mfma_frag<BF16>(kf[kg][fr], qf[qs][fr], acc[kg][qs]);
                __builtin_amdgcn_sched_barrier(0);
                qf[qs][fr] = load_frag(qrs, lane_off, nxt + (unsigned)qs * GROUP_BYTES, fr);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        float lcur[NS];
#pragma unroll
        for (int qs = 0; qs < NS; ++qs) {
            lcur[qs] = lq[qs];
            lq[qs] = lse_seq[tqn + qs * 32 + (lane & 31)];
        }
        const bool cut = ARB | (tq0 + QT > L) | (tk0 + BK > L) |
                         ((p.mask != STREAM_MASK_FULL) & (tk0 + BK - 1 > tq0)) |
                         ((p.mask == STREAM_MASK_SLIDING) & (tq0 + QT - 1 - tk0 >= p.window));
        unsigned cwd[NG][NS];                        // ARB: this lane's queries against the block's key groups
        if constexpr (ARB) {
#pragma unroll
            for (int qs = 0; qs < NS; ++qs) {
                const int tq = tq0 + qs * 32 + (lane & 31);
#pragma unroll
                for (int kg = 0; kg < NG; ++kg)
                    cwd[kg][qs] = (tq < L && tk0 + kg * 32 < L) ? p.cbits[(long long)tq * p.cpitch + (tk0 >> 5) + kg] : 0u;
            }
        }
#pragma unroll
        for (int kg = 0; kg < NG; ++kg)
#pragma unroll
            for (int qs = 0; qs < NS; ++qs)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    float pr = __builtin_amdgcn_exp2f(acc[kg][qs][i] * p.c - lcur[qs]);
                    if (cut) {
                        const int tq = tq0 + qs * 32 + (lane & 31);
                        const int tk = tk0 + kg * 32 + (i >> 2) * 8 + (lane >> 5) * 4 + (i & 3);
                        bool vis = (tq < L) & (tk < L);
                        if constexpr (ARB) vis = vis & ((cwd[kg][qs] >> ((i >> 2) * 8 + (lane >> 5) * 4 + (i & 3))) & 1u);
                        else vis = vis & mask_token(p.mask, p.window, tq, tk);
                        pr = vis ? pr : 0.f;
                    }
                    psum += pr;
                }
        if ((t + 1) % TPB == 0) {
            // a b x b span is complete: its mean over the real token pairs
            const int i_blk = imin + t / TPB;
            const int nq = L - i_blk * BQ < BQ ? L - i_blk * BQ : BQ;
            const float mval = wave_sum(psum) / (float)(nq * nk);
            psum = 0.f;
            bool defined = true;
            if constexpr (ARB) defined = span_valid(i_blk);
            if (defined) {
                if (bm && lane == 0) bm[(long long)i_blk * p.NBk] = mval;
                const double x = (double)mval;
                if (n_spans == 0) x0 = x;
                const double y = x - x0, y2 = y * y;
                s1 += y;
                s2 += y2;
                s3 = fma(y2, y, s3);
                s4 = fma(y2, y2, s4);
                ++n_spans;
            }
        }
    }
    if (lane == 0) {
        const long long o = (long long)h * p.NBk + gbj;
        if constexpr (ARB) p.col_n[o] = n_spans;
        const double cn = (double)n_spans;
        const double mu = s1 / cn;                                  // mean of the shifted values
        const double m2 = s2 / cn - mu * mu;
        const double m4 = s4 / cn - 4.0 * mu * (s3 / cn) + 6.0 * mu * mu * (s2 / cn) - 3.0 * mu * mu * mu * mu;
        p.col_mean[o] = (float)(x0 + mu);
        p.col_kurt[o] = (cn >= 4.0 && m2 > 0.0) ? (float)(m4 / (m2 * m2) - 3.0) : 0.f;
    }
}

// ---------------------------------------------------------------------------------------------
// heads: one wavefront per (head, sequence) reduces the column statistics.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ double wave_sum_f64(double v)
{
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) v += __shfl_xor(v, s);
    return v;
}

__global__ void __launch_bounds__(64) stats_heads_kernel(const StatsParams p)
{
    const int lane = threadIdx.x;
    const int h = blockIdx.x / p.seqs.n, s = blockIdx.x % p.seqs.n;
    const SeqDesc sd = p.seqs.d[s];
    const int L = sd.len;
    const int N = (L + p.bk - 1) / p.bk;            // columns: the key blocks that hold a real key
    const long long kblk0 = (long long)sd.blk0 * p.b / p.bk;
    const float *cm = p.col_mean + (long long)h * p.NBk + kblk0;
    const float *ck = p.col_kurt + (long long)h * p.NBk + kblk0;
    const bool arb = p.mask == STREAM_MASK_ARRAY;
    const int *cnn = p.col_n + (long long)h * p.NBk + kblk0;     // (read with an array only)
    double s1 = 0.0;
    float mx = -INFINITY;
    int n_cols = 0;                                 // columns some query block sees
    for (int j = lane; j < N; j += 64) {
        int imin, imax;
        mask_irange(p.mask, p.window, j, p.b, p.bk, L, imin, imax);
        const int n = arb ? cnn[j] : imax - imin + 1;
        if (n > 0) { s1 += (double)cm[j]; ++n_cols; }
        if (n >= 4) mx = fmaxf(mx, ck[j]);
    }
    for (int sft = 32; sft >= 1; sft >>= 1) n_cols += __shfl_xor(n_cols, sft);
    if (!arb) n_cols = N;
    const int Ncol = n_cols;
    const double mean = wave_sum_f64(s1) / (double)(Ncol > 0 ? Ncol : 1);
    double c2 = 0.0, c4 = 0.0;
    for (int j = lane; j < N; j += 64) {
        if (arb && cnn[j] <= 0) continue;
        const double c = (double)cm[j] - mean;
        c2 += c * c;
        c4 += c * c * c * c;
    }
    const double m2 = wave_sum_f64(c2) / (double)(Ncol > 0 ? Ncol : 1), m4 = wave_sum_f64(c4) / (double)(Ncol > 0 ? Ncol : 1);
    mx = wave_max(mx);
    if (lane == 0) {
        float *o = p.head_stats + ((long long)h * p.seqs.n + s) * 2;
        o[0] = mx == -INFINITY ? 0.f : mx;
        o[1] = (Ncol >= 4 && m2 > 0.0) ? (float)(m4 / (m2 * m2) - 3.0) : 0.f;
    }
}

__global__ void __launch_bounds__(256) stats_zero_kernel(float *p, long long n)
{
    const long long stride = (long long)gridDim.x * blockDim.x;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = 0.f;
}

struct StatsWorkspace {
    size_t qp, kp, lse2, cany, call, coln, total;
};

static StatsWorkspace stats_layout(const Problem &pb)
{
    StatsWorkspace w;
    size_t off = 0;
    w.qp = off;   off += align_up((size_t)pb.H * pb.NB * pb.b * pb.d * pb.esize, 256);
    w.kp = off;   off += align_up((size_t)pb.Hkv * pb.NB * pb.b * pb.d * pb.esize, 256);
    w.lse2 = off; off += align_up((size_t)pb.H * pb.NB * pb.b * 4, 256);
    // with a mask array: its block-level summaries and the number of spans of every column
    const bool arb = pb.mask == STREAM_MASK_ARRAY;
    const size_t bm = arb ? align_up((size_t)pb.NB * block_bitmap_words(pb) * 4, 256) : 0;
    w.cany = off; off += bm;
    w.call = off; off += bm;
    w.coln = off; off += arb ? align_up((size_t)pb.H * ((size_t)pb.NB * pb.b / pb.bk) * 4, 256) : 0;
    w.total = off;
    return w;
}

typedef void (*stats_fn)(const StatsParams);

template <bool BF16, int D, int NS, int TPB, bool ARB>
static stats_fn pick_stats_cols_bk(int bk)
{
    constexpr int OCC = (BF16 || D == 64) ? 2 : 1;   // fp32 with d = 128 holds 16 fragments per group
    if (bk == 32) return stats_cols_kernel<BF16, D, 1, NS, TPB, OCC, ARB>;
    if (bk == 64) return stats_cols_kernel<BF16, D, 2, NS, TPB, OCC, ARB>;
    if constexpr (BF16 || D == 64)
        return stats_cols_kernel<BF16, D, 4, NS, TPB, 1, ARB>;
    else
        return nullptr;                              // 128 keys of fp32 x 128 do not fit a wavefront's registers
}

template <bool BF16, int D, bool ARB>
static void pick_stats_kernels_m(int bq, int bk, stats_fn &rows, stats_fn &cols)
{
    constexpr int OCC = (BF16 || D == 64) ? 2 : 1;
    if (bq == 32) {
        rows = stats_rows_kernel<BF16, D, 1, OCC, ARB>;
        cols = pick_stats_cols_bk<BF16, D, 1, 1, ARB>(bk);
    } else if (bq == 64) {
        rows = stats_rows_kernel<BF16, D, 2, OCC, ARB>;
        cols = pick_stats_cols_bk<BF16, D, 2, 1, ARB>(bk);
    } else {
        rows = stats_rows_kernel<BF16, D, 2, OCC, ARB>;
        cols = pick_stats_cols_bk<BF16, D, 2, 2, ARB>(bk);
    }
}

template <bool BF16, int D>
static void pick_stats_kernels_t(int bq, int bk, bool arb, stats_fn &rows, stats_fn &cols)
{
    if (arb) pick_stats_kernels_m<BF16, D, true>(bq, bk, rows, cols);
    else pick_stats_kernels_m<BF16, D, false>(bq, bk, rows, cols);
}

}  // namespace stream

using namespace stream;

extern "C" {

size_t stream_receiver_stats_workspace_bytes(const stream_shape *shape)
{
    Problem pb;
    if (make_problem(shape, 0, nullptr, 0, &pb) != STREAM_OK) return 0;
    return stats_layout(pb).total;
}

stream_status stream_receiver_stats(const void *Q, const void *K, const stream_shape *shape, float scale,
                                    float *block_mean, float *col_mean, float *col_kurt,
                                    float *head_stats, void *workspace, size_t workspace_bytes,
                                    void *hip_stream)
{
    if (!Q || !K || !shape || !col_mean || !col_kurt || !head_stats) return STREAM_EINVAL;
    if (!(scale > 0.f) || !isfinite(scale)) return STREAM_EINVAL;
    Problem pb;
    stream_status rc = make_problem(shape, 0, nullptr, 0, &pb);
    if (rc != STREAM_OK) return rc;
    const long long q_sh = shape->q_stride_h ? shape->q_stride_h : pb.T * pb.d;
    const long long q_st = shape->q_stride_t ? shape->q_stride_t : pb.d;
    const long long k_sh = shape->k_stride_h ? shape->k_stride_h : pb.T * pb.d;
    const long long k_st = shape->k_stride_t ? shape->k_stride_t : pb.d;
    if (q_st < pb.d || k_st < pb.d || q_sh < 0 || k_sh < 0) return STREAM_EINVAL;
    if (((uintptr_t)Q | (uintptr_t)K) & 15) return STREAM_EINVAL;
    if ((q_sh * pb.esize | q_st * pb.esize | k_sh * pb.esize | k_st * pb.esize) & 15) return STREAM_EINVAL;
    stats_fn rows = nullptr, cols = nullptr;
    const bool arb = pb.mask == STREAM_MASK_ARRAY;
    if (pb.dtype == STREAM_BF16) {
        if (pb.d == 128) pick_stats_kernels_t<true, 128>(pb.b, pb.bk, arb, rows, cols);
        else pick_stats_kernels_t<true, 64>(pb.b, pb.bk, arb, rows, cols);
    } else {
        if (pb.d == 128) pick_stats_kernels_t<false, 128>(pb.b, pb.bk, arb, rows, cols);
        else pick_stats_kernels_t<false, 64>(pb.b, pb.bk, arb, rows, cols);
    }
    if (!rows || !cols) return STREAM_EUNSUPPORTED;
    const StatsWorkspace w = stats_layout(pb);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < w.total) return STREAM_EWORKSPACE;
    hipStream_t st = (hipStream_t)hip_stream;
    char *ws = (char *)workspace;

    // Q is packed like K: one region of tiles per query head
    Problem pq = pb;
    pq.Hkv = pb.H;
    rc = launch_pack(Q, q_sh, q_st, ws + w.qp, pq, st);
    if (rc != STREAM_OK) return rc;
    rc = launch_pack(K, k_sh, k_st, ws + w.kp, pb, st);
    if (rc != STREAM_OK) return rc;

    StatsParams p;
    p.Qp = ws + w.qp;
    p.Kp = ws + w.kp;
    p.lse2 = (float *)(ws + w.lse2);
    p.block_mean = block_mean;
    p.col_mean = col_mean; p.col_kurt = col_kurt; p.head_stats = head_stats;
    p.c = scale * 1.4426950408889634f;
    p.H = pb.H; p.g = pb.g; p.NB = pb.NB; p.b = pb.b;
    p.bk = pb.bk; p.NBk = (int)((long long)pb.NB * pb.b / pb.bk);
    p.mask = pb.mask; p.window = pb.window;
    p.cbits = pb.cbits; p.cpitch = pb.cpitch;
    p.cany = (const unsigned *)(ws + w.cany);
    p.cw = arb ? block_bitmap_words(pb) : 0;
    p.col_n = (int *)(ws + w.coln);
    p.seqs = pb.seqs;
    if (arb) {
        rc = launch_block_bitmaps(pb, (unsigned *)(ws + w.cany), (unsigned *)(ws + w.call), st);
        if (rc != STREAM_OK) return rc;
    }

    if (block_mean) {
        // entries no kernel writes (blocks the mask hides, pairs of different sequences) are zero
        const long long n = (long long)pb.H * pb.NB * p.NBk;
        const long long wgs = (n + 255) / 256;
        hipLaunchKernelGGL(stats_zero_kernel, dim3((unsigned)(wgs < 8192 ? wgs : 8192)), dim3(256), 0, st,
                           block_mean, n);
        if (hipGetLastError() != hipSuccess) return STREAM_EDEVICE;
    }

    const int qt = pb.b == 32 ? 32 : 64;
    const long long row_items = (long long)pb.NB * (pb.b / qt) * pb.g;
    const long long col_items = (long long)p.NBk * pb.g;
    if ((row_items + 3) / 4 * pb.Hkv + 64 > 0x7fffffffLL) return STREAM_EUNSUPPORTED;
    p.map = make_wg_map(pb.Hkv, (int)((row_items + 3) / 4));
    hipLaunchKernelGGL(rows, dim3((unsigned)p.map.grid), dim3(256), 0, st, p);
    if (hipGetLastError() != hipSuccess) return STREAM_EDEVICE;
    p.map = make_wg_map(pb.Hkv, (int)((col_items + 3) / 4));
    hipLaunchKernelGGL(cols, dim3((unsigned)p.map.grid), dim3(256), 0, st, p);
    if (hipGetLastError() != hipSuccess) return STREAM_EDEVICE;
    hipLaunchKernelGGL(stats_heads_kernel, dim3((unsigned)(pb.H * pb.batch)), dim3(64), 0, st, p);
    return hipGetLastError() == hipSuccess ? STREAM_OK : STREAM_EDEVICE;
}

}  // extern "C"
