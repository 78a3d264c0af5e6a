// stream_prune: Algorithm 2 ("Stream", Appendix C) on gfx950.
//
// One kernel launch per refinement level.  A wavefront owns one (query head, query block) row
// (four wavefronts share a row when block = 128): it holds the row's Q tile in registers as
// MFMA operand fragments, gathers the packed K tiles of the branches that need a new score,
// reduces each 32x32 accumulator set to the masked maximum (score line of Alg. 2 / Eq. (4)),
// ranks the 2k branch scores across its lanes, and writes the surviving nodes back in place in
// positional order.  The node lists [heads, NB, k] are the only state: O(T) memory.
#include "stream_select.h"

#include <math.h>

namespace stream {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct PruneParams {
    const char *Q;
    const char *Kp;              // packed K tiles [kv_head][global block][b * d]
    long long q_sh_b, q_st_b;    // byte strides of Q (head, token)
    int H, g, NB, kmax;
    int level;                   // 1-based refinement level of this launch
    int *nf, *nl;                // node ranges [H, NB, kmax]
    float *ns;                   // node scores (score of the node's representative block)
    int *ncnt;                   // live nodes per row [H, NB]
    int *idx, *cnt;              // outputs, written by a row's last level
    float *score;                // nullable
    unsigned long long *tiles;   // nullable diagnostic counter
    WgMap map;
    SeqTable seqs;
};

__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int CTRL>
__device__ __forceinline__ float dpp_f(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL,
                                                                 0xf, 0xf, false));
}

// Maximum over the 64 lanes, returned in every lane.
__device__ __forceinline__ float wave_max(float v)
{
    v = fmaxf(v, dpp_f<0xB1>(v));   // quad_perm [1,0,3,2]
    v = fmaxf(v, dpp_f<0x4E>(v));   // quad_perm [2,3,0,1]
    v = fmaxf(v, dpp_f<0x141>(v));  // row_half_mirror
    v = fmaxf(v, dpp_f<0x140>(v));  // row_mirror: every lane of a 16-lane row holds the row max
    const int iv = __builtin_bit_cast(int, v);
    const float a = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 0));
    const float b = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 16));
    const float c = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 32));
    const float d = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 48));
    return fmaxf(fmaxf(a, b), fmaxf(c, d));
}

// One operand fragment (16 bytes per lane) times another, accumulated into a 32x32 tile.
template <bool BF16>
__device__ __forceinline__ floatx16 mfma_frag(const uint4 &a, const uint4 &b, floatx16 c)
{
    if constexpr (BF16) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                       __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    } else {
        // fp32: the fragment's 8 contraction indices are split 4 + 4 between the lane halves;
        // step j multiplies component j of both operands (32x32x2 MFMA, 2 indices per step).
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_bit_cast(float, a.x), __builtin_bit_cast(float, b.x), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_bit_cast(float, a.y), __builtin_bit_cast(float, b.y), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_bit_cast(float, a.z), __builtin_bit_cast(float, b.z), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_bit_cast(float, a.w), __builtin_bit_cast(float, b.w), c, 0, 0, 0);
        return c;
    }
}

// Template parameters: element type, head dim, 32-row groups of Q per wavefront (MB), 32-key
// groups of K per wavefront (NG), wavefronts per row (WPR: 1, or 4 = 2 query halves x 2 key
// halves for block 128), occupancy hint.
template <bool BF16, int D, int MB, int NG, int WPR, int OCC>
__global__ void __launch_bounds__(256, OCC) level_kernel(const PruneParams p)
{
    constexpr int ES = BF16 ? 2 : 4;
    constexpr int FR = D * ES / 32;                       // fragments per 32-token group
    constexpr int B = 32 * MB * (WPR == 4 ? 2 : 1);       // block size b_q = b_k
    constexpr long long TILE_BYTES = (long long)B * D * ES;
    constexpr int GROUP_BYTES = 32 * D * ES;
    __shared__ int s_rep[4][2 * kMaxTopk];
    __shared__ float s_sc[4][2 * kMaxTopk];

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
    if (p.level > sd.levels) return;
    const int q = gb - sd.blk0, N = sd.nblk, k = sd.k, L = sd.len;
    const long long row = (long long)h * p.NB + gb;
    const bool first = p.level == 1;
    const int qh = WPR == 4 ? (wave >> 1) : 0;            // query half / key half of this wavefront
    const int kh = WPR == 4 ? (wave & 1) : 0;

    // ---- Q tile of this wavefront as A-operand fragments: lane (mrow = lane % 32, gh = lane / 32)
    //      holds, for fragment fr, the 16 bytes at chunk 2*fr + gh of row mrow.  Issued first so
    //      that the loads overlap the node-state loads below; rows past the end of the sequence
    //      fall outside the buffer resource and read as zeros.
    uint4 qf[MB][FR];
    {
        const int mrow = lane & 31, gh = lane >> 5;
        const __amdgpu_buffer_rsrc_t qrs = make_tile_rsrc(
            p.Q + (long long)h * p.q_sh_b + sd.tok0 * p.q_st_b,
            (unsigned)((long long)(L - 1) * p.q_st_b + D * ES));
#pragma unroll
        for (int rb = 0; rb < MB; ++rb) {
            const unsigned tok = (unsigned)(q * B + qh * 32 * MB + rb * 32 + mrow);
            const unsigned voff = tok * (unsigned)p.q_st_b + gh * 16;
#pragma unroll
            for (int fr = 0; fr < FR; ++fr) {
                const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(qrs, voff + fr * 32, 0, 0);
                qf[rb][fr] = make_uint4(v[0], v[1], v[2], v[3]);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }

    // ---- node of this lane (node init line of Alg. 2 at the first level)
    int f = 0, l = -1;
    float sc = -INFINITY;
    bool live = false;
    if (first) {
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
    // ---- split at the midpoint; causal validity: a branch is valid iff it is non-empty and
    //      starts at or before the query block; its representative is its first block.
    const int m = (f + l + 1) >> 1;
    const bool v0 = live && m > f && f <= q;              // left child [f, m-1]
    const bool v1 = live && m <= q;                       // right child [m, l] (never empty)
    const bool need0 = v0 && first;                       // otherwise the parent's score carries over
    const bool need1 = v1 && (first || m > f);

    const unsigned long long lt = (1ull << lane) - 1ull;
    const unsigned long long b0 = __ballot(need0), b1 = __ballot(need1);
    const int n0 = __popcll(b0), nt = n0 + __popcll(b1);
    const int pos0 = __popcll(b0 & lt), pos1 = n0 + __popcll(b1 & lt);
    if (need0) s_rep[wave][pos0] = f;
    if (need1) s_rep[wave][pos1] = m;
    wave_sync();

    // K tiles of this (kv head, sequence), from this wavefront's key half on
    const __amdgpu_buffer_rsrc_t krs = make_tile_rsrc(
        p.Kp + ((long long)kvh * p.NB + sd.blk0) * TILE_BYTES + (long long)kh * NG * GROUP_BYTES,
        (unsigned)((long long)N * TILE_BYTES - (long long)kh * NG * GROUP_BYTES));
    const unsigned lane_off = lane * 16;
    const bool tail_row = (q == N - 1) && (L % B != 0);
    const int qtok0 = q * B + qh * 32 * MB;

    uint4 kf[NG][FR];
    if (nt > 0) {
        const int r0 = __builtin_amdgcn_readfirstlane(s_rep[wave][0]);
        // same order as the refills in the loop below: waits count loads in issue order
#pragma unroll
        for (int fr = 0; fr < FR; ++fr)
#pragma unroll
            for (int cb = 0; cb < NG; ++cb) {
                kf[cb][fr] = load_frag(krs, lane_off, (unsigned)r0 * (unsigned)TILE_BYTES, cb * FR + fr);
                __builtin_amdgcn_sched_barrier(0);
            }
    }
    for (int t = 0; t < nt; ++t) {
        const int r = __builtin_amdgcn_readfirstlane(s_rep[wave][t]);
        const int tn = t + 1 < nt ? t + 1 : t;
        const unsigned nxt = (unsigned)__builtin_amdgcn_readfirstlane(s_rep[wave][tn]) * (unsigned)TILE_BYTES;
        floatx16 acc[MB][NG];
#pragma unroll
        for (int rb = 0; rb < MB; ++rb)
#pragma unroll
            for (int cb = 0; cb < NG; ++cb)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[rb][cb][i] = 0.f;
#pragma unroll
        for (int fr = 0; fr < FR; ++fr) {
#pragma unroll
            for (int cb = 0; cb < NG; ++cb) {
#pragma unroll
                for (int rb = 0; rb < MB; ++rb)
                    acc[rb][cb] = mfma_frag<BF16>(qf[rb][fr], kf[cb][fr], acc[rb][cb]);
                // the fragment is consumed: refill its registers from the next tile right here,
                // so that every fragment of the next tile has a whole tile of MFMA time to arrive
                // (the scheduling barriers stop the compiler from sinking the loads to the end)
                __builtin_amdgcn_sched_barrier(0);
                kf[cb][fr] = load_frag(krs, lane_off, nxt, cb * FR + fr);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        float mx = -INFINITY;
        if (!(r == q || tail_row)) {
#pragma unroll
            for (int rb = 0; rb < MB; ++rb)
#pragma unroll
                for (int cb = 0; cb < NG; ++cb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) mx = fmaxf(mx, acc[rb][cb][i]);
        } else {
            // diagonal block: token-level causal mask; last block of a sequence: padded rows/cols.
            // 32x32 accumulator layout: lane holds column (lane % 32); element i is row
            // 8*(i/4) + 4*(lane/32) + (i%4).
            const int ktok0 = r * B + kh * 32 * NG;
#pragma unroll
            for (int rb = 0; rb < MB; ++rb)
#pragma unroll
                for (int cb = 0; cb < NG; ++cb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int tq = qtok0 + rb * 32 + (i >> 2) * 8 + (lane >> 5) * 4 + (i & 3);
                        const int tk = ktok0 + cb * 32 + (lane & 31);
                        if (tq < L && tk <= tq) mx = fmaxf(mx, acc[rb][cb][i]);
                    }
        }
        mx = wave_max(mx);
        if (lane == 0) s_sc[wave][t] = mx;
    }
    wave_sync();
    if constexpr (WPR == 4) __syncthreads();

    auto tile_score = [&](int t) -> float {
        if constexpr (WPR == 4)
            return fmaxf(fmaxf(s_sc[0][t], s_sc[1][t]), fmaxf(s_sc[2][t], s_sc[3][t]));
        else
            return s_sc[wave][t];
    };
    float s0 = -INFINITY, s1 = -INFINITY;
    if (v0) s0 = need0 ? tile_score(pos0) : sc;
    if (v1) s1 = need1 ? tile_score(pos1) : sc;

    // ---- top-k of the 2k branch scores (ties to the lower position): see select_topk_wave
    const float sel_s[2] = {s0, s1};
    const bool sel_v[2] = {v0, v1};
    bool sel_keep[2];
    select_topk_wave<2>(sel_s, sel_v, k, lane, sel_keep);
    const bool keep0 = sel_keep[0], keep1 = sel_keep[1];
    const unsigned long long kb0 = __ballot(keep0), kb1 = __ballot(keep1);
    const int before = __popcll(kb0 & lt) + __popcll(kb1 & lt);
    const int p0 = before, p1 = before + (keep0 ? 1 : 0);
    const int newcnt = __popcll(kb0) + __popcll(kb1);

    // ---- update: survivors overwrite the row's node list in positional order
    if (WPR == 1 || wave == 0) {
        const long long o = row * p.kmax;
        if (keep0) { p.nf[o + p0] = f; p.nl[o + p0] = m - 1; p.ns[o + p0] = s0; }
        if (keep1) { p.nf[o + p1] = m; p.nl[o + p1] = l;     p.ns[o + p1] = s1; }
        if (lane == 0) p.ncnt[row] = newcnt;
        if (p.level == sd.levels) {
            // every node is now a single block: emit I (ascending), pad, count
            if (keep0) { p.idx[o + p0] = f; if (p.score) p.score[o + p0] = s0; }
            if (keep1) { p.idx[o + p1] = m; if (p.score) p.score[o + p1] = s1; }
            if (lane >= newcnt && lane < p.kmax) {
                p.idx[o + lane] = -1;
                if (p.score) p.score[o + lane] = -INFINITY;
            }
            if (lane == 0) p.cnt[row] = newcnt;
        }
        if (p.tiles && lane == 0) atomicAdd(p.tiles, (unsigned long long)nt);
    }
}

// Copies the node ranges of one level into the caller's trace buffer, -1 in dead slots.
__global__ void __launch_bounds__(256) trace_kernel(const int *nf, const int *nl, const int *ncnt,
                                                    int *out, long long rows, int kmax)
{
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= rows * kmax) return;
    const long long row = i / kmax;
    const int j = (int)(i % kmax);
    const bool live = j < ncnt[row];
    out[2 * i] = live ? nf[i] : -1;
    out[2 * i + 1] = live ? nl[i] : -1;
}

struct PruneWorkspace {
    size_t kp, nf, nl, ns, ncnt, total;
};

static PruneWorkspace prune_layout(const Problem &pb)
{
    PruneWorkspace w;
    size_t off = 0;
    const size_t rows = (size_t)pb.H * pb.NB;
    w.kp = off;   off += align_up((size_t)pb.Hkv * pb.NB * pb.b * pb.d * pb.esize, 256);
    w.nf = off;   off += align_up(rows * pb.kmax * 4, 256);
    w.nl = off;   off += align_up(rows * pb.kmax * 4, 256);
    w.ns = off;   off += align_up(rows * pb.kmax * 4, 256);
    w.ncnt = off; off += align_up(rows * 4, 256);
    w.total = off;
    return w;
}

typedef void (*level_fn)(const PruneParams);

static level_fn pick_level_kernel(const Problem &pb, int &wpr)
{
    const bool bf = pb.dtype == STREAM_BF16;
    wpr = pb.b == 128 ? 4 : 1;
    if (pb.b == 32) {
        if (bf) return pb.d == 128 ? level_kernel<true, 128, 1, 1, 1, 2> : level_kernel<true, 64, 1, 1, 1, 2>;
        return pb.d == 128 ? level_kernel<false, 128, 1, 1, 1, 2> : level_kernel<false, 64, 1, 1, 1, 2>;
    }
    if (pb.b == 64) {
        if (bf) return pb.d == 128 ? level_kernel<true, 128, 2, 2, 1, 2> : level_kernel<true, 64, 2, 2, 1, 2>;
        return pb.d == 128 ? level_kernel<false, 128, 2, 2, 1, 1> : level_kernel<false, 64, 2, 2, 1, 2>;
    }
    if (bf) return pb.d == 128 ? level_kernel<true, 128, 2, 2, 4, 2> : level_kernel<true, 64, 2, 2, 4, 2>;
    return pb.d == 128 ? level_kernel<false, 128, 2, 2, 4, 1> : level_kernel<false, 64, 2, 2, 4, 2>;
}

}  // namespace stream

using namespace stream;

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
    const long long q_sh = shape->q_stride_h ? shape->q_stride_h : pb.T * pb.d;
    const long long q_st = shape->q_stride_t ? shape->q_stride_t : pb.d;
    const long long k_sh = shape->k_stride_h ? shape->k_stride_h : pb.T * pb.d;
    const long long k_st = shape->k_stride_t ? shape->k_stride_t : pb.d;
    if (q_st < pb.d || k_st < pb.d || q_sh < 0 || k_sh < 0) return STREAM_EINVAL;
    // 16-byte vector loads: base pointers and strides must keep rows 16-byte aligned
    if (((uintptr_t)Q | (uintptr_t)K) & 15) return STREAM_EINVAL;
    if ((q_sh * pb.esize | q_st * pb.esize | k_sh * pb.esize | k_st * pb.esize) & 15) return STREAM_EINVAL;
    const PruneWorkspace w = prune_layout(pb);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < w.total) return STREAM_EWORKSPACE;
    hipStream_t st = (hipStream_t)hip_stream;
    char *ws = (char *)workspace;

    rc = launch_pack(K, k_sh, k_st, ws + w.kp, pb, st);
    if (rc != STREAM_OK) return rc;

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
    p.seqs = pb.seqs;
    int wpr = 1;
    level_fn fn = pick_level_kernel(pb, wpr);
    const long long rows_per_kv = (long long)pb.NB * pb.g;
    const long long per_kv = wpr == 1 ? (rows_per_kv + 3) / 4 : rows_per_kv;
    if (per_kv * pb.Hkv + 64 > 0x7fffffffLL) return STREAM_EUNSUPPORTED;
    p.map = make_wg_map(pb.Hkv, (int)per_kv);
    const long long rows = (long long)pb.H * pb.NB;
    for (int level = 1; level <= pb.max_levels; ++level) {
        p.level = level;
        void *const *ev = diag ? diag->level_events : nullptr;
        if (ev && hipEventRecord((hipEvent_t)ev[2 * (level - 1)], st) != hipSuccess) return STREAM_EDEVICE;
        hipLaunchKernelGGL(fn, dim3((unsigned)p.map.grid), dim3(256), 0, st, p);
        if (hipGetLastError() != hipSuccess) return STREAM_EDEVICE;
        if (ev && hipEventRecord((hipEvent_t)ev[2 * (level - 1) + 1], st) != hipSuccess) return STREAM_EDEVICE;
        if (diag && diag->trace) {
            const long long n = rows * pb.kmax;
            hipLaunchKernelGGL(trace_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st,
                               p.nf, p.nl, p.ncnt, diag->trace + (long long)(level - 1) * n * 2,
                               rows, pb.kmax);
            if (hipGetLastError() != hipSuccess) return STREAM_EDEVICE;
        }
    }
    return STREAM_OK;
}

}  // extern "C"
