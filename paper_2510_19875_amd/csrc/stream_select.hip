// stream_select_update: the top-k selection and node update of Alg. 2 as a pass of its own.
// stream_prune fuses this step into the scoring kernel (the branch scores never leave the
// chip); this entry point runs it from a score tensor in memory so that the step can be used
// and measured alone.  A wavefront ranks one row at a time, several rows in a row.
#include "stream_select.h"
#include "stream_mfma.h"

#include <math.h>

namespace stream {

struct SelectParams {
    const float *score;   // [rows, 2 * kmax]
    int *nf, *nl;         // [rows, kmax]
    int *ncnt;            // [rows]
    long long rows;
    int k, kmax;
};

// Rows a wavefront handles, one after the other; the loads of the next row are in flight while
// the current one is ranked, so that a wavefront keeps two rows' worth of memory requests going.
constexpr int kSelectRowsPerWave = 8;

// NB = 1 (kmax <= 32): lane j holds branch position j, i.e. side j % 2 of node j / 2;
// NB = 2: lane j holds both children of node j.
template <int NB>
struct SelectRow {
    int c, f, l;
    float s[NB];
};

// The row's loads go through buffer resources over the whole arrays: the address of a load is a
// scalar row offset plus the lane's constant offset, so a row costs no vector address arithmetic,
// and what lies past the arrays (the prefetch after the last row) reads as zeros.  A lane past
// the row's slots reads its neighbour row's data, which is never used: such a lane is not live.
struct SelectBuffers {
    __amdgpu_buffer_rsrc_t nf, nl, sc, cnt;
    unsigned voff_node, voff_score;      // this lane's byte offsets inside a row
    unsigned kmax;
};

template <int NB>
__device__ __forceinline__ SelectRow<NB> select_load(const SelectBuffers &b, unsigned row)
{
    SelectRow<NB> r;
    const unsigned so = row * b.kmax * 4u;                 // the row's byte offset in nf / nl (scalar)
    r.c = (int)__builtin_amdgcn_raw_buffer_load_b32(b.cnt, 0, row * 4u, 0);
    r.f = (int)__builtin_amdgcn_raw_buffer_load_b32(b.nf, b.voff_node, so, 0);
    r.l = (int)__builtin_amdgcn_raw_buffer_load_b32(b.nl, b.voff_node, so, 0);
    if constexpr (NB == 2) {
        typedef unsigned u32x2_t __attribute__((ext_vector_type(2)));
        const u32x2_t v = __builtin_amdgcn_raw_buffer_load_b64(b.sc, b.voff_score, 2u * so, 0);
        // (elements copied out by value first: __builtin_bit_cast applied directly to an element
        // of an ext_vector_type lvalue reads element 0 whatever the index, with this compiler)
        const unsigned s0 = v[0], s1 = v[1];
        r.s[0] = __builtin_bit_cast(float, s0);
        r.s[1] = __builtin_bit_cast(float, s1);
    } else {
        r.s[0] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(b.sc, b.voff_score, 2u * so, 0));
    }
    return r;
}

// The selection of select_topk_wave with the search state kept in vector registers.  With many
// wavefronts per SIMD (this pass has no matrix work to hide behind) what limits the search is the
// scalar unit: it issues one instruction per wavefront turn and the scalar form of a step is seven
// of them against one vector compare.  Here a step is: candidate = threshold | bit (vector),
// compare (vector), count of the lane mask (scalar), count >= k and the conditional move
// (vector), and the scalar test for the early exit: three scalar and four vector instructions.
// The values are wave-uniform all the same; the empty asm below only hides that from the
// compiler, which would otherwise move them back to the scalar unit.  Same result bit for bit.
template <int NB>
__device__ __forceinline__ void select_topk_wave_v(const float (&s)[NB], const bool (&v)[NB], int k, int lane,
                                                   bool (&keep)[NB])
{
    unsigned u[NB];
    int n_valid = 0;
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const unsigned b = sortable_bits(s[i]);
        u[i] = v[i] ? (b ? b : 1u) : 0u;
        n_valid += __popcll(__ballot(v[i]));
    }
    if (n_valid <= k) {                           // wave-uniform
#pragma unroll
        for (int i = 0; i < NB; ++i) keep[i] = v[i];
        return;
    }
    unsigned thr = 0;
    int kv = k;
    asm volatile("" : "+v"(thr), "+v"(kv));       // (a vector register each; see above)
#pragma unroll
    for (int bit = 31; bit >= 0; --bit) {
        const unsigned t = thr | (1u << bit);
        int ge = 0;
#pragma unroll
        for (int i = 0; i < NB; ++i) ge += __popcll(__ballot(u[i] >= t));
        thr = ge >= kv ? t : thr;
        if (ge == k) break;
    }
    int n_ge = 0;                                 // (counted again: cheaper than a flag set in every step)
#pragma unroll
    for (int i = 0; i < NB; ++i) n_ge += __popcll(__ballot(u[i] >= thr));
    if (n_ge == k) {
#pragma unroll
        for (int i = 0; i < NB; ++i) keep[i] = u[i] >= thr;
        return;
    }
    // ties at the threshold
    const unsigned long long lt = (1ull << lane) - 1ull;
    int n_gt = 0;
#pragma unroll
    for (int i = 0; i < NB; ++i) n_gt += __popcll(__ballot(u[i] > thr));
    const int need = k - n_gt;
    int before = 0;                               // equal branches at lower positions
#pragma unroll
    for (int i = 0; i < NB; ++i) before += __popcll(__ballot(u[i] == thr) & lt);
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const bool eq = u[i] == thr;
        keep[i] = u[i] > thr || (eq && before < need);
        before += eq ? 1 : 0;                     // this lane's own lower position
    }
}

// p.rows here is one launch's share of the rows, few enough that every byte offset fits 31 bits.
template <int NB>
__global__ void __launch_bounds__(256) select_kernel(const SelectParams p)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // consecutive wavefronts take consecutive rows; a wavefront's own rows are a grid apart
    const unsigned rows = (unsigned)p.rows;
    const unsigned stride = gridDim.x * 4u;
    unsigned row = blockIdx.x * 4u + (unsigned)wave;
    const int node = NB == 2 ? lane : lane >> 1;
    SelectBuffers b;
    b.kmax = (unsigned)p.kmax;
    b.nf = make_tile_rsrc(p.nf, rows * b.kmax * 4u);
    b.nl = make_tile_rsrc(p.nl, rows * b.kmax * 4u);
    b.sc = make_tile_rsrc(p.score, rows * b.kmax * 8u);
    b.cnt = make_tile_rsrc(p.ncnt, rows * 4u);
    b.voff_node = (unsigned)node * 4u;
    b.voff_score = NB == 2 ? (unsigned)lane * 8u : (unsigned)lane * 4u;
    SelectRow<NB> nx = select_load<NB>(b, row);
    // (the first row's loads are waited for here, once: with them still pending at the loop's
    // entry the compiler waited, in every iteration, for the loads of the next row right after
    // issuing them; now those stay in flight during the search and are waited for after it)
    __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt(0), the other counters untouched
    for (int i = 0; i < kSelectRowsPerWave && row < rows; ++i, row += stride) {
        const SelectRow<NB> cur = nx;
        nx = select_load<NB>(b, row + stride);
        int c = __builtin_amdgcn_readfirstlane(cur.c);
        c = c < 0 ? 0 : (c > p.kmax ? p.kmax : c);
        const int f = cur.f, l = cur.l;
        const bool live = node < c && f <= l;
        const int m = (f + l + 1) >> 1;                     // children [f, m-1] and [m, l]
        bool v[NB], keep[NB];
        int first[NB], last[NB];
        if constexpr (NB == 2) {
            v[0] = live && m > f && cur.s[0] > -INFINITY;
            v[1] = live && cur.s[1] > -INFINITY;
            first[0] = f; last[0] = m - 1; first[1] = m; last[1] = l;
        } else {
            const bool right = lane & 1;
            v[0] = live && (right || m > f) && cur.s[0] > -INFINITY;
            first[0] = right ? m : f; last[0] = right ? l : m - 1;
        }
        select_topk_wave_v<NB>(cur.s, v, p.k, lane, keep);
        // update: survivors overwrite the row's node list in positional order
        unsigned long long kb[NB];
        int pos = 0, total = 0;
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            kb[j] = __ballot(keep[j]);
            pos += lanes_below(kb[j]);
            total += __popcll(kb[j]);
        }
        // The next row's data is taken here, before this row's stores are issued: stores and loads
        // share one counter and complete in order, so a wait for the loads placed after the stores
        // would wait for the stores' acknowledgements as well.  (The count as an operand keeps
        // the compiler from moving this, and the wait, above the search.)
        asm volatile("" : "+v"(nx.c), "+v"(nx.f), "+v"(nx.l), "+v"(nx.s[0]) : "s"(total));
        if constexpr (NB == 2) asm volatile("" : "+v"(nx.s[1]) : "s"(total));
        const unsigned so = row * b.kmax * 4u;
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            if (keep[j]) {
                __builtin_amdgcn_raw_buffer_store_b32((unsigned)first[j], b.nf, (unsigned)pos * 4u, so, 0);
                __builtin_amdgcn_raw_buffer_store_b32((unsigned)last[j], b.nl, (unsigned)pos * 4u, so, 0);
            }
            pos += keep[j] ? 1 : 0;
        }
        if (lane == 0) __builtin_amdgcn_raw_buffer_store_b32((unsigned)total, b.cnt, 0, row * 4u, 0);
    }
}

// Rows of more than 64 nodes (up to kMaxTopkWide): a wavefront per row, the branch keys and the
// node list in LDS, every step in chunks of 64 branch positions (position 2j + side = child
// `side` of node j), as the wide refinement kernel does it.
__global__ void __launch_bounds__(256) select_wide_kernel(const SelectParams p)
{
    __shared__ unsigned s_key[4][2 * kMaxTopkWide];
    __shared__ int s_f[4][kMaxTopkWide], s_l[4][kMaxTopkWide];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const long long row = (long long)blockIdx.x * 4 + wave;
    if (row >= p.rows) return;
    const long long o = row * p.kmax;
    const unsigned long long lt = (1ull << lane) - 1ull;
    int c = p.ncnt[row];
    c = c < 0 ? 0 : (c > p.kmax ? p.kmax : c);
    unsigned *key_of = s_key[wave];
    int *nf = s_f[wave], *nl = s_l[wave];
    for (int j = lane; j < c; j += 64) { nf[j] = p.nf[o + j]; nl[j] = p.nl[o + j]; }
    wave_sync();
    const int npos = 2 * c, k = p.k;
    int n_valid = 0;
    for (int c0 = 0; c0 < npos; c0 += 64) {
        const int pp = c0 + lane;
        unsigned key = 0;
        if (pp < npos) {
            const int f = nf[pp >> 1], l = nl[pp >> 1];
            const int m = (f + l + 1) >> 1;                 // children [f, m-1] and [m, l]
            const float sc = p.score[2 * o + pp];
            if (f <= l && ((pp & 1) || m > f) && sc > -INFINITY) {
                const unsigned b = sortable_bits(sc);
                key = b ? b : 1u;
            }
            key_of[pp] = key;
        }
        n_valid += __popcll(__ballot(key != 0));
    }
    wave_sync();
    unsigned thr = 1;            // n_valid <= k: every candidate is kept (keys are >= 1)
    int need_eq = 0;
    bool ties = false;           // keep key > thr plus the first need_eq of the equal ones
    if (n_valid > k) {
        thr = 0;
        bool exact = false;
        for (int bit = 31; bit >= 0 && !exact; --bit) {
            const unsigned t = thr | (1u << bit);
            int ge = 0;
            for (int c0 = 0; c0 < npos; c0 += 64)
                ge += __popcll(__ballot(c0 + lane < npos && key_of[c0 + lane] >= t));
            if (ge >= k) {
                thr = t;
                exact = ge == k;
            }
        }
        if (!exact) {
            int n_gt = 0;
            for (int c0 = 0; c0 < npos; c0 += 64)
                n_gt += __popcll(__ballot(c0 + lane < npos && key_of[c0 + lane] > thr));
            need_eq = k - n_gt;
            ties = true;
        }
    }
    int out_base = 0, eq_seen = 0;
    for (int c0 = 0; c0 < npos; c0 += 64) {
        const int pp = c0 + lane;
        const unsigned key = pp < npos ? key_of[pp] : 0u;
        bool keep = key >= thr;
        if (ties) {
            const bool eq = key == thr;
            const unsigned long long be = __ballot(eq);
            keep = key > thr || (eq && eq_seen + __popcll(be & lt) < need_eq);
            eq_seen += __popcll(be);
        }
        const unsigned long long kb = __ballot(keep);
        const int out = out_base + __popcll(kb & lt);
        if (keep) {
            const int f = nf[pp >> 1], l = nl[pp >> 1];
            const int m = (f + l + 1) >> 1;
            p.nf[o + out] = (pp & 1) ? m : f;
            p.nl[o + out] = (pp & 1) ? l : m - 1;
        }
        out_base += __popcll(kb);
    }
    if (lane == 0) p.ncnt[row] = out_base;
}

}  // namespace stream

using namespace stream;

extern "C" stream_status stream_select_update(const float *branch_score, int *node_first, int *node_last,
                                              int *node_count, long long rows, int topk, int topk_max,
                                              void *hip_stream)
{
    if (rows < 0 || topk < 1 || topk > topk_max) return STREAM_EINVAL;
    if (topk_max > kMaxTopkWide) return STREAM_EUNSUPPORTED;
    const bool wide = topk_max > kMaxTopk;
    const long long per_wg = wide ? 4 : 4 * kSelectRowsPerWave;
    const long long grid = (rows + per_wg - 1) / per_wg;
    if (grid > 0x7fffffffLL) return STREAM_EUNSUPPORTED;
    if (rows == 0) return STREAM_OK;                           // empty tensors may have no address
    if (!branch_score || !node_first || !node_last || !node_count) return STREAM_EINVAL;
    if ((uintptr_t)branch_score & 7) return STREAM_EINVAL;     // scores are read in pairs
    SelectParams p;
    p.score = branch_score; p.nf = node_first; p.nl = node_last; p.ncnt = node_count;
    p.rows = rows; p.k = topk; p.kmax = topk_max;
    if (wide) {
        hipLaunchKernelGGL(select_wide_kernel, dim3((unsigned)grid), dim3(256), 0, (hipStream_t)hip_stream, p);
        return hipGetLastError() == hipSuccess ? STREAM_OK : STREAM_EDEVICE;
    }
    // The narrow kernel addresses a launch's rows with 32-bit byte offsets: at most 2^31 bytes of
    // scores (8 bytes per node slot) per launch, more rows in further launches behind it.
    const long long chunk = ((1LL << 31) / (8LL * topk_max)) & ~3LL;
    for (long long r0 = 0; r0 < rows; r0 += chunk) {
        const long long n = rows - r0 < chunk ? rows - r0 : chunk;
        p.score = branch_score + 2 * r0 * topk_max;
        p.nf = node_first + r0 * topk_max;
        p.nl = node_last + r0 * topk_max;
        p.ncnt = node_count + r0;
        p.rows = n;
        const long long g = (n + per_wg - 1) / per_wg;
        hipLaunchKernelGGL(topk_max <= 32 ? select_kernel<1> : select_kernel<2>, dim3((unsigned)g), dim3(256), 0,
                           (hipStream_t)hip_stream, p);
        if (hipGetLastError() != hipSuccess) return STREAM_EDEVICE;
    }
    return STREAM_OK;
}
