// stream_mask_diff: per (head, query block) row, the key blocks retained with k_success and
// not retained with k_fail (Section 4.2.2, "Exploring Information Flow"), with the block scores
// of the k_success run as weights.  Both lists are ascending, so membership is a binary search;
// a lane holds one entry of each list and the search reads the other list across lanes.  Lists of
// at most 32 entries take half a wavefront each.
#include "stream_common.h"
#include "stream_mfma.h"

#include <math.h>

namespace stream {

struct DiffParams {
    const int *ia, *ca;      // [rows, ka], [rows]
    const float *sa;         // [rows, ka] or null
    const int *ib, *cb;      // [rows, kb], [rows]
    int *io, *co;            // [rows, ka], [rows]
    float *wo;               // [rows, ka] or null
    long long rows;
    int ka, kb;
};

constexpr int kDiffRowsPerWave = 8;

struct DiffRow {
    int ca, cb, a, b;
    float s;
};

// RPW rows per wavefront step: 1 (a row on 64 lanes) or, when both lists have at most 32 entries,
// 2 (a row on each half of the wavefront).
template <int RPW>
__device__ __forceinline__ DiffRow diff_load(const DiffParams &p, long long row, int l)
{
    DiffRow r;
    r.ca = 0; r.cb = 0; r.a = -1; r.b = -1; r.s = -INFINITY;
    if (row < p.rows) {
        r.ca = p.ca[row];
        r.cb = p.cb[row];
        if (l < p.ka) {
            r.a = p.ia[row * p.ka + l];
            if (p.sa) r.s = p.sa[row * p.ka + l];
        }
        if (l < p.kb) r.b = p.ib[row * p.kb + l];
    }
    return r;
}

template <int RPW>
__global__ void __launch_bounds__(256) diff_kernel(const DiffParams p)
{
    constexpr int LPR = 64 / RPW;                      // lanes per row
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int sub = lane / LPR, l = lane % LPR;        // which row of the step, which entry
    const long long stride = (long long)gridDim.x * 4 * RPW;
    long long row = ((long long)blockIdx.x * 4 + wave) * RPW + sub;
    DiffRow nx = diff_load<RPW>(p, row, l);
    // (the first rows' loads are waited for here, once: with them still pending at the loop's
    // entry the compiler waited, in every iteration, for the next rows' loads right after issuing them)
    __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt(0), the other counters untouched
    for (int i = 0; i < kDiffRowsPerWave; ++i, row += stride) {
        if (row - sub >= p.rows) break;                // wave-uniform: the step's first row
        const DiffRow cur = nx;
        nx = diff_load<RPW>(p, row + stride, l);       // next rows' loads fly while these are searched
        int ca = cur.ca, cb = cur.cb;
        ca = ca < 0 ? 0 : (ca > p.ka ? p.ka : ca);
        cb = cb < 0 ? 0 : (cb > p.kb ? p.kb : cb);
        // lower bound of this lane's a in b[0 .. cb): first position whose entry is >= a
        int lo = 0, hi = cb;
#pragma unroll
        for (int step = 0; step < (RPW == 1 ? 7 : 6); ++step) {   // 2^7 > 64, 2^6 > 32 entries
            const int mid = (lo + hi) >> 1;
            const int bm = __shfl(cur.b, sub * LPR + (mid & (LPR - 1)));
            const bool go = lo < hi && bm < cur.a;
            const bool stay = lo < hi && !(bm < cur.a);
            lo = go ? mid + 1 : lo;
            hi = stay ? mid : hi;
        }
        const int bl = __shfl(cur.b, sub * LPR + (lo & (LPR - 1)));
        const bool in_b = lo < cb && bl == cur.a;
        const bool keep = row < p.rows && l < ca && !in_b;
        const unsigned long long kb_all = __ballot(keep);
        const unsigned long long kb = RPW == 1 ? kb_all : ((kb_all >> (sub * LPR)) & 0xffffffffull);
        const int pos = __popcll(kb & ((1ull << l) - 1ull));
        const int n = __popcll(kb);
        // The next rows' data is taken here, before these rows' stores are issued: stores and loads
        // share one counter and complete in order, so a wait for the loads placed after the stores
        // would wait for the stores' acknowledgements as well.
        // (the count as an operand keeps the compiler from moving this, and the wait, above the search)
        asm volatile("" : "+v"(nx.ca), "+v"(nx.cb), "+v"(nx.a), "+v"(nx.b), "+v"(nx.s) : "s"(n));
        if (row < p.rows) {
            const long long o = row * p.ka;
            if (keep) {
                p.io[o + pos] = cur.a;
                if (p.wo) p.wo[o + pos] = cur.s;
            }
            if (l >= n && l < p.ka) {
                p.io[o + l] = -1;
                if (p.wo) p.wo[o + l] = -INFINITY;
            }
            if (l == 0) p.co[row] = n;
        }
    }
}

// Lists of more than 64 entries (up to kMaxTopkWide): a wavefront per row, the row's b list in LDS,
// the a list taken 64 entries at a time (lower-bound search in LDS, ballot compaction, outputs
// appended in order).
__global__ void __launch_bounds__(256) diff_wide_kernel(const DiffParams p)
{
    __shared__ int s_b[4][kMaxTopkWide];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const long long row = (long long)blockIdx.x * 4 + wave;
    if (row >= p.rows) return;
    int ca = p.ca[row], cb = p.cb[row];
    ca = ca < 0 ? 0 : (ca > p.ka ? p.ka : ca);
    cb = cb < 0 ? 0 : (cb > p.kb ? p.kb : cb);
    int *b = s_b[wave];
    for (int i = lane; i < cb; i += 64) b[i] = p.ib[row * p.kb + i];
    wave_sync();
    const long long o = row * p.ka;
    const unsigned long long lt = (1ull << lane) - 1ull;
    int n = 0;
    for (int c0 = 0; c0 < ca; c0 += 64) {
        const int j = c0 + lane;
        const bool live = j < ca;
        const int a = live ? p.ia[o + j] : -1;
        const float sc = live && p.sa ? p.sa[o + j] : -INFINITY;
        int lo = 0, hi = cb;                               // first position of b whose entry is >= a
#pragma unroll
        for (int step = 0; step < 10; ++step) {            // 2^10 > 512 entries
            const int mid = (lo + hi) >> 1;
            const bool open = lo < hi;
            const int bm = open ? b[mid] : 0;
            lo = open && bm < a ? mid + 1 : lo;
            hi = open && !(bm < a) ? mid : hi;
        }
        const bool in_b = lo < cb && b[lo < cb ? lo : 0] == a;
        const bool keep = live && !in_b;
        const unsigned long long kb = __ballot(keep);
        const int pos = n + __popcll(kb & lt);
        if (keep) {
            p.io[o + pos] = a;
            if (p.wo) p.wo[o + pos] = sc;
        }
        n += __popcll(kb);
    }
    for (int j = n + lane; j < p.ka; j += 64) {
        p.io[o + j] = -1;
        if (p.wo) p.wo[o + j] = -INFINITY;
    }
    if (lane == 0) p.co[row] = n;
}

}  // namespace stream

using namespace stream;

extern "C" stream_status stream_mask_diff(const int *idx_a, const int *cnt_a, const float *score_a, int kmax_a,
                                          const int *idx_b, const int *cnt_b, int kmax_b, long long rows,
                                          int *idx_out, int *cnt_out, float *weight_out, void *hip_stream)
{
    if (rows < 0 || kmax_a < 1 || kmax_b < 1) return STREAM_EINVAL;
    if (kmax_a > kMaxTopkWide || kmax_b > kMaxTopkWide) return STREAM_EUNSUPPORTED;
    const bool wide = kmax_a > kMaxTopk || kmax_b > kMaxTopk;
    const int rpw = (kmax_a <= 32 && kmax_b <= 32) ? 2 : 1;
    const long long per_wg = wide ? 4LL : 4LL * kDiffRowsPerWave * rpw;
    const long long grid = (rows + per_wg - 1) / per_wg;
    if (grid > 0x7fffffffLL) return STREAM_EUNSUPPORTED;
    if (rows == 0) return STREAM_OK;                 // empty tensors may have no address
    if (!idx_a || !cnt_a || !idx_b || !cnt_b || !idx_out || !cnt_out) return STREAM_EINVAL;
    if (weight_out && !score_a) return STREAM_EINVAL;
    // in place is not supported: a row's output would overwrite entries other lanes still read
    if (idx_out == idx_a || idx_out == idx_b) return STREAM_EINVAL;
    DiffParams p;
    p.ia = idx_a; p.ca = cnt_a; p.sa = score_a; p.ib = idx_b; p.cb = cnt_b;
    p.io = idx_out; p.co = cnt_out; p.wo = weight_out;
    p.rows = rows; p.ka = kmax_a; p.kb = kmax_b;
    if (wide)
        hipLaunchKernelGGL(diff_wide_kernel, dim3((unsigned)grid), dim3(256), 0, (hipStream_t)hip_stream, p);
    else
        hipLaunchKernelGGL(rpw == 2 ? diff_kernel<2> : diff_kernel<1>, dim3((unsigned)grid), dim3(256), 0, (hipStream_t)hip_stream, p);
    return hipGetLastError() == hipSuccess ? STREAM_OK : STREAM_EDEVICE;
}
