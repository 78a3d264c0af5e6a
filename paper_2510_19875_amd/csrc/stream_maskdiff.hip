// stream_mask_diff: per (head, query block) row, the key blocks retained with k_success and
// not retained with k_fail (Section 4.2.2, "Exploring Information Flow"), with the block scores
// of the k_success run as weights.  Both lists are ascending, so membership is a binary search;
// a lane holds one entry of each list and the search reads the other list across lanes.
#include "stream_common.h"

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

__device__ __forceinline__ DiffRow diff_load(const DiffParams &p, long long row, int lane)
{
    DiffRow r;
    r.ca = 0; r.cb = 0; r.a = -1; r.b = -1; r.s = -INFINITY;
    if (row < p.rows) {
        r.ca = p.ca[row];
        r.cb = p.cb[row];
        if (lane < p.ka) {
            r.a = p.ia[row * p.ka + lane];
            if (p.sa) r.s = p.sa[row * p.ka + lane];
        }
        if (lane < p.kb) r.b = p.ib[row * p.kb + lane];
    }
    return r;
}

__global__ void __launch_bounds__(256) diff_kernel(const DiffParams p)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const long long stride = (long long)gridDim.x * 4;
    long long row = (long long)blockIdx.x * 4 + wave;
    DiffRow nx = diff_load(p, row, lane);
    for (int i = 0; i < kDiffRowsPerWave && row < p.rows; ++i, row += stride) {
        const DiffRow cur = nx;
        nx = diff_load(p, row + stride, lane);      // next row's loads fly while this one is searched
        int ca = __builtin_amdgcn_readfirstlane(cur.ca), cb = __builtin_amdgcn_readfirstlane(cur.cb);
        ca = ca < 0 ? 0 : (ca > p.ka ? p.ka : ca);
        cb = cb < 0 ? 0 : (cb > p.kb ? p.kb : cb);
        // lower bound of this lane's a in b[0 .. cb): first position whose entry is >= a
        int lo = 0, hi = cb;
#pragma unroll
        for (int step = 0; step < 7; ++step) {       // 2^7 > 64 entries
            const int mid = (lo + hi) >> 1;
            const int bm = __shfl(cur.b, mid & 63);
            const bool go = lo < hi && bm < cur.a;
            const bool stay = lo < hi && !(bm < cur.a);
            lo = go ? mid + 1 : lo;
            hi = stay ? mid : hi;
        }
        const int bl = __shfl(cur.b, lo & 63);
        const bool in_b = lo < cb && bl == cur.a;
        const bool keep = lane < ca && !in_b;
        const unsigned long long kb = __ballot(keep);
        const int pos = __popcll(kb & ((1ull << lane) - 1ull));
        const int n = __popcll(kb);
        const long long o = row * p.ka;
        if (keep) {
            p.io[o + pos] = cur.a;
            if (p.wo) p.wo[o + pos] = cur.s;
        }
        if (lane >= n && lane < p.ka) {
            p.io[o + lane] = -1;
            if (p.wo) p.wo[o + lane] = -INFINITY;
        }
        if (lane == 0) p.co[row] = n;
    }
}

}  // namespace stream

using namespace stream;

extern "C" stream_status stream_mask_diff(const int *idx_a, const int *cnt_a, const float *score_a, int kmax_a,
                                          const int *idx_b, const int *cnt_b, int kmax_b, long long rows,
                                          int *idx_out, int *cnt_out, float *weight_out, void *hip_stream)
{
    if (rows < 0 || kmax_a < 1 || kmax_b < 1) return STREAM_EINVAL;
    if (kmax_a > kMaxTopk || kmax_b > kMaxTopk) return STREAM_EUNSUPPORTED;
    const long long grid = (rows + 4 * kDiffRowsPerWave - 1) / (4 * kDiffRowsPerWave);
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
    hipLaunchKernelGGL(diff_kernel, dim3((unsigned)grid), dim3(256), 0, (hipStream_t)hip_stream, p);
    return hipGetLastError() == hipSuccess ? STREAM_OK : STREAM_EDEVICE;
}
