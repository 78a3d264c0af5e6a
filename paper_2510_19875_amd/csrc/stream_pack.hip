// Host-side argument validation shared by the entry points, and the K/V tile packer.
#include "stream_common.h"

namespace stream {

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

static int ceil_log2_ll(long long n)
{
    int it = 0;
    long long v = 1;
    while (v < n) { v <<= 1; ++it; }
    return it;
}

// Validates a shape (+ optional top-k arguments; topk_max <= 0 skips them) and derives the
// per-sequence block geometry of the preamble of Alg. 2: T_p = T rounded up to a multiple of
// lcm(b_q, b_k) per sequence.
stream_status make_problem(const stream_shape *s, int topk, const int *topk_per_seq, int topk_max,
                           Problem *out)
{
    if (!s || !out) return STREAM_EINVAL;
    if (s->heads <= 0 || s->kv_heads <= 0 || s->T <= 0 || s->batch <= 0) return STREAM_EINVAL;
    if (s->heads % s->kv_heads != 0) return STREAM_EINVAL;
    if (s->dtype != STREAM_F32 && s->dtype != STREAM_BF16) return STREAM_EINVAL;
    if (s->batch > 1 && !s->cu_seqlens) return STREAM_EINVAL;
    if (s->head_dim != 64 && s->head_dim != 128) return STREAM_EUNSUPPORTED;
    if (s->block != 32 && s->block != 64 && s->block != 128) return STREAM_EUNSUPPORTED;
    if (s->block_k != 0 && s->block_k != 32 && s->block_k != 64 && s->block_k != 128) return STREAM_EUNSUPPORTED;
    if (s->batch > kMaxBatch) return STREAM_EUNSUPPORTED;
    if (s->T > (1LL << 31) - 4096) return STREAM_EUNSUPPORTED;
    if (s->mask != STREAM_MASK_CAUSAL && s->mask != STREAM_MASK_FULL && s->mask != STREAM_MASK_SLIDING &&
        s->mask != STREAM_MASK_ARRAY)
        return STREAM_EINVAL;
    if (s->mask == STREAM_MASK_SLIDING && s->window < 1) return STREAM_EINVAL;
    if (s->mask == STREAM_MASK_ARRAY) {
        if (!s->mask_bits || ((uintptr_t)s->mask_bits & 3)) return STREAM_EINVAL;
        if (s->mask_pitch < (s->T + 31) / 32) return STREAM_EINVAL;
        if (s->batch != 1) return STREAM_EUNSUPPORTED;
    }

    Problem &p = *out;
    p.H = s->heads; p.Hkv = s->kv_heads; p.g = s->heads / s->kv_heads;
    p.d = s->head_dim; p.b = s->block; p.bk = s->block_k ? s->block_k : s->block; p.dtype = s->dtype;
    const int lcm = p.b > p.bk ? p.b : p.bk;          // both are powers of two
    p.esize = s->dtype == STREAM_BF16 ? 2 : 4;
    p.batch = s->batch; p.T = s->T; p.kmax = topk_max;
    p.mask = s->mask;
    // a window that reaches past the longest possible sequence is the causal mask
    p.window = s->mask == STREAM_MASK_SLIDING ? (int)(s->window < s->T ? s->window : s->T) : 0;
    p.cbits = s->mask == STREAM_MASK_ARRAY ? s->mask_bits : nullptr;
    p.cpitch = s->mask == STREAM_MASK_ARRAY ? s->mask_pitch : 0;
    p.seqs.n = s->batch;
    long long nb = 0, tok = 0;
    int maxlev = 0;
    for (int i = 0; i < s->batch; ++i) {
        long long a = s->cu_seqlens ? s->cu_seqlens[i] : 0;
        long long e = s->cu_seqlens ? s->cu_seqlens[i + 1] : s->T;
        if (a != tok || e <= a) return STREAM_EINVAL;  // cu[0] = 0, strictly increasing
        SeqDesc &sd = p.seqs.d[i];
        sd.tok0 = a;
        sd.len = (int)(e - a);
        const long long t_pad = (e - a + lcm - 1) / lcm * lcm;      // T_p of the preamble of Alg. 2
        sd.nblk = (int)(t_pad / p.b);
        const long long nkb = t_pad / p.bk;                          // key blocks: the nodes range over these
        // tile offsets inside one (kv head, sequence) region are 32-bit
        if (t_pad * s->head_dim * p.esize >= (1LL << 31)) return STREAM_EUNSUPPORTED;
        sd.blk0 = (int)nb;
        sd.k = 0; sd.levels = 0; sd.pad_ = 0;
        if (topk_max > 0) {
            int k = topk_per_seq ? topk_per_seq[i] : topk;
            if (k < 1) return STREAM_EINVAL;
            if (k > topk_max) return STREAM_EINVAL;
            sd.k = k;
            long long per = (nkb + (long long)k - 1) / k;
            int lv = ceil_log2_ll(per);
            sd.levels = lv < 1 ? 1 : lv;
            if (sd.levels > maxlev) maxlev = sd.levels;
        }
        nb += sd.nblk;
        tok = e;
    }
    if (tok != s->T) return STREAM_EINVAL;
    if (nb > (1LL << 30)) return STREAM_EUNSUPPORTED;
    if (topk_max > kMaxTopkWide) return STREAM_EUNSUPPORTED;
    p.NB = (int)nb;
    p.max_levels = maxlev;
    return STREAM_OK;
}

// ---------------------------------------------------------------------------------------------
// Tile packing.
//
// A 32x32 MFMA reads, per lane, 16 contiguous bytes of one operand row: lane (n = lane % 32,
// g = lane / 32) supplies row n, and the g-th half of the fragment's slice of the contraction
// axis.  Reading those 16 bytes straight from a row-major [token, d] tensor makes every lane of
// a load instruction touch a different row.  The packer therefore rewrites each group of 32
// tokens so that the 64 lanes' chunks of fragment `fr` are contiguous (1 KiB per fragment):
//
//     dst chunk (fr * 64 + g * 32 + n)  <-  src row n, 16-byte chunk (2 * fr + g)
//
// A block of b tokens is b/32 consecutive groups; tokens past the end of a sequence are zero
// (they are masked out wherever they could matter).  Layout: [kv_head][global block][b * d].
// The permutation is per 32-token group, so the same packed tensor serves every block size.
// With kPackFrag16 (operands of the 16x16x32 bf16 MFMA: lane (g = lane / 16, n = lane % 16) supplies
// row n and the g-th 16-byte chunk of the fragment's 64-byte slice) the group is cut into
// fragments of 16 rows x 64 bytes instead:
//
//     dst chunk ((n / 16 * (row_bytes / 64) + cc / 4) * 64 + (cc % 4) * 16 + n % 16)  <-  src row n, chunk cc
// ---------------------------------------------------------------------------------------------
struct PackParams {
    const char *src;
    char *dst;
    long long stride_h_bytes, stride_t_bytes;
    int row_bytes;   // d * esize
    int b, NB, Hkv;
    int frag16;      // kPackFrag16 layout
    SeqTable seqs;
};

__global__ void __launch_bounds__(256) pack_kernel(PackParams p)
{
    const int cpr = p.row_bytes / 16;         // 16-byte chunks per row
    const int groups = p.b / 32;
    const long long grp = blockIdx.x;          // (kvh * NB + gb) * groups + gi
    const int gi = (int)(grp % groups);
    const long long t = grp / groups;
    const int gb = (int)(t % p.NB);
    const int kvh = (int)(t / p.NB);
    const int s = seq_of_block(p.seqs, gb);
    const SeqDesc sd = p.seqs.d[s];
    const int r = gb - sd.blk0;
    const int tok_in_seq0 = r * p.b + gi * 32;
    char *dst = p.dst + grp * (32LL * p.row_bytes);
    for (int c = threadIdx.x; c < 32 * cpr; c += blockDim.x) {
        const int n = c / cpr, cc = c % cpr;
        const int fr = cc >> 1, g = cc & 1;
        uint4 v = make_uint4(0, 0, 0, 0);
        const int tok = tok_in_seq0 + n;
        if (tok < sd.len)
            v = *reinterpret_cast<const uint4 *>(p.src + kvh * p.stride_h_bytes +
                                                 (sd.tok0 + tok) * p.stride_t_bytes + cc * 16);
        int chunk = fr * 64 + g * 32 + n;
        if (p.frag16) {
            // fragment (16-row group n / 16, 64-byte slice cc / 4), lane (chunk cc % 4 of the slice, row n % 16)
            const int kf = cpr >> 2;
            chunk = ((n >> 4) * kf + (cc >> 2)) * 64 + (cc & 3) * 16 + (n & 15);
        }
        *reinterpret_cast<uint4 *>(dst + chunk * 16) = v;
    }
}

stream_status launch_pack(const void *src, long long stride_h, long long stride_t, void *dst,
                          const Problem &pb, hipStream_t st, PackLayout layout)
{
    PackParams p;
    p.frag16 = layout == kPackFrag16 ? 1 : 0;
    p.src = (const char *)src;
    p.dst = (char *)dst;
    p.stride_h_bytes = stride_h * pb.esize;
    p.stride_t_bytes = stride_t * pb.esize;
    p.row_bytes = pb.d * pb.esize;
    p.b = pb.b; p.NB = pb.NB; p.Hkv = pb.Hkv;
    p.seqs = pb.seqs;
    long long grid = (long long)pb.Hkv * pb.NB * (pb.b / 32);
    if (grid > 0x7fffffffLL) return STREAM_EUNSUPPORTED;
    hipLaunchKernelGGL(pack_kernel, dim3((unsigned)grid), dim3(256), 0, st, p);
    return hipGetLastError() == hipSuccess ? STREAM_OK : STREAM_EDEVICE;
}

// ---------------------------------------------------------------------------------------------
// Block-level summaries of an explicit mask (STREAM_MASK_ARRAY).  A thread owns one (query block,
// key block) pair and walks the b_q rows of its b_k / 32 words; consecutive threads own
// consecutive key blocks, so a wavefront reads consecutive words of every row.
// ---------------------------------------------------------------------------------------------
struct BitmapParams {
    const unsigned *cbits;
    long long cpitch;
    unsigned *any_bits, *all_bits;
    int T, bq, bk, nq, nk, words;
};

template <int WPB>   // 32-bit words of a row per key block: b_k / 32
__global__ void __launch_bounds__(256) block_bitmap_kernel(BitmapParams p)
{
    const int lane = threadIdx.x & 63;
    const int q = blockIdx.y;
    const int chunk = blockIdx.x * 4 + (threadIdx.x >> 6);        // a wavefront per 64 key blocks: the
    const int r = chunk * 64 + lane;                              // workgroup reads 256 adjacent ones
    bool any = false, all = false;
    if (r < p.nk && (long long)r * p.bk < p.T && (long long)q * p.bq < p.T) {
        const int t0 = q * p.bq, u0 = r * p.bk;
        const int t1 = t0 + p.bq < p.T ? t0 + p.bq : p.T;
        unsigned acc_or = 0, acc_and = ~0u;
        unsigned keep[WPB];                                       // keys past the end do not exist
#pragma unroll
        for (int w = 0; w < WPB; ++w) {
            const int ub = u0 + w * 32;                           // first key of this word
            keep[w] = ub >= p.T ? 0u : (ub + 32 > p.T ? (1u << (p.T - ub)) - 1u : ~0u);
        }
        // (a word wholly past the end of the rows is not read: its lane reads the last real word
        // in its place and masks it away, so that every load is unconditional and many are in flight)
        const int lastw = (p.T - 1) >> 5;
        int wofs[WPB];
#pragma unroll
        for (int w = 0; w < WPB; ++w) wofs[w] = (u0 >> 5) + w < lastw ? (u0 >> 5) + w : lastw;
        const unsigned *src = p.cbits + (long long)t0 * p.cpitch;
#pragma unroll 16
        for (int t = t0; t < t1; ++t, src += p.cpitch)
#pragma unroll
            for (int w = 0; w < WPB; ++w) {
                const unsigned x = src[wofs[w]] & keep[w];
                acc_or |= x;
                acc_and &= x;
            }
        any = acc_or != 0;
        all = acc_and == ~0u && t0 + p.bq <= p.T && u0 + p.bk <= p.T;
    }
    const unsigned long long ba = __ballot(any), bl = __ballot(all);
    if (lane == 0 || lane == 32) {
        const int w = chunk * 2 + (lane >> 5);
        if (w < p.words) {
            p.any_bits[(long long)q * p.words + w] = (unsigned)(ba >> lane);
            p.all_bits[(long long)q * p.words + w] = (unsigned)(bl >> lane);
        }
    }
}

int block_bitmap_words(const Problem &pb)
{
    const long long nk = (long long)pb.NB * pb.b / pb.bk;
    return (int)((nk + 31) / 32);
}

stream_status launch_block_bitmaps(const Problem &pb, unsigned *any_bits, unsigned *all_bits, hipStream_t st)
{
    BitmapParams p;
    p.cbits = pb.cbits; p.cpitch = pb.cpitch;
    p.any_bits = any_bits; p.all_bits = all_bits;
    p.T = (int)pb.T; p.bq = pb.b; p.bk = pb.bk;
    p.nq = pb.NB; p.nk = (int)((long long)pb.NB * pb.b / pb.bk);
    p.words = block_bitmap_words(pb);
    if (pb.NB > 65535) return STREAM_EUNSUPPORTED;                 // grid.y
    const dim3 grid((unsigned)((p.nk + 255) / 256), (unsigned)pb.NB);
    if (pb.bk == 32) hipLaunchKernelGGL(block_bitmap_kernel<1>, grid, dim3(256), 0, st, p);
    else if (pb.bk == 64) hipLaunchKernelGGL(block_bitmap_kernel<2>, grid, dim3(256), 0, st, p);
    else hipLaunchKernelGGL(block_bitmap_kernel<4>, grid, dim3(256), 0, st, p);
    return hipGetLastError() == hipSuccess ? STREAM_OK : STREAM_EDEVICE;
}

}  // namespace stream

extern "C" {

long long stream_num_blocks(const stream_shape *shape)
{
    stream::Problem pb;
    if (stream::make_problem(shape, 0, nullptr, 0, &pb) != STREAM_OK) return -1;
    return pb.NB;
}

long long stream_num_key_blocks(const stream_shape *shape)
{
    stream::Problem pb;
    if (stream::make_problem(shape, 0, nullptr, 0, &pb) != STREAM_OK) return -1;
    return (long long)pb.NB * pb.b / pb.bk;
}

int stream_prune_levels(const stream_shape *shape, int topk, const int *topk_per_seq)
{
    stream::Problem pb;
    if (stream::make_problem(shape, topk, topk_per_seq, stream::kMaxTopkWide, &pb) != STREAM_OK)
        return -1;
    return pb.max_levels;
}

const char *stream_status_str(stream_status s)
{
    switch (s) {
    case STREAM_OK: return "ok";
    case STREAM_EINVAL: return "invalid argument";
    case STREAM_EUNSUPPORTED: return "unsupported configuration";
    case STREAM_EWORKSPACE: return "workspace missing, misaligned or too small";
    case STREAM_EDEVICE: return "HIP error";
    }
    return "unknown status";
}

}  // extern "C"
