// Declarations shared by the refinement kernels of stream_prune (stream_prune.hip: up to 64
// blocks kept per row, one node per lane; stream_prune_wide.hip: up to 512, nodes in LDS).
#pragma once

#include "stream_mfma.h"
#include "stream_select.h"

#include <math.h>

namespace stream {

constexpr int kMaxSweep = 32;        // values of k in one stream_prune_multi call
constexpr int kScoreCache = 1024;    // entries of a row's block-score cache (k sweep)

struct PruneParams {
    const char *Q;
    const char *Kp;              // packed K tiles [kv_head][global block][b * d]
    long long q_sh_b, q_st_b;    // byte strides of Q (head, token)
    int H, g, NB, kmax;
    int level_begin, level_end;  // 1-based refinement levels this launch runs for every row
    int max_levels;              // levels of the deepest row (length of the trace)
    int *nf, *nl;                // node ranges [H, NB, kmax]
    float *ns;                   // node scores (score of the node's representative block)
    int *ncnt;                   // live nodes per row [H, NB]
    int *idx, *cnt;              // outputs, written by a row's last level
    float *score;                // nullable
    unsigned long long *tiles;   // nullable diagnostic counter
    int *trace;                  // nullable diagnostic [max_levels, H, NB, kmax, 2]
    WgMap map;
    SeqTable seqs;
    int mask, window;            // the mask rule C (stream_mask) and its window
    // STREAM_MASK_ARRAY (ARB kernels): the bit array C, its block-level summaries [NB, cw] (any =
    // C^blk of Alg. 2, all = no token-level test needed) and the words per row of either
    const unsigned *cbits, *cany, *call;
    long long cpitch;
    int cw;
    int vk_num, vk_den, vk_min;  // variable k (vk_den > 0): k(row) = clamp(ceil(valid * num / den), min, kmax)
    int n_k;                     // k sweep (MULTI kernels): values of k, outputs [H, n_k, NB, ...]
    int klist[kMaxSweep];
    int wide_ki;                 // wide kernel in a sweep: which value of the list this launch runs
};

static_assert(sizeof(PruneParams) <= 4096, "kernel arguments are limited to 4 KB");

// max(1, ceil(log2(ceil(N / k)))): the levels after which every node is a single block
__host__ __device__ __forceinline__ int levels_for(int N, int k)
{
    const int per = (N + k - 1) / k;
    int lv = 0;
    for (long long v = 1; v < per; v <<= 1) ++lv;
    return lv < 1 ? 1 : lv;
}

// k of a row under the variable-k rule: a fixed share of the row's valid key blocks
__host__ __device__ __forceinline__ int variable_k(int valid, int num, int den, int kmin, int kmax)
{
    long long k = ((long long)valid * num + den - 1) / den;
    k = k < kmin ? kmin : k;
    return (int)(k > kmax ? kmax : k);
}

constexpr int kWideTopk = 512;       // blocks kept per row by the wide kernel (node lists in LDS)

// Runs every row's levels in one launch of the wide kernel (p.wide_ki selects the k of a sweep).
bool level_wide_supported(const Problem &pb);
stream_status launch_level_wide(const Problem &pb, const PruneParams &p, hipStream_t st);

}  // namespace stream
