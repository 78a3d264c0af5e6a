// The library used from plain C++ through its C ABI alone (no Python, no torch): device buffers
// from hipMalloc, one stream_prune + stream_sparse_attn on a small causal problem, checks of the
// laws that hold for any input (cnt = min(k, q+1), ascending causal ids, rows of P sum to 1,
// finite outputs).  Exit code 0 = all checks passed.  Run by tests/test_gpu_c_abi.py.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "stream.h"

#define HIP_OK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { std::printf("HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__); return 2; } } while (0)
#define CHECK(c) do { if (!(c)) { std::printf("check failed: %s (line %d)\n", #c, __LINE__); return 1; } } while (0)

static uint64_t rng_state = 0x2510198750ull;
static float uniform() { rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull; return (float)((rng_state >> 40) & 0xffffff) / 8388608.0f - 1.0f; }

int main()
{
    const int H = 4, Hkv = 2, d = 64, b = 64, k = 4;
    const long long T = 64 * 20 + 17;
    stream_shape s;
    std::memset(&s, 0, sizeof s);                     // causal mask, b_k = b_q, contiguous strides
    s.heads = H; s.kv_heads = Hkv; s.head_dim = d; s.block = b; s.dtype = STREAM_F32; s.batch = 1; s.T = T;
    const long long NB = stream_num_blocks(&s);
    CHECK(NB == 21);
    std::vector<float> q((size_t)H * T * d), kk((size_t)Hkv * T * d), v((size_t)Hkv * T * d);
    for (auto &x : q) x = uniform();
    for (auto &x : kk) x = uniform();
    for (auto &x : v) x = uniform();
    float *Q, *K, *V, *O, *lse, *mass, *score;
    int *idx, *cnt;
    void *wp, *wa;
    const size_t wpb = stream_prune_workspace_bytes(&s, k), wab = stream_sparse_attn_workspace_bytes(&s, k);
    CHECK(wpb > 0 && wab > 0);
    HIP_OK(hipMalloc(&Q, q.size() * 4)); HIP_OK(hipMalloc(&K, kk.size() * 4)); HIP_OK(hipMalloc(&V, v.size() * 4));
    HIP_OK(hipMalloc(&O, q.size() * 4)); HIP_OK(hipMalloc(&lse, (size_t)H * T * 4)); HIP_OK(hipMalloc(&mass, (size_t)H * T * 4));
    HIP_OK(hipMalloc(&idx, (size_t)H * NB * k * 4)); HIP_OK(hipMalloc(&cnt, (size_t)H * NB * 4));
    HIP_OK(hipMalloc(&score, (size_t)H * NB * k * 4));
    HIP_OK(hipMalloc(&wp, wpb)); HIP_OK(hipMalloc(&wa, wab));
    HIP_OK(hipMemcpy(Q, q.data(), q.size() * 4, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(K, kk.data(), kk.size() * 4, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(V, v.data(), v.size() * 4, hipMemcpyHostToDevice));
    hipStream_t st;
    HIP_OK(hipStreamCreate(&st));

    // argument errors come back as codes, before any launch
    CHECK(stream_prune(nullptr, K, &s, k, nullptr, k, idx, cnt, score, nullptr, wp, wpb, st) == STREAM_EINVAL);
    CHECK(stream_prune(Q, K, &s, k, nullptr, k, idx, cnt, score, nullptr, wp, wpb - 1, st) == STREAM_EWORKSPACE);

    CHECK(stream_prune(Q, K, &s, k, nullptr, k, idx, cnt, score, nullptr, wp, wpb, st) == STREAM_OK);
    CHECK(stream_sparse_attn(Q, K, V, &s, idx, cnt, k, 0.125f, O, lse, mass, wa, wab, st) == STREAM_OK);
    HIP_OK(hipStreamSynchronize(st));

    std::vector<int> hidx((size_t)H * NB * k), hcnt((size_t)H * NB);
    std::vector<float> hO(q.size()), hl((size_t)H * T), hm((size_t)H * T), hs((size_t)H * NB * k);
    HIP_OK(hipMemcpy(hidx.data(), idx, hidx.size() * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(hcnt.data(), cnt, hcnt.size() * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(hs.data(), score, hs.size() * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(hO.data(), O, hO.size() * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(hl.data(), lse, hl.size() * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(hm.data(), mass, hm.size() * 4, hipMemcpyDeviceToHost));
    for (int h = 0; h < H; ++h)
        for (long long qb = 0; qb < NB; ++qb) {
            const int c = hcnt[h * NB + qb];
            CHECK(c == (qb + 1 < k ? (int)qb + 1 : k));
            for (int j = 0; j < k; ++j) {
                const int r = hidx[(h * NB + qb) * k + j];
                if (j < c) {
                    CHECK(r >= 0 && r <= qb && (j == 0 || r > hidx[(h * NB + qb) * k + j - 1]));
                    CHECK(std::isfinite(hs[(h * NB + qb) * k + j]));
                } else {
                    CHECK(r == -1);
                }
            }
        }
    for (int h = 0; h < H; ++h) {
        double total = 0.0;
        for (long long t = 0; t < T; ++t) {
            CHECK(std::isfinite(hl[h * T + t]) && hm[h * T + t] >= 0.f);
            total += hm[h * T + t];
            for (int c = 0; c < d; ++c) CHECK(std::fabs(hO[(h * T + t) * d + c]) <= 1.0001f);   // a convex combination of V rows
        }
        CHECK(std::fabs(total - (double)T) < 1e-3 * T);
    }
    std::printf("c abi smoke ok: NB=%lld, prune workspace %zu B, attention workspace %zu B\n", NB, wpb, wab);
    return 0;
}
