// Top-K dynamic block mask (Sec. 3 "Top-K attention", App. A.1.2), d = 128, bf16.
//   step 1  kblock_mean_kernel      mean key of every run of key_block consecutive stored tokens
//   step 2  topk_select_kernel      per query token: the topk key blocks with the largest q . mean, as a 64-bit mask
//           topk_tile_lists_kernel  per tile of 256 queries: the 64-token blocks the attention kernel has to visit
//   step 3  the large-tile attention kernel in its token-mask mode
// The selection is an integer decided by floating point, so its arithmetic is fixed: fp32 throughout, a block's sum
// taken token by token in ascending order and divided by the token count, a score accumulated over the channels in
// ascending order with a fused multiply-add, a block replaces a kept one only on a strictly larger score (ties go
// to the lower index).  No fast-math: the division and the fused multiply-adds are the IEEE ones.
#include "salad_internal.h"

namespace salad {

namespace {
constexpr int D = 128;
__device__ inline float bf16_to_f32(u16 x) { return __uint_as_float((uint32_t)x << 16); }
}  // namespace

// grid (nbk, BH), 128 threads: thread c sums channel c of the block's keys in token order.
__global__ __launch_bounds__(128) void kblock_mean_kernel(const u16 *__restrict__ k, int N, int key_block, int nbk,
                                                          float *__restrict__ means)
{
    const int J = blockIdx.x, bh = blockIdx.y, c = threadIdx.x;
    const int t0 = J * key_block, t1 = min(N, t0 + key_block);
    const u16 *src = k + ((size_t)bh * N + t0) * D + c;
    float sum = 0.f;
    int t = t0;
    for (; t + 16 <= t1; t += 16) {           // 16 independent loads in flight, added in token order
        u16 x[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) x[i] = src[(size_t)i * D];
#pragma unroll
        for (int i = 0; i < 16; ++i) sum = __fadd_rn(sum, bf16_to_f32(x[i]));
        src += 16 * D;
    }
    for (; t < t1; ++t) {
        sum = __fadd_rn(sum, bf16_to_f32(*src));
        src += D;
    }
    means[((size_t)bh * nbk + J) * D + c] = __fdiv_rn(sum, (float)(t1 - t0));
}

hipError_t launch_kblock_mean(const u16 *k, int BH, int N, int key_block, int nbk, float *means, hipStream_t st)
{
    hipLaunchKernelGGL(kblock_mean_kernel, dim3(nbk, BH), dim3(128), 0, st, k, N, key_block, nbk, means);
    return hipGetLastError();
}

// grid (ceil(N / 256), BH), 256 threads: a thread owns one query; the block means are the same for every lane
// (scalar loads).  The best 8 scores are kept in descending order; the first topk of them are the selection.
__global__ __launch_bounds__(256) void topk_select_kernel(const u16 *__restrict__ q, const float *__restrict__ means,
                                                          int N, int nbk, int topk,
                                                          unsigned long long *__restrict__ mask)
{
    const int bh = blockIdx.y;
    const int n = blockIdx.x * 256 + threadIdx.x;
    const int nr = n < N ? n : N - 1;
    float qv[D];
    {
        const uint4 *src = reinterpret_cast<const uint4 *>(q + ((size_t)bh * N + nr) * D);
#pragma unroll
        for (int i = 0; i < D / 8; ++i) {
            const uint4 u = src[i];
            const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                qv[i * 8 + 2 * j] = __uint_as_float(w[j] << 16);
                qv[i * 8 + 2 * j + 1] = __uint_as_float(w[j] & 0xffff0000u);
            }
        }
    }
    float best[8];
    int bidx[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) { best[i] = -INFINITY; bidx[i] = -1; }
    const float *mrow = means + (size_t)bh * nbk * D;
    for (int J = 0; J < nbk; ++J) {
        float sc = 0.f;
#pragma unroll
        for (int c = 0; c < D; ++c) sc = __fmaf_rn(qv[c], mrow[c], sc);
        mrow += D;
        // bubble the new pair down the descending list; a strict comparison keeps earlier blocks ahead on ties.
        // An empty slot (index -1) always gives way, whatever the score (-inf scores included).
        float v = sc;
        int id = J;
        bool carry = false;                    // once placed, the displaced pairs all move down one slot
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const bool take = (id >= 0) && (carry || bidx[i] < 0 || v > best[i]);
            carry = carry || take;
            const float tv = best[i];
            const int ti = bidx[i];
            best[i] = take ? v : tv;
            bidx[i] = take ? id : ti;
            v = take ? tv : v;
            id = take ? ti : id;
        }
    }
    unsigned long long m = 0ull;
#pragma unroll
    for (int i = 0; i < 8; ++i)
        if (i < topk && bidx[i] >= 0) m |= 1ull << bidx[i];
    if (n < N) mask[(size_t)bh * N + n] = m;
}

hipError_t launch_topk_select(const u16 *q, const float *means, int BH, int N, int nbk, int topk,
                              unsigned long long *mask, hipStream_t st)
{
    hipLaunchKernelGGL(topk_select_kernel, dim3((N + 255) / 256, BH), dim3(256), 0, st, q, means, N, nbk, topk, mask);
    return hipGetLastError();
}

// grid (ntiles, BH), 256 threads: thread t holds the mask of query 256 tile + t; attention wave w of the tile owns
// queries 32 w .. 32 w + 31.  Entry = block | J << 16 | wave bits << 24, key blocks ascending, their 64-token
// blocks ascending.
__global__ __launch_bounds__(256) void topk_tile_lists_kernel(const unsigned long long *__restrict__ mask, int N, int nb,
                                                              int bpb, int nbk, int ntiles, int cap,
                                                              uint32_t *__restrict__ lists, int32_t *__restrict__ counts)
{
    __shared__ unsigned long long wmask[8];
    __shared__ int offs[65];
    const int tile = blockIdx.x, bh = blockIdx.y, t = threadIdx.x, lane = t & 63;
    const int n = tile * 256 + t;
    unsigned long long m = n < N ? mask[(size_t)bh * N + n] : 0ull;
    // OR over each run of 32 lanes
#pragma unroll
    for (int o = 1; o < 32; o <<= 1) {
        const uint32_t lo = __shfl_xor((uint32_t)m, o), hi = __shfl_xor((uint32_t)(m >> 32), o);
        m |= ((unsigned long long)hi << 32) | lo;
    }
    if ((lane & 31) == 0) wmask[t >> 5] = m;
    __syncthreads();
    if (t < 64) {
        unsigned long long u = 0ull;
#pragma unroll
        for (int w = 0; w < 8; ++w) u |= wmask[w];
        const int J = t;
        int cnt = 0;
        if (J < nbk && ((u >> J) & 1ull)) cnt = min(nb, (J + 1) * bpb) - J * bpb;
        // exclusive prefix sum over the 64 lanes
        int incl = cnt;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int x = __shfl_up(incl, o);
            if (lane >= o) incl += x;
        }
        offs[J] = incl - cnt;
        if (J == 63) offs[64] = incl;
    }
    __syncthreads();
    uint32_t *out = lists + ((size_t)bh * ntiles + tile) * cap;
    for (int J = 0; J < nbk; ++J) {
        const int o0 = offs[J], c = offs[J + 1] - o0;
        if (c == 0) continue;
        uint32_t bits = 0u;
#pragma unroll
        for (int w = 0; w < 8; ++w) bits |= (uint32_t)((wmask[w] >> J) & 1ull) << (24 + w);
        for (int i = t; i < c; i += 256) out[o0 + i] = (uint32_t)(J * bpb + i) | ((uint32_t)J << 16) | bits;
    }
    if (t == 0) counts[bh * ntiles + tile] = offs[64];
}

hipError_t launch_topk_tile_lists(const unsigned long long *mask, int BH, int N, int nb, int key_block, int nbk,
                                  uint32_t *lists, int32_t *counts, hipStream_t st)
{
    const int ntiles = (nb + 3) / 4;
    hipLaunchKernelGGL(topk_tile_lists_kernel, dim3(ntiles, BH), dim3(256), 0, st, mask, N, nb, key_block / 64, nbk,
                       ntiles, tile_list_cap(nb), lists, counts);
    return hipGetLastError();
}

}  // namespace salad
