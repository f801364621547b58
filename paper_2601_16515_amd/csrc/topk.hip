// Top-K dynamic block mask (Sec. 3 "Top-K attention", App. A.1.2), d = 128, bf16.
//   step 1  kblock_mean_kernel      mean key of every run of key_block consecutive tokens of the head's own order
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

// grid (nbk, BH), 128 threads: thread c sums channel c of the block's keys in the order of the head's positions
// (App. A.1.1: position p of a temporal head is stored row (p mod T) HW + p div T; a spatial head's is row p).
__global__ __launch_bounds__(128) void kblock_mean_kernel(const u16 *__restrict__ k, int N, int key_block, int nbk,
                                                          float *__restrict__ means, unsigned long long kind_mask, int H,
                                                          int T, int HW)
{
    const int J = blockIdx.x, bh = blockIdx.y, c = threadIdx.x;
    const int t0 = J * key_block, t1 = min(N, t0 + key_block);
    const bool temporal = T > 1 && ((kind_mask >> (bh % H)) & 1ull);
    const u16 *base = k + (size_t)bh * N * D + c;
    float sum = 0.f;
    int t = t0;
    if (!temporal) {
        const u16 *src = base + (size_t)t0 * D;   // one running address, the 16 rows at constant offsets from it
        for (; t + 16 <= t1; t += 16) {           // 16 independent loads in flight, added in position order
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
    } else {
        // position p = loc T + f (location loc, frame f) is stored row f HW + loc; the pair is stepped, not divided
        int loc = t0 / T, f = t0 - loc * T;
        auto next_row = [&]() {
            const int row = f * HW + loc;
            if (++f == T) { f = 0; ++loc; }
            return row;
        };
        for (; t + 16 <= t1; t += 16) {
            u16 x[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) x[i] = base[(size_t)next_row() * D];
#pragma unroll
            for (int i = 0; i < 16; ++i) sum = __fadd_rn(sum, bf16_to_f32(x[i]));
        }
        for (; t < t1; ++t) sum = __fadd_rn(sum, bf16_to_f32(base[(size_t)next_row() * D]));
    }
    means[((size_t)bh * nbk + J) * D + c] = __fdiv_rn(sum, (float)(t1 - t0));
}

hipError_t launch_kblock_mean(const u16 *k, int BH, int N, int key_block, int nbk, float *means, unsigned long long kind_mask,
                              int H, int T, int HW, hipStream_t st)
{
    launch_kernel(kblock_mean_kernel, dim3(nbk, BH), dim3(128), 0, st, k, N, key_block, nbk, means, kind_mask, H, T, HW);
    return take_launch_status();
}

// grid (ceil(N / 256), BH), 256 threads: a thread owns one query and keeps one score accumulator per key block
// (NBK of them, the smallest instantiation >= nbk: the chains are independent, each runs over the channels in
// ascending order).  The head's block means sit in LDS; every lane reads the same word (broadcast).  The best SLOTS
// (4 or 8, >= topk) scores are then collected in descending order, blocks in ascending order; the first topk of them
// are the selection.
template <int NBK, int SLOTS>
__global__ __launch_bounds__(256) void topk_select_kernel(const u16 *__restrict__ q, const float *__restrict__ means,
                                                          int N, int nbk, int topk,
                                                          unsigned long long *__restrict__ mask)
{
    __shared__ float sm[NBK * D];
    const int bh = blockIdx.y;
    const int n = blockIdx.x * 256 + threadIdx.x;
    const int nr = n < N ? n : N - 1;
    for (int i = threadIdx.x; i < NBK * D; i += 256) sm[i] = i < nbk * D ? means[(size_t)bh * nbk * D + i] : 0.f;
    __syncthreads();
    float sc[NBK];
#pragma unroll
    for (int J = 0; J < NBK; ++J) sc[J] = 0.f;
    const uint4 *src = reinterpret_cast<const uint4 *>(q + ((size_t)bh * N + nr) * D);
#pragma unroll 1
    for (int c64 = 0; c64 < D / 64; ++c64) {           // 64 channels = one 128-byte line of the query row at a time:
        uint4 u[8];                                    // its 8 loads go out together, so the line is fetched once
#pragma unroll
        for (int i = 0; i < 8; ++i) u[i] = src[c64 * 8 + i];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t w[4] = {u[i].x, u[i].y, u[i].z, u[i].w};
            float qv[8];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                qv[2 * j] = __uint_as_float(w[j] << 16);
                qv[2 * j + 1] = __uint_as_float(w[j] & 0xffff0000u);
            }
            const float *mc = sm + c64 * 64 + i * 8;
#pragma unroll
            for (int J = 0; J < NBK; ++J) {
                const float4 m0 = *reinterpret_cast<const float4 *>(mc + J * D);
                const float4 m1 = *reinterpret_cast<const float4 *>(mc + J * D + 4);
                float x = sc[J];
                x = __fmaf_rn(qv[0], m0.x, x); x = __fmaf_rn(qv[1], m0.y, x);
                x = __fmaf_rn(qv[2], m0.z, x); x = __fmaf_rn(qv[3], m0.w, x);
                x = __fmaf_rn(qv[4], m1.x, x); x = __fmaf_rn(qv[5], m1.y, x);
                x = __fmaf_rn(qv[6], m1.z, x); x = __fmaf_rn(qv[7], m1.w, x);
                sc[J] = x;
            }
        }
    }
    float best[SLOTS];                                 // SLOTS >= topk: 4 or 8
    int bidx[SLOTS];
#pragma unroll
    for (int i = 0; i < SLOTS; ++i) { best[i] = -INFINITY; bidx[i] = -1; }
#pragma unroll
    for (int J = 0; J < NBK; ++J) {
        if (J < nbk) {
            // bubble the pair down the descending list; a strict comparison keeps earlier blocks ahead on ties; an
            // empty slot (index -1) always gives way; once placed, the displaced pairs all move down one slot
            float v = sc[J];
            int id = J;
            bool carry = false;
#pragma unroll
            for (int i = 0; i < SLOTS; ++i) {
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
    }
    unsigned long long m = 0ull;
#pragma unroll
    for (int i = 0; i < SLOTS; ++i)
        if (i < topk && bidx[i] >= 0) m |= 1ull << bidx[i];
    if (n < N) mask[(size_t)bh * N + n] = m;
}

hipError_t launch_topk_select(const u16 *q, const float *means, int BH, int N, int nbk, int topk,
                              unsigned long long *mask, hipStream_t st)
{
    const dim3 grid((N + 255) / 256, BH), block(256);
#define SALAD_TOPK_SELECT(NBK_)                                                                                              \
    do {                                                                                                                     \
        if (topk <= 4) launch_kernel((topk_select_kernel<NBK_, 4>), grid, block, 0, st, q, means, N, nbk, topk, mask);  \
        else launch_kernel((topk_select_kernel<NBK_, 8>), grid, block, 0, st, q, means, N, nbk, topk, mask);            \
    } while (0)
    if (nbk <= 8) SALAD_TOPK_SELECT(8);
    else if (nbk <= 16) SALAD_TOPK_SELECT(16);
    else if (nbk <= 24) SALAD_TOPK_SELECT(24);
    else if (nbk <= 32) SALAD_TOPK_SELECT(32);
    else if (nbk <= 40) SALAD_TOPK_SELECT(40);
    else if (nbk <= 48) SALAD_TOPK_SELECT(48);
    else if (nbk <= 56) SALAD_TOPK_SELECT(56);
    else SALAD_TOPK_SELECT(64);
#undef SALAD_TOPK_SELECT
    return take_launch_status();
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
    launch_kernel(topk_tile_lists_kernel, dim3(ntiles, BH), dim3(256), 0, st, mask, N, nb, key_block / 64, nbk,
                       ntiles, tile_list_cap(nb), lists, counts);
    return take_launch_status();
}

// ---- regrouping by key block -----------------------------------------------------------------------------------
// The queries that keep key block J are gathered into runs of 256 ("query tiles" of the attention kernel), so that
// the work is the kept (query, key block) pairs whatever the selection looks like; every pair gets a slot in
// [0, N * kk) of its (sample, head), key blocks ascending, queries ascending inside a key block.

// Chunks of 1024 queries.  Wave w of a chunk publishes, for every key block J, the ballot of its 64 queries' bit J.
__device__ inline void chunk_ballots(unsigned long long m, int nbk, unsigned long long (*wb)[64], int wv, int lane)
{
    for (int J = 0; J < nbk; ++J) {
        const unsigned long long bal = __ballot((m >> J) & 1ull);
        if (lane == 0) wb[wv][J] = bal;
    }
}

// grid (nch, BH), 1024 threads: ccnt[(bh * nch + chunk) * 64 + J] = queries of the chunk keeping block J
__global__ __launch_bounds__(1024) void topk_count_kernel(const unsigned long long *__restrict__ mask, int N, int nbk,
                                                          int nch, int32_t *__restrict__ ccnt)
{
    __shared__ unsigned long long wb[16][64];
    const int chunk = blockIdx.x, bh = blockIdx.y, t = threadIdx.x, lane = t & 63, wv = t >> 6;
    const int n = chunk * 1024 + t;
    const unsigned long long m = n < N ? mask[(size_t)bh * N + n] : 0ull;
    chunk_ballots(m, nbk, wb, wv, lane);
    __syncthreads();
    if (t < 64) {
        int c = 0;
        if (t < nbk)
#pragma unroll
            for (int w = 0; w < 16; ++w) c += __popcll(wb[w][t]);
        ccnt[((size_t)bh * nch + chunk) * 64 + t] = c;
    }
}

// grid (BH), 64 threads (lane J = key block J).  cbase[(bh * nch + chunk) * 64 + J] = first slot (within the
// sample-head) of the chunk's queries keeping J = slots of key blocks < J + those of earlier chunks.  Tile descriptors
// (bh, J, first slot, queries) for every run of up to 256 queries, key blocks in order, at desc[bh * mt ...]; the
// unused descriptors of the sample-head's mt are written with zero queries (their workgroups return at once).
__global__ __launch_bounds__(64) void topk_plan_kernel(const int32_t *__restrict__ ccnt, int nbk, int nch,
                                                       int32_t *__restrict__ cbase, uint4 *__restrict__ desc, int mt)
{
    const int bh = blockIdx.x, J = threadIdx.x;
    // the per-chunk counts of this key block, 32 chunks' loads in flight at a time (the loop is latency-bound)
    const int32_t *cc = ccnt + (size_t)bh * nch * 64 + J;
    int c = 0;
    if (J < nbk)
        for (int ch0 = 0; ch0 < nch; ch0 += 32) {
            int x[32];
#pragma unroll
            for (int i = 0; i < 32; ++i) x[i] = ch0 + i < nch ? cc[(size_t)(ch0 + i) * 64] : 0;
#pragma unroll
            for (int i = 0; i < 32; ++i) c += x[i];
        }
    // exclusive prefix sums over the key blocks: slots and tiles
    const int tl = (c + 255) >> 8;
    int s_incl = c, t_incl = tl;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int xs = __shfl_up(s_incl, o), xt = __shfl_up(t_incl, o);
        if (J >= o) { s_incl += xs; t_incl += xt; }
    }
    const int s0 = s_incl - c, t0 = t_incl - tl;
    const int used = __shfl(t_incl, 63);
    if (J < nbk) {
        int run = s0;
        int32_t *cb = cbase + (size_t)bh * nch * 64 + J;
        for (int ch0 = 0; ch0 < nch; ch0 += 32) {
            int x[32];
#pragma unroll
            for (int i = 0; i < 32; ++i) x[i] = ch0 + i < nch ? cc[(size_t)(ch0 + i) * 64] : 0;
#pragma unroll
            for (int i = 0; i < 32; ++i) {
                if (ch0 + i < nch) cb[(size_t)(ch0 + i) * 64] = run;
                run += x[i];
            }
        }
        for (int i = 0; i < tl; ++i)
            if (t0 + i < mt)
                desc[(size_t)bh * mt + t0 + i] = make_uint4((uint32_t)bh, (uint32_t)J, (uint32_t)(s0 + i * 256), (uint32_t)min(256, c - i * 256));
    }
    for (int i = used + J; i < mt; i += 64) desc[(size_t)bh * mt + i] = make_uint4((uint32_t)bh, 0u, 0u, 0u);
}

// grid (nch, BH), 1024 threads: gidx[bh * slots + slot] = n and slot_of[(bh * N + n) * kk + r] = slot for every kept
// pair of the chunk; inside a key block the queries stay in ascending order (slot = chunk base + queries of lower
// waves + lower lanes keeping the block), r = rank of the block among the query's kept blocks.
__global__ __launch_bounds__(1024) void topk_group_kernel(const unsigned long long *__restrict__ mask, int N, int nbk, int kk,
                                                          int nch, const int32_t *__restrict__ cbase,
                                                          int32_t *__restrict__ gidx, int32_t *__restrict__ slot_of)
{
    __shared__ unsigned long long wb[16][64];
    __shared__ int wpre[16][64];
    const int chunk = blockIdx.x, bh = blockIdx.y, t = threadIdx.x, lane = t & 63, wv = t >> 6;
    const int n = chunk * 1024 + t;
    const size_t slots = (size_t)N * kk;
    unsigned long long m = n < N ? mask[(size_t)bh * N + n] : 0ull;
    chunk_ballots(m, nbk, wb, wv, lane);
    __syncthreads();
    {
        const int J = lane;                             // thread (wv, J): queries of lower waves keeping J
        int c = 0;
        if (J < nbk)
            for (int w = 0; w < wv; ++w) c += __popcll(wb[w][J]);
        wpre[wv][J] = c + (J < nbk ? cbase[((size_t)bh * nch + chunk) * 64 + J] : 0);
    }
    __syncthreads();
    int r = 0;
    while (m != 0ull && r < kk) {
        const int J = __ffsll((long long)m) - 1;
        m &= m - 1ull;
        if (J < nbk) {
            const int slot = wpre[wv][J] + __popcll(wb[wv][J] & ((1ull << lane) - 1ull));
            if (slot >= 0 && (size_t)slot < slots) {
                gidx[(size_t)bh * slots + slot] = n;
                slot_of[((size_t)bh * N + n) * kk + r] = slot;
            }
        }
        ++r;
    }
}

// out[bh, n, :] = sum_r w_r O_r / sum_r w_r over the query's kk partial results (normalised per key block, bf16, with
// log2-domain log-sum-exp lse_r), w_r = 2^(lse_r - max lse): Eq. (2) over the union of the kept blocks.
// 16 lanes per query (8 channels each) and two queries per thread, so that enough independent gathers are in flight
// (the chain mask -> slot -> partial row is three dependent loads); grid ceil(BH * N / 32), 256 threads.
__global__ __launch_bounds__(256) void topk_merge_kernel(const u16 *__restrict__ po, const float *__restrict__ lse,
                                                         const int32_t *__restrict__ slot_of,
                                                         const unsigned long long *__restrict__ mask, int BH, int N, int kk,
                                                         u16 *__restrict__ out, float *__restrict__ o_dbg)
{
    const size_t nq = (size_t)BH * N;
    const size_t q0 = (size_t)blockIdx.x * 32 + (threadIdx.x >> 4);
    const int c8 = (threadIdx.x & 15) * 8;
    const size_t slots = (size_t)N * kk;
    size_t qi[2];
    int cnt[2], sl[2][8];
    float l[2][8], mx[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        qi[u] = q0 + 16 * u;
        cnt[u] = qi[u] < nq ? min(kk, (int)__popcll(mask[qi[u]])) : 0;     // only the ranks the regrouping pass filled in
    }
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int r = 0; r < 8; ++r) sl[u][r] = r < cnt[u] ? slot_of[qi[u] * kk + r] : 0;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const size_t bh = qi[u] < nq ? qi[u] / N : 0;
        mx[u] = -INFINITY;
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            l[u][r] = r < cnt[u] ? lse[bh * slots + sl[u][r]] : -INFINITY;
            mx[u] = fmaxf(mx[u], l[u][r]);
        }
    }
    uint4 x[2][8];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const size_t bh = qi[u] < nq ? qi[u] / N : 0;
#pragma unroll
        for (int r = 0; r < 8; ++r)
            if (r < cnt[u]) x[u][r] = *reinterpret_cast<const uint4 *>(po + (bh * slots + sl[u][r]) * D + c8);
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        if (qi[u] >= nq) continue;
        float acc[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = 0.f;
        float den = 0.f;
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            if (r < cnt[u]) {
                const float wgt = __builtin_amdgcn_exp2f(l[u][r] - mx[u]);
                const uint32_t w4[4] = {x[u][r].x, x[u][r].y, x[u][r].z, x[u][r].w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    acc[2 * j] = fmaf(wgt, __uint_as_float(w4[j] << 16), acc[2 * j]);
                    acc[2 * j + 1] = fmaf(wgt, __uint_as_float(w4[j] & 0xffff0000u), acc[2 * j + 1]);
                }
                den += wgt;
            }
        }
        const float inv = den > 0.f ? 1.f / den : 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] *= inv;
        typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
        typedef float f32x2_t __attribute__((ext_vector_type(2)));
        uint4 pk;
        pk.x = __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2_t){acc[0], acc[1]}, bf16x2_t));
        pk.y = __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2_t){acc[2], acc[3]}, bf16x2_t));
        pk.z = __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2_t){acc[4], acc[5]}, bf16x2_t));
        pk.w = __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2_t){acc[6], acc[7]}, bf16x2_t));
        *reinterpret_cast<uint4 *>(out + qi[u] * D + c8) = pk;
        if (o_dbg) {
            *reinterpret_cast<float4 *>(o_dbg + qi[u] * D + c8) = make_float4(acc[0], acc[1], acc[2], acc[3]);
            *reinterpret_cast<float4 *>(o_dbg + qi[u] * D + c8 + 4) = make_float4(acc[4], acc[5], acc[6], acc[7]);
        }
    }
}

// query tiles per sample-head: every key block can leave one partly filled tile
int topk_tiles_per_head(int N, int kk, int nbk) { return (int)(((long long)N * kk + 255) / 256) + nbk; }
int topk_max_tiles(int BH, int N, int kk, int nbk) { return BH * topk_tiles_per_head(N, kk, nbk); }

hipError_t launch_topk_group(const unsigned long long *mask, int BH, int N, int nbk, int kk, int32_t *ccnt,
                             int32_t *cbase, uint4 *desc, int32_t *gidx, int32_t *slot_of, hipStream_t st)
{
    const int nch = (N + 1023) / 1024;
    launch_kernel(topk_count_kernel, dim3(nch, BH), dim3(1024), 0, st, mask, N, nbk, nch, ccnt);
    launch_kernel(topk_plan_kernel, dim3(BH), dim3(64), 0, st, ccnt, nbk, nch, cbase, desc, topk_tiles_per_head(N, kk, nbk));
    launch_kernel(topk_group_kernel, dim3(nch, BH), dim3(1024), 0, st, mask, N, nbk, kk, nch, cbase, gidx, slot_of);
    return take_launch_status();
}

hipError_t launch_topk_merge(const u16 *po, const float *lse, const int32_t *slot_of, const unsigned long long *mask,
                             int BH, int N, int kk, u16 *out, float *o_dbg, hipStream_t st)
{
    const size_t nq = (size_t)BH * N;
    launch_kernel(topk_merge_kernel, dim3((unsigned)((nq + 31) / 32)), dim3(256), 0, st, po, lse, slot_of, mask, BH, N, kk, out, o_dbg);
    return take_launch_status();
}

}  // namespace salad
