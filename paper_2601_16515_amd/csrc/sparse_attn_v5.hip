// Block-sparse softmax attention (Eq. (2)) with the fused linear apply / scale / sum epilogue,
// d = 128 (and d = 64 on half-size tiles).  Large tile, deep LDS prefetch, ping-pong wave groups.
//
//   * One workgroup = 8 waves = 256 query positions = 4 CSR rows of one (batch, head); one workgroup
//     per CU (LDS: 4 K + 5 V tiles of 16 KB plus the block list; registers at d = 64, where the tiles are 8 KB).
//   * The ascending union of the 4 rows' kept-block lists is built once per workgroup in LDS (bitmap +
//     ballot compaction), each entry carrying a 4-bit "kept by query block i" mask.  The main loop
//     reads one entry per iteration from LDS; no global or scalar load sits on its critical path.
//   * K and V tiles go straight from global memory into a ring of LDS slots PD blocks ahead of their
//     use, PD = 3 (global_load_lds_dwordx4, bank swizzle applied on the global side).  The wait before the
//     per-block barrier is counted (s_waitcnt vmcnt(n)), so PD - 1 blocks of loads stay in flight and
//     L2 / fabric latency is covered without a second resident workgroup.
//   * Ping-pong: waves 0-3 (group 0) and 4-7 (group 1) share the 4 SIMDs pairwise.  Per KV block a wave
//     has a matrix part (O += V^T P of the previous block, S = K Q^T of the current one: 32 MFMAs) and a
//     vector part (softmax of S, then the address arithmetic and issue of the next prefetch).  Group 0
//     runs matrix then vector, group 1 vector then matrix, so that one wave of a SIMD feeds the matrix
//     pipe while the other uses the vector ALU.  One barrier per KV block (it also protects the ring).
//   * V^T operands come from ds_read_b64_tr_b16, K rows are read through the kappa permutation so
//     that P never moves between lanes.  LDS operand reads are spread evenly between the MFMAs through a
//     small ring of fragment registers.
//   * Softmax with few vector instructions: logits live in the log2 domain (one fma and one v_exp_f32 per
//     element); row sums are taken from the bf16-rounded probabilities with v_dot2c_f32_bf16; the block
//     maximum is not computed unless a block's sums show that some logit exceeds the running reference
//     by more than 13 binades (the reference then moves to the true maximum and the block is redone).
//   * Epilogue: the bf16 fragments of the linear state are staged once per workgroup in LDS.
#include "salad_internal.h"

namespace salad {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef short s16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

#define LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))
#define GLB_PTR(p) ((const __attribute__((address_space(1))) void *)(p))
#define TR_READ(p) __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)LDS_PTR(p))
#define INL __attribute__((always_inline))
// s_waitcnt with only vmcnt constrained (gfx9 encoding: vmcnt[3:0] | expcnt 7 << 4 | lgkmcnt 15 << 8)
#define WAIT_VM(n) __builtin_amdgcn_s_waitcnt(0x0F70 | (n))

namespace {

__device__ inline int row_of_position5(int kind, int p, int T, int HW, unsigned magic)
{
    if (!kind) return p;
    const int loc = (int)__umulhi((unsigned)p, magic);   // exact p / T (the host checks the range)
    return (p - loc * T) * HW + loc;
}

__device__ inline uint32_t pack2e(float a, float b)
{
    f32x2 x = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf16x2));
}

__device__ inline uint32_t relu2e(uint32_t x)
{
    s16x2 v = __builtin_bit_cast(s16x2, x);
    s16x2 z = {0, 0};
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(v, z));
}

// One 16-byte-per-lane global -> LDS load (lane i lands at lds_addr + 16 i).  Issued through inline
// assembly so that the compiler's automatic "wait for every pending LDS load before any LDS read"
// does not apply: which loads must have landed is known exactly and waited for with WAIT_VM below.
__device__ inline void lds_dma16(const void *gptr, unsigned lds_addr_uniform)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :
                 : "s"(lds_addr_uniform), "v"(gptr)
                 : "memory", "m0");
}

// Same, addressed as (wave-uniform 64-bit base) + (per-lane unsigned 32-bit byte offset): no 64-bit
// vector arithmetic per load.
__device__ inline void lds_dma16_base(const void *base_uniform, unsigned byte_off, unsigned lds_addr_uniform)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr_uniform), "v"(byte_off), "s"(base_uniform)
                 : "memory", "m0");
}

__device__ inline unsigned lds_addr_of(const void *p)
{
    return __builtin_amdgcn_readfirstlane((unsigned)(size_t)LDS_PTR(p));
}

// max of a value with its copy in the other 32-lane half, on the VALU (v_permlane32_swap): the LDS
// unit, which a cross-lane shuffle would go through, is saturated by the other group's operand reads.
__device__ inline float max_with_other_half(float x)
{
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// acc + lo(w) + hi(w) for a packed pair of bf16 (dot product with (1, 1), fp32 accumulate).  Chains of these
// on one accumulator need no wait; any other instruction reading the result needs four idle slots first
// (see the s_nop where the sums are consumed).
__device__ inline float add_bf16_pair(float acc, uint32_t w)
{
    asm("v_dot2c_f32_bf16 %0, %1, %2" : "+v"(acc) : "v"(w), "v"(0x3f803f80u));
    return acc;
}

union Frag5 {
    bf16x8 v;
    uint4 u;
    uint32_t w[4];
    s16x4 h[2];
};

}  // namespace

// Pre-pass: for every (head, tile of 4 query blocks) the union of the 4 CSR rows' kept blocks, each entry
// tagged with which of the 4 rows keep it.  One wave per tile: bitmap in LDS, ordered compaction with
// ballots, then the ascending list is rotated so that it starts at the entry whose block id is smallest
// modulo the list length.  Softmax does not care about the order, and with sliding windows the rotation makes
// neighbouring tiles (which run at the same time on one XCD and whose windows overlap) reach a given KV
// block at about the same iteration, so the block is fetched into that XCD's L2 once instead of once per
// tile.  The mask is static, but the layer call accepts any CSR, so this runs per call (a few microseconds).
__global__ __launch_bounds__(64) void tile_lists_kernel(const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ col_idx,
                                                        int nb, int ntiles, int cap, uint32_t *__restrict__ lists,
                                                        int32_t *__restrict__ counts)
{
    extern __shared__ uint32_t bm[];          // [cap] bitmap, then [cap] compacted list
    uint32_t *lst = bm + cap;
    __shared__ uint32_t best;
    const int h = blockIdx.y, tile = blockIdx.x, lane = threadIdx.x;
    for (int i = lane; i < nb; i += 64) bm[i] = 0u;
    if (lane == 0) best = 0xffffffffu;
    __syncthreads();
    for (int i = 0; i < 4; ++i) {
        const int r = tile * 4 + i;
        if (r < nb) {
            const int b0 = row_ptr[h * nb + r], b1 = row_ptr[h * nb + r + 1];
            for (int e = b0 + lane; e < b1; e += 64) {
                const int c = col_idx[e];
                if (c >= 0 && c < nb) atomicOr(&bm[c], 1u << (24 + i));
            }
        }
    }
    __syncthreads();
    int count = 0;
    for (int base = 0; base < nb; base += 64) {
        const int b = base + lane;
        const uint32_t f = b < nb ? bm[b] : 0u;
        const unsigned long long bal = __ballot(f != 0u);
        const int pos = count + __popcll(bal & ((1ull << lane) - 1ull));
        if (f) lst[pos] = (uint32_t)b | f;
        count += __popcll(bal);
    }
    __syncthreads();
    // rotation point: the entry with the smallest (block id mod count); ties cannot occur within count
    // consecutive ids, and for any other list the lowest position wins
    for (int i = lane; i < count; i += 64) {
        const uint32_t key = (lst[i] & 0xffffffu) % (uint32_t)count;
        atomicMin(&best, (key << 13) | (uint32_t)i);      // at most 6144 entries (list size limit checked on the host)
    }
    __syncthreads();
    const int rot = count > 0 ? (int)(best & 0x1fffu) : 0;
    uint32_t *out = lists + ((size_t)h * ntiles + tile) * cap;
    for (int i = lane; i < count; i += 64) {
        int src = i + rot;
        if (src >= count) src -= count;
        out[i] = lst[src];
    }
    if (lane == 0) counts[h * ntiles + tile] = count;
}

int tile_list_cap(int nb) { return (nb + 63) & ~63; }

hipError_t launch_tile_lists(const int32_t *row_ptr, const int32_t *col_idx, int H, int nb, uint32_t *lists,
                             int32_t *counts, hipStream_t st)
{
    const int ntiles = (nb + 3) / 4;
    const int cap = tile_list_cap(nb);
    launch_kernel(tile_lists_kernel, dim3(ntiles, H), dim3(64), (size_t)cap * 8, st, row_ptr, col_idx, nb, ntiles, cap, lists, counts);
    return take_launch_status();
}

// PD: prefetch distance in KV blocks.  K(b) is read in iteration b only, V(b) also in iteration b+1: the K ring
// has PD + 1 slots, the V ring PD + 2.
// MODE 0: block rows (CSR) through the per-tile union lists.
// MODE 1: token-level Top-K mask (App. A.1.2).  The tile lists are per (sample, head, tile); an entry is
//   block | key-block index << 16 | wave mask << 24 (bit 24 + w: some query of wave w keeps the block); each lane
//   tests its own query's bit of a.topk_mask and contributes nothing for a block it did not select.
// MODE 2: Top-K regrouped by key block.  A query tile is a run of up to 256 gathered queries that all keep the same
//   key block; the list is that key block's 64-token blocks; the normalised partial result and its log-sum-exp go
//   to a.g_po / a.g_lse (one slot per kept (query, key block) pair) for the merge kernel.
// ROPE (MODE 0 only): rotary position embedding inside the linear branch (Sec. 4.1).  The state fragments then hold
//   sum_j (R_j relu(K_j))^T V_j, and the epilogue rotates this tile's relu(Q) fragments in registers (channel pair
//   (2p, 2p+1) of the query's stored row n by the angle word a.rope_tab[n * 64 + p] = fp16 cos | fp16 sin << 16) after
//   the normaliser has been taken from the unrotated features.
// D = 64 (MODE 0 without ROPE only): the same kernel on half-size tiles.  A row is 8 chunks of 16 bytes instead of 16,
// so one pass of the 512 threads fetches a whole 64-row tile, the swizzles below take the row pair instead of the row
// (rows 128 bytes apart alternate between the two halves of the banks), and every fragment count halves.
template <int D, int PD, bool DBG, int MODE = 0, bool ROPE = false>
__global__ __launch_bounds__(512, 2) void sparse_attn_v5_kernel(AttnArgs a, int ntiles, int total, int per_xcd, int list_cap)
{
    static_assert(D == 128 || (D == 64 && MODE == 0 && !ROPE), "d = 64 has the CSR mode only");
    constexpr int NS = D / 16, NDT = D / 32;     // 16-channel steps of S, 32-channel tiles of O^T
    constexpr int CH = D / 8;                    // 16-byte chunks per row
    constexpr int RPP = 512 / CH, NPASS = 64 / RPP;   // rows per pass of the 512 threads over a tile, passes per tile
    constexpr int TILE = 64 * D;                 // elements
    constexpr int NK = PD + 1, NV = PD + 2;
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    u16 *Kb = reinterpret_cast<u16 *>(smem);                       // NK tiles
    u16 *Vb = Kb + NK * TILE;                                       // NV tiles
    uint32_t *blist = reinterpret_cast<uint32_t *>(Vb + NV * TILE);      // [list_cap] union list: blk | mask << 24

    constexpr bool TOPK = MODE == 1, GATHER = MODE == 2;
    // chunk swizzles of the K tile, the V tile and the output staging as functions of the row
    auto kswz = [](int row) INL -> int { return D == 128 ? (row & 15) : ((row >> 1) & 7); };
    auto vswz = [](int row) INL -> int { return D == 128 ? ((row & 3) << 2) : (((row >> 1) & 1) << 2); };
    const int g = blockIdx.x;
    const int L = (g & 7) * per_xcd + (g >> 3);
    if (L >= total) return;
    int bh = L / ntiles, tile = L - bh * ntiles;
    int g_J = 0, g_slot0 = 0, g_cnt = 0;
    if (GATHER) {
        const uint4 dsc = a.g_desc[L];
        bh = (int)dsc.x; g_J = (int)dsc.y; g_slot0 = (int)dsc.z; g_cnt = (int)dsc.w;
        if (g_cnt == 0) return;            // unused descriptor
        tile = 0;
    }
    const int h = bh % a.H;
    const int N = a.N, T = a.T, HW = a.HW, nb = a.nb;
    const int kind = (T > 1 && !TOPK) ? (int)((a.kind_mask >> h) & 1ull) : 0;
    const unsigned magic = a.t_magic;
    constexpr uint32_t BLKMASK = TOPK ? 0xffffu : 0xffffffu;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hh = lane >> 5;
    const int group = wave >> 2;
    const u16 *qb = reinterpret_cast<const u16 *>(a.q) + (size_t)bh * N * D;
    const u16 *kb = reinterpret_cast<const u16 *>(a.k) + (size_t)bh * N * D;
    const u16 *vb = reinterpret_cast<const u16 *>(a.v) + (size_t)bh * N * D;

    const int qsub = wave >> 1;
    const int qblk = tile * 4 + qsub;
    unsigned mybit = qblk < nb ? (1u << (24 + (TOPK ? (wave & 7) : qsub))) : 0u;
    const int qpos = qblk * 64 + (wave & 1) * 32 + l32;
    bool qvalid = (qblk < nb) && (qpos < N);
    int qrow;
    size_t g_slot = 0;                    // GATHER: this lane's (query, key block) pair
    if (GATHER) {
        const int qi = wave * 32 + l32;   // position in the run of gathered queries
        qvalid = qi < g_cnt;
        mybit = wave * 32 < g_cnt ? (1u << (24 + (wave & 7))) : 0u;
        g_slot = (size_t)bh * N * a.g_kk + g_slot0 + (qvalid ? qi : 0);
        qrow = a.g_idx[g_slot];
        qrow = min(max(qrow, 0), N - 1);
    } else {
        qrow = row_of_position5(kind, qvalid ? qpos : N - 1, T, HW, magic);
    }

    Frag5 qf[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s)
        qf[s].u = *reinterpret_cast<const uint4 *>(qb + (size_t)qrow * D + s * 16 + hh * 8);

    // ---- this tile's union list (built by the pre-pass): the whole row of list_cap slots is copied, so
    // the copy does not wait for the count (slots past the count hold stale words that are never used)
    const int g_blk0 = g_J * a.g_bpb;
    const int n = GATHER ? min(min(nb, g_blk0 + a.g_bpb) - g_blk0, list_cap) : a.tile_counts[(TOPK ? bh : h) * ntiles + tile];
    uint32_t qm_lo = 0u, qm_hi = 0u;     // TOPK: this lane's query's key-block bits
    if (TOPK && qvalid) {
        const unsigned long long m = a.topk_mask[(size_t)bh * N + qrow];
        qm_lo = (uint32_t)m;
        qm_hi = (uint32_t)(m >> 32);
    }
    if (GATHER) {
        for (int i = tid; i < list_cap; i += 512) blist[i] = (uint32_t)min(g_blk0 + i, nb - 1) | 0xff000000u;
    } else {
        const uint32_t *src = a.tile_lists + ((size_t)(TOPK ? bh : h) * ntiles + tile) * list_cap;
        for (int i = tid; i < list_cap; i += 512) blist[i] = src[i];
    }
    __syncthreads();
    // Retire the Q loads here: inside the loop the only vector-memory operations in flight must be the
    // K/V prefetches, whose completion is tracked by hand.
#pragma unroll
    for (int s = 0; s < NS; ++s)
        asm volatile("" : "+v"(qf[s].w[0]), "+v"(qf[s].w[1]), "+v"(qf[s].w[2]), "+v"(qf[s].w[3]));
    asm volatile("" : "+v"(qm_lo), "+v"(qm_hi));

    const float c2 = a.scale * 1.44269504088896340736f;   // logits are handled in the log2 domain

    // ---- global -> LDS: thread owns LDS slots (row RPP i + tid/CH, chunk tid%CH), i < NPASS, of a tile.
    // LDS destinations are wave-uniform scalars; global sources are a uniform base plus a 32-bit offset.
    const int lr = tid / CH, pc = tid % CH;
    const unsigned kchunk_b = (unsigned)((pc ^ kswz(lr)) * 16);
    const unsigned vchunk_b = (unsigned)((pc ^ vswz(lr)) * 16);
    const unsigned wave_u = (unsigned)__builtin_amdgcn_readfirstlane(wave);
    const unsigned k_lds0 = lds_addr_of(Kb) + wave_u * 1024u;
    const unsigned v_lds0 = lds_addr_of(Vb) + wave_u * 1024u;
    auto fetch = [&](int blk, int kslot, int vslot) INL {
        const unsigned kl = k_lds0 + (unsigned)kslot * (unsigned)(TILE * 2);
        const unsigned vl = v_lds0 + (unsigned)vslot * (unsigned)(TILE * 2);
#pragma unroll
        for (int i = 0; i < NPASS; ++i) {
            int p = blk * 64 + i * RPP + lr;
            p = p < N ? p : N - 1;
            const unsigned row_b = (unsigned)row_of_position5(kind, p, T, HW, magic) * (unsigned)(D * 2);
            lds_dma16_base(kb, row_b + kchunk_b, kl + i * 8192u);
            lds_dma16_base(vb, row_b + vchunk_b, vl + i * 8192u);
        }
    };
    // list entries travel in a vector register (lane l holds entry 64 c + l of the current 64-entry
    // chunk c) and are picked with v_readlane: no LDS round trip per iteration
    uint32_t ev = blist[lane];
    auto entry = [&](int idx) INL -> uint32_t { return (uint32_t)__builtin_amdgcn_readlane((int)ev, idx & 63); };

    // ---- LDS operand addresses (element offsets inside a tile)
    const int kappa = (l32 & 0x13) | ((l32 & 4) << 1) | ((l32 & 8) >> 1);
    int koff[NS];
#pragma unroll
    for (int st = 0; st < NS; ++st) koff[st] = kappa * D + (((2 * st + hh) ^ kswz(kappa)) << 3);
    const int vr = 8 * hh + ((l32 >> 2) & 3);
    int voff[NDT];
#pragma unroll
    for (int dt = 0; dt < NDT; ++dt) {
        int chunk = 4 * dt + 2 * (l32 >> 4) + ((l32 & 3) >> 1);
        voff[dt] = vr * D + ((chunk ^ vswz(vr)) << 3) + 4 * (l32 & 1);
    }

    f32x16 o[NDT];
#pragma unroll
    for (int i = 0; i < NDT; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[i][r] = 0.f;
    float m_run = 0.f, l_run = 0.f;
    bool have_ref = false;                 // m_run has been set from a block's true maximum (wave-uniform unless TOPK)
    f32x16 s[2];
    Frag5 pf[4];

    // Matrix phase = 32 MFMAs per wave: 16 for O^T += V^T P^T (A = V^T fragment: two transposing 8-byte reads),
    // then 16 for S^T = K Q^T (A = K fragment: one 16-byte read; the NS products of the block's first 32 keys, then
    // those of the other 32, so that the softmax finds its first logits finished).  Operand fragments move through a ring of
    // RING register quads: MFMA i takes ring[i % RING] and the read of fragment i + RING is issued right after
    // it, so LDS requests are spread evenly over the phase (the LDS has to deliver 1 KB per MFMA per wave,
    // about three quarters of what it can sustain, and bursts of reads stall the matrix pipe) and at most
    // 2 RING <= 15 of them are in flight.  The first RING fragments are requested in the preceding vector
    // phase, once the V tile they come from is known to have landed.
    constexpr int RING = 7;
    Frag5 ring[RING];
    constexpr int NPV = 4 * NDT, NSTEP = NPV + 2 * NS;     // PV steps (4 key groups x NDT), all steps of a block
    auto read_frag = [&](int i, const u16 *Vt, const u16 *Kt, Frag5 &f) INL {
        if (i < NPV) {
            const u16 *vp = Vt + (i / NDT) * 16 * D + voff[i % NDT];
            f.h[0] = TR_READ(vp);
            f.h[1] = TR_READ(vp + 4 * D);
        } else {
            const int t = i - NPV;
            f.v = *reinterpret_cast<const bf16x8 *>(Kt + (t / NS) * 32 * D + koff[t % NS]);
        }
    };
    auto mfma_step = [&](int i, const Frag5 &f) INL {
        if (i < NPV) {
            o[i % NDT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.v, pf[i / NDT].v, o[i % NDT], 0, 0, 0);
        } else {
            const int t = i - NPV, kt = t / NS, st = t % NS;   // the first 32 keys' logits are complete NS MFMAs before the phase ends
            if (st == 0) {
                f32x16 z;
#pragma unroll
                for (int r = 0; r < 16; ++r) z[r] = 0.f;
                s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.v, qf[st].v, z, 0, 0, 0);
            } else {
                s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.v, qf[st].v, s[kt], 0, 0, 0);
            }
        }
    };
    auto preload_V = [&](const u16 *Vt) INL {      // fragments 0 .. RING-1 (all of them V^T fragments)
#pragma unroll
        for (int i = 0; i < RING; ++i) read_frag(i, Vt, nullptr, ring[i]);
    };
    // steps FIRST .. LAST-1 of the sequence; ring[(FIRST + k) % RING], k < RING, already requested
    auto run_steps = [&](const u16 *Vt, const u16 *Kt, int first, int last) INL {
#pragma unroll
        for (int i = first; i < last; ++i) {
            mfma_step(i, ring[i % RING]);
            if (i + RING < last) read_frag(i + RING, Vt, Kt, ring[i % RING]);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    auto stage_PV_S = [&](const u16 *Vt, const u16 *Kt) INL { run_steps(Vt, Kt, 0, NSTEP); };
    auto stage_PV = [&](const u16 *Vt) INL { run_steps(Vt, nullptr, 0, NPV); };
    auto stage_S = [&](const u16 *Kt) INL {          // rare (first block of a row, blocks another row's mask drops)
#pragma unroll
        for (int i = 0; i < RING; ++i) read_frag(NPV + i, nullptr, Kt, ring[(NPV + i) % RING]);
        run_steps(nullptr, Kt, NPV, NSTEP);
    };
    auto stage_softmax = [&](uint32_t e) INL {
        const int blk = (int)(e & BLKMASK);
        // TOPK: a lane whose query did not select this key block gets P = 0 (scale 0, reference +inf) and takes
        // no part in the reference updates
        bool sel = true;
        if (TOPK) {
            const int J = (int)((e >> 16) & 63u);
            sel = (((J & 32) ? qm_hi : qm_lo) >> (J & 31)) & 1u;
        }
        const float cs = (TOPK && !sel) ? 0.f : c2;
        const float ms = (TOPK && !sel) ? INFINITY : m_run;
        if (blk * 64 + 64 > N) {
            const int kbase = blk * 64 + hh * 8;
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (kbase + kt * 32 + 16 * (r >> 3) + (r & 7) >= N) s[kt][r] = TOPK ? -1e30f : -INFINITY;   // TOPK: stays finite times a zero scale
        }
        // P = 2^(S c2 - m) rounded to bf16; returns the lane's sum of the rounded values (what the PV product sees)
        auto exp_pack = [&]() INL -> float {
            float ps0 = 0.f, ps1 = 0.f;
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int r = 0; r < 16; r += 2) {
                    const float mref = TOPK ? (sel ? m_run : ms) : m_run;
                    const uint32_t w = pack2e(__builtin_amdgcn_exp2f(fmaf(s[kt][r], cs, -mref)),
                                              __builtin_amdgcn_exp2f(fmaf(s[kt][r + 1], cs, -mref)));
                    pf[kt * 2 + (r >> 3)].w[(r & 7) >> 1] = w;
                    if (r & 2) ps1 = add_bf16_pair(ps1, w); else ps0 = add_bf16_pair(ps0, w);
                }
            // the dot instructions come from inline assembly, so the compiler does not know that another
            // vector instruction must not read their result in the next four issue slots
            asm volatile("s_nop 4" : "+v"(ps0), "+v"(ps1));
            return ps0 + ps1;
        };
        // The reference only has to keep 2^S in range, so the block maximum is not computed unless the
        // sums say that some logit rose more than 13 binades above the reference (or no reference exists
        // yet): then the reference moves to the true maximum and the block is redone.
        float psum = 0.f;
        bool redo = sel && !have_ref;
        if (!redo) {
            psum = exp_pack();
            redo = __any(!(psum <= 8192.f)) && sel;
        }
        if (redo) {
            float mx = s[0][0];
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kt][r]);
            mx = fmaf(fmaxf(max_with_other_half(mx), -1e30f), c2, -m_run);   // block maximum minus reference
            const float shift = have_ref ? fmaxf(mx, 0.f) : mx;                // new reference minus old reference
            if (have_ref) {
                const float alpha = __builtin_amdgcn_exp2f(-shift);
                l_run *= alpha;
#pragma unroll
                for (int i = 0; i < NDT; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o[i][r] *= alpha;
            }
            m_run += shift;
            have_ref = true;
            psum = exp_pack();
        }
        l_run += psum;
    };

    const bool lin = !GATHER && a.use_linear && !a.write_sparse_only && !(a.drop && a.drop[bh / a.H]);   // pruned sample (Sec. 4.3): out = O_s
    const u16 *hf = a.hfrag + (size_t)bh * D * D;
    // the D x D linear-state fragments (32 KB at d = 128) for the epilogue, staged into the K ring once it is idle
    auto stage_state = [&]() INL {
#pragma unroll
        for (int i = 0; i < D * D / (512 * 8); ++i) lds_dma16(hf + (size_t)(i * 512 + tid) * 8, lds_addr_of(Kb + (i * 512 + wave * 64) * 8));
    };

    // ROPE: this lane's 32 angle words (its query's row of the table: pairs 8 st + 4 hh + j), fetched under the last
    // PV product of the tile
    uint4 ang[ROPE ? NS : 1];
    auto load_angles = [&]() INL {
        if (ROPE) {
            const uint32_t *tr = a.rope_tab + (size_t)qrow * (D / 2) + hh * 4;
#pragma unroll
            for (int st = 0; st < NS; ++st) ang[st] = *reinterpret_cast<const uint4 *>(tr + st * 8);
        }
    };

    // ---- main loop over the union list.  Iteration j: S(j) and softmax(j), PV(j-1); fetch block j+PD.
    // Block b lives in slot b % NK of the K ring and b % NV of the V ring.
    // The fetch of block j+PD is issued from each group's vector phase, where its address arithmetic
    // runs under the other group's MFMAs; the slots it goes to were last read in iteration j-1.
    int v_last = 0;                         // V-ring slot of the last block: the only tile still read after the loop
    if (n > 0) {
#pragma unroll
        for (int b = 0; b < PD; ++b)
            if (b < n) fetch((int)(entry(b) & BLKMASK), b, b);
        uint32_t e_prev = 0u;
        uint32_t eq[PD];                          // eq[i] = entry j + i
#pragma unroll
        for (int b = 0; b < PD; ++b) eq[b] = b < n ? entry(b) : 0u;
        int kslot = 0, vslot = 0;                 // j % NK, j % NV
        for (int j = 0; j < n; ++j) {
            // all fetches up to block j must have landed; newer ones may stay in flight
            {
                int newer = n - 1 - j;
                if (newer > PD - 1) newer = PD - 1;
                constexpr int LPB = 2 * NPASS;          // loads per lane and block (K and V, NPASS each)
                if (newer >= 3) WAIT_VM(3 * LPB);
                else if (newer == 2) WAIT_VM(2 * LPB);
                else if (newer == 1) WAIT_VM(LPB);
                else WAIT_VM(0);
            }
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            const int jf = j + PD;
            uint32_t e_f = 0u;
            if (jf < n) {
                if ((jf & 63) == 0) ev = blist[jf + lane];
                e_f = entry(jf);
            }
            const bool do_fetch = jf < n;
            int kslot_f = kslot + PD; if (kslot_f >= NK) kslot_f -= NK;
            int vslot_f = vslot + PD; if (vslot_f >= NV) vslot_f -= NV;
            int vslot_prev = vslot - 1; if (vslot_prev < 0) vslot_prev += NV;
            const uint32_t e_cur = eq[0];
            const bool kS = (e_cur & mybit) != 0, kP = (j >= 1) && (e_prev & mybit);
            const u16 *Kt = Kb + kslot * TILE;
            const u16 *Vt = Vb + vslot_prev * TILE;
            const u16 *Vc = Vb + vslot * TILE;         // V tile of block j (already landed with K(j))
            if (group == 0) {
                if (kP && kS) stage_PV_S(Vt, Kt);
                else { if (kP) stage_PV(Vt); if (kS) stage_S(Kt); }
                asm volatile("" ::: "memory");
                if (kS) preload_V(Vc);                  // for PV(j) in the next iteration; lands under the softmax
                if (kS) stage_softmax(e_cur);
                if (do_fetch) fetch((int)(e_f & BLKMASK), kslot_f, vslot_f);
            } else {
                if (kP) preload_V(Vt);                  // for PV(j-1) right after the barrier; lands under the softmax
                if (kP) stage_softmax(e_prev);
                if (do_fetch) fetch((int)(e_f & BLKMASK), kslot_f, vslot_f);
                asm volatile("" ::: "memory");
                if (kP && kS) stage_PV_S(Vt, Kt);
                else { if (kP) stage_PV(Vt); if (kS) stage_S(Kt); }
            }
            e_prev = e_cur;
#pragma unroll
            for (int b = 0; b + 1 < PD; ++b) eq[b] = eq[b + 1];
            eq[PD - 1] = e_f;
            ++kslot; if (kslot >= NK) kslot = 0;
            ++vslot; if (vslot >= NV) vslot = 0;
        }
        // tail: the PV product of the last block (group 1 still owes its softmax).  The K ring is idle
        // from here on, so the epilogue's state fragments are fetched into it under these MFMAs.
        WAIT_VM(0);
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if (lin) stage_state();
        if (ROPE && lin) load_angles();
        {
            int vslot_prev = vslot - 1; if (vslot_prev < 0) vslot_prev += NV;
            v_last = vslot_prev;
            const u16 *Vt = Vb + vslot_prev * TILE;
            const bool kP = (e_prev & mybit) != 0;
            if (group == 1 && kP) { preload_V(Vt); stage_softmax(e_prev); }
            if (kP) stage_PV(Vt);
        }
    }

    // ---- epilogue ---------------------------------------------------------------------------------
    float l_tot = l_run + __shfl_xor(l_run, 32);
    const float inv_l = l_tot > 0.f ? 1.f / l_tot : 0.f;
    f32x16 num[NDT];
    float lin_scale = 0.f, inv_den = 0.f;
    if (lin) {
        if (n == 0) { stage_state(); if (ROPE) load_angles(); }
        float dpart = 0.f;
        const float *Zh = a.Z + (size_t)bh * D;
#pragma unroll
        for (int st = 0; st < NS; ++st) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                uint32_t w = relu2e(qf[st].w[j]);
                qf[st].w[j] = w;
                dpart = fmaf(__uint_as_float(w << 16), Zh[st * 16 + hh * 8 + 2 * j], dpart);
                dpart = fmaf(__uint_as_float(w & 0xffff0000u), Zh[st * 16 + hh * 8 + 2 * j + 1], dpart);
            }
        }
        const float den = dpart + __shfl_xor(dpart, 32) + a.eps;
        inv_den = 1.f / den;
        lin_scale = a.coef[bh] * inv_den;
        WAIT_VM(0);
        if (ROPE) {
            // numerator operand: R_i relu(Q_i), rounded to bf16 like every MFMA operand (the normaliser above keeps the
            // unrotated features)
#pragma unroll
            for (int st = 0; st < NS; ++st) {
                const uint32_t cw[4] = {ang[st].x, ang[st].y, ang[st].z, ang[st].w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t w = qf[st].w[j];
                    const float x = __uint_as_float(w << 16), y = __uint_as_float(w & 0xffff0000u);
                    const f16x2 hcs = __builtin_bit_cast(f16x2, cw[j]);
                    const float cc = (float)hcs[0], ss = (float)hcs[1];
                    qf[st].w[j] = pack2e(x * cc - y * ss, x * ss + y * cc);
                }
            }
        }
        __syncthreads();   // the staged fragments have landed in every wave's view
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt) {
#pragma unroll
            for (int r = 0; r < 16; ++r) num[dt][r] = 0.f;
#pragma unroll
            for (int st = 0; st < NS; ++st) {
                const int idx = ((dt * NS + st) * 64 + lane) * 8;
                bf16x8 hi = *reinterpret_cast<const bf16x8 *>(Kb + idx);
                num[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(hi, qf[st].v, num[dt], 0, 0, 0);
            }
        }
    }
    if (!DBG) {
        // bf16 results leave through LDS so that every global store is a run of full 256-byte rows: accumulator
        // layout (lane = query l32; 4 consecutive columns per (dt, g4, hh)) -> a wave-private 8 KB of the V ring
        // (the four slots that do not hold the last block: nobody reads them any more), 16-byte chunk c of row r at
        // r * 256 + ((c ^ (r & 15)) << 4) -> row layout (4 rows x 16 chunks per instruction).
        int vs = v_last + 1 + (wave >> 1);
        if (vs >= NV) vs -= NV;
        constexpr int ROWB = D * 2;          // bytes of a row
        unsigned char *stg = reinterpret_cast<unsigned char *>(Vb + vs * TILE) + (wave & 1) * (32 * ROWB);
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                float ov[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const float os = o[dt][g4 * 4 + t] * inv_l;
                    ov[t] = lin ? fmaf(num[dt][g4 * 4 + t], lin_scale, os) : os;
                }
                uint2 pk;
                pk.x = pack2e(ov[0], ov[1]);
                pk.y = pack2e(ov[2], ov[3]);
                *reinterpret_cast<uint2 *>(stg + l32 * ROWB + (((dt * 4 + g4) ^ kswz(l32)) << 4) + hh * 8) = pk;
            }
        asm volatile("" ::: "memory");       // the wave's LDS operations execute in order
        // destination of row r: the stored row (or the pair slot) of the lane that owns query r
        const int dest_mine = !qvalid ? -1 : GATHER ? g_slot0 + wave * 32 + l32 : qrow;
        constexpr int RPI = 64 / CH;          // rows per store instruction (4 rows x 16 chunks, or 8 x 8)
        const int r4 = lane / CH, c16 = lane % CH;
        u16 *dbase = GATHER ? a.g_po + (size_t)bh * N * a.g_kk * D : reinterpret_cast<u16 *>(a.out) + (size_t)bh * N * D;
#pragma unroll
        for (int i = 0; i < 32 / RPI; ++i) {
            const int r = RPI * i + r4;
            const uint4 v = *reinterpret_cast<const uint4 *>(stg + r * ROWB + ((c16 ^ kswz(r)) << 4));
            const int dest = __shfl(dest_mine, r);
            if (dest >= 0) *reinterpret_cast<uint4 *>(dbase + (size_t)dest * D + c16 * 8) = v;
        }
        if (GATHER && qvalid && hh == 0) a.g_lse[g_slot] = l_tot > 0.f ? m_run + log2f(l_tot) : -INFINITY;
    } else {
    if (!qvalid) return;
    const size_t obase = ((size_t)bh * N + qrow) * D;
    u16 *outp = reinterpret_cast<u16 *>(a.out) + obase;
#pragma unroll
    for (int dt = 0; dt < NDT; ++dt) {
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
            const int col = dt * 32 + 8 * g4 + 4 * hh;
            float os[4], ol[4], ov[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                os[t] = o[dt][g4 * 4 + t] * inv_l;
                ol[t] = lin ? num[dt][g4 * 4 + t] : 0.f;
                ov[t] = lin ? fmaf(ol[t], lin_scale, os[t]) : os[t];
            }
            uint2 pk;
            pk.x = pack2e(ov[0], ov[1]);
            pk.y = pack2e(ov[2], ov[3]);
            *reinterpret_cast<uint2 *>(outp + col) = pk;
            if (DBG && a.o_sparse_dbg)
                *reinterpret_cast<float4 *>(a.o_sparse_dbg + obase + col) = make_float4(os[0], os[1], os[2], os[3]);
            if (DBG && a.o_linear_dbg && lin)
                *reinterpret_cast<float4 *>(a.o_linear_dbg + obase + col) =
                    make_float4(ol[0] * inv_den, ol[1] * inv_den, ol[2] * inv_den, ol[3] * inv_den);
        }
    }
    }
}

template <int PD, bool DBG, int MODE = 0, bool ROPE = false, int D = 128>
static hipError_t launch_v5(const AttnArgs &a, hipStream_t st)
{
    const int ntiles = (a.nb + 3) / 4;
    const int total = MODE == 2 ? a.g_max_tiles : a.B * a.H * ntiles;
    const int per_xcd = (total + 7) / 8;
    const int list_cap = (a.nb + 63) & ~63;
    const size_t lds = (size_t)(2 * PD + 3) * 64 * D * 2 + (size_t)list_cap * 4;
    static_assert(PD + 1 >= 2, "the epilogue stages the state fragments (two tiles' worth) in the K ring");
    constexpr int kMaxDyn = 160 * 1024 - 2048;   // the static part is rounded up to its 1 KB alignment
    if (lds > (size_t)kMaxDyn) return hipErrorInvalidValue;
    auto kern = sparse_attn_v5_kernel<D, PD, DBG, MODE, ROPE>;
    static bool attr_done[16] = {};
    if (hipError_t e = dyn_lds_attr_once(reinterpret_cast<const void *>(kern), kMaxDyn, attr_done); e != hipSuccess) return e;
    launch_kernel(kern, dim3(per_xcd * 8), dim3(512), lds, st, a, ntiles, total, per_xcd, list_cap);
    return take_launch_status();
}

hipError_t launch_sparse_attn_v5(const AttnArgs &a, hipStream_t st)
{
    const bool dbg = a.o_sparse_dbg || a.o_linear_dbg;
    if (a.D == 64) {
        if (a.g_desc || a.topk_mask || a.rope_tab) return hipErrorInvalidValue;
        return dbg ? launch_v5<3, true, 0, false, 64>(a, st) : launch_v5<3, false, 0, false, 64>(a, st);
    }
    if (a.g_desc) return launch_v5<3, false, 2>(a, st);
    if (a.topk_mask) return dbg ? launch_v5<3, true, 1>(a, st) : launch_v5<3, false, 1>(a, st);
    if (a.rope_tab) return dbg ? launch_v5<3, true, 0, true>(a, st) : launch_v5<3, false, 0, true>(a, st);
    return dbg ? launch_v5<3, true>(a, st) : launch_v5<3, false>(a, st);
}

}  // namespace salad
