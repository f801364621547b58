// Block-sparse softmax attention (Eq. (2)) with the fused linear apply / scale / sum epilogue, d = 128, bf16.
// Variant with 64 queries per wave.
//
// The ping-pong kernel reads one 1 KB operand fragment from LDS for every MFMA (a wave owns 32 queries), which
// is what the LDS can just about deliver while four waves per CU run their matrix phases; its MFMA pipe waits
// on those reads.  Here a wave owns a whole 64-query block (two 32-query sub-tiles), so every K and V^T fragment
// read from LDS feeds two MFMAs and the LDS traffic per MFMA halves.  That takes 4 waves of 64 queries per
// 256-query tile: one wave per SIMD with the full 512-register file (accumulators in the upper half), no second
// wave to overlap with, so the softmax runs between the two MFMA runs of a block.
//
//   * workgroup = 4 waves = 256 query positions = 4 CSR rows of one (batch, head), one workgroup per CU; the same
//     per-tile union lists as the ping-pong kernel (entry = block | keep bits << 24, bit 24 + w for wave w);
//   * K and V tiles of a block go global -> LDS (DMA) PD = 3 blocks ahead into a ring of 4 slots of 32 KB; counted
//     waits, one barrier per KV block;
//   * per block and wave: S^T = K Q^T for both sub-tiles (16 K fragments, 32 MFMAs), softmax of both sub-tiles
//     (log2 domain, lazy reference, sums from the bf16-rounded probabilities), O^T += V^T P^T (16 V^T fragments,
//     32 MFMAs); operand fragments move through a small register ring so that LDS reads are spread between MFMAs;
//   * epilogue as in the ping-pong kernel: state fragments staged in the idle K slots, results leave through LDS
//     in full rows.
#include "salad_internal.h"

namespace salad {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef short s16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

#define LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))
#define TR_READ(p) __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)LDS_PTR(p))
#define INL __attribute__((always_inline))
// s_waitcnt with only vmcnt constrained (gfx9 encoding: vmcnt[3:0] | expcnt 7 << 4 | lgkmcnt 15 << 8 | vmcnt[5:4] << 14)
#define WAIT_VM7(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | (((n) >> 4) << 14))

namespace {

__device__ inline int row_of_position7(int kind, int p, int T, int HW, unsigned magic)
{
    if (!kind) return p;
    const int loc = (int)__umulhi((unsigned)p, magic);   // exact p / T (the host checks the range)
    return (p - loc * T) * HW + loc;
}

__device__ inline uint32_t pack2e7(float a, float b)
{
    f32x2 x = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf16x2));
}

__device__ inline uint32_t relu2e7(uint32_t x)
{
    s16x2 v = __builtin_bit_cast(s16x2, x);
    s16x2 z = {0, 0};
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(v, z));
}

// 16-byte-per-lane global -> LDS load (lane i lands at lds_addr + 16 i), addressed as a wave-uniform 64-bit base
// plus a per-lane unsigned 32-bit byte offset; inline assembly, so its completion is tracked by hand (WAIT_VM7).
__device__ inline void lds_dma16_base7(const void *base_uniform, unsigned byte_off, unsigned lds_addr_uniform)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr_uniform), "v"(byte_off), "s"(base_uniform)
                 : "memory", "m0");
}

__device__ inline void lds_dma16_7(const void *gptr, unsigned lds_addr_uniform)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(lds_addr_uniform), "v"(gptr) : "memory", "m0");
}

__device__ inline unsigned lds_addr_of7(const void *p)
{
    return __builtin_amdgcn_readfirstlane((unsigned)(size_t)LDS_PTR(p));
}

__device__ inline float max_with_other_half7(float x)
{
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// acc + lo(w) + hi(w) for a packed pair of bf16 (dot product with (1, 1), fp32 accumulate); any other instruction
// reading the result needs four idle slots first (see the s_nop where the sums are consumed)
__device__ inline float add_bf16_pair7(float acc, uint32_t w)
{
    asm("v_dot2c_f32_bf16 %0, %1, %2" : "+v"(acc) : "v"(w), "v"(0x3f803f80u));
    return acc;
}

union Frag7 {
    bf16x8 v;
    uint4 u;
    uint32_t w[4];
    s16x4 h[2];
};

}  // namespace

template <int PD, bool DBG>
__global__ __launch_bounds__(256, 1) void sparse_attn_v7_kernel(AttnArgs a, int ntiles, int total, int per_xcd, int list_cap)
{
    constexpr int D = 128, NS = 8, NDT = 4, NQ = 2;
    constexpr int TILE = 64 * D;                 // elements
    constexpr int NSLOT = PD + 1;
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    u16 *Kb = reinterpret_cast<u16 *>(smem);                       // NSLOT K tiles
    u16 *Vb = Kb + NSLOT * TILE;                                    // NSLOT V tiles
    uint32_t *blist = reinterpret_cast<uint32_t *>(Vb + NSLOT * TILE);   // [list_cap] union list: blk | mask << 24

    const int g = blockIdx.x;
    const int L = (g & 7) * per_xcd + (g >> 3);
    if (L >= total) return;
    const int bh = L / ntiles, tile = L - bh * ntiles;
    const int h = bh % a.H;
    const int N = a.N, T = a.T, HW = a.HW, nb = a.nb;
    const int kind = T > 1 ? (int)((a.kind_mask >> h) & 1ull) : 0;
    const unsigned magic = a.t_magic;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hh = lane >> 5;
    const u16 *qb = reinterpret_cast<const u16 *>(a.q) + (size_t)bh * N * D;
    const u16 *kb = reinterpret_cast<const u16 *>(a.k) + (size_t)bh * N * D;
    const u16 *vb = reinterpret_cast<const u16 *>(a.v) + (size_t)bh * N * D;

    const int qblk = tile * 4 + wave;
    const unsigned mybit = qblk < nb ? (1u << (24 + wave)) : 0u;
    bool qvalid[NQ];
    int qrow[NQ];
    Frag7 qf[NQ][NS];
#pragma unroll
    for (int qt = 0; qt < NQ; ++qt) {
        const int qpos = qblk * 64 + qt * 32 + l32;
        qvalid[qt] = (qblk < nb) && (qpos < N);
        qrow[qt] = row_of_position7(kind, qvalid[qt] ? qpos : N - 1, T, HW, magic);
#pragma unroll
        for (int s = 0; s < NS; ++s)
            qf[qt][s].u = *reinterpret_cast<const uint4 *>(qb + (size_t)qrow[qt] * D + s * 16 + hh * 8);
    }

    // this tile's union list (built by the pre-pass); the whole row of list_cap slots is copied
    const int n = a.tile_counts[h * ntiles + tile];
    {
        const uint32_t *src = a.tile_lists + ((size_t)h * ntiles + tile) * list_cap;
        for (int i = tid; i < list_cap; i += 256) blist[i] = src[i];
    }
    __syncthreads();
    // retire the Q loads here: inside the loop the only vector-memory operations in flight are the K/V prefetches
#pragma unroll
    for (int qt = 0; qt < NQ; ++qt)
#pragma unroll
        for (int s = 0; s < NS; ++s)
            asm volatile("" : "+v"(qf[qt][s].w[0]), "+v"(qf[qt][s].w[1]), "+v"(qf[qt][s].w[2]), "+v"(qf[qt][s].w[3]));

    const float c2 = a.scale * 1.44269504088896340736f;   // logits are handled in the log2 domain

    // ---- global -> LDS: thread owns LDS slots (row 16 i + tid/16, chunk tid%16), i = 0..3, of a tile
    const int lr = tid >> 4, pc = tid & 15;
    const unsigned kchunk_b = (unsigned)((pc ^ (lr & 15)) * 16);
    const unsigned vchunk_b = (unsigned)((pc ^ ((lr & 3) << 2)) * 16);
    const unsigned wave_u = (unsigned)__builtin_amdgcn_readfirstlane(wave);
    const unsigned k_lds0 = lds_addr_of7(Kb) + wave_u * 1024u;
    const unsigned v_lds0 = lds_addr_of7(Vb) + wave_u * 1024u;
    auto fetch = [&](int blk, int slot) INL {     // 8 loads per lane
        const unsigned kl = k_lds0 + (unsigned)slot * (unsigned)(TILE * 2);
        const unsigned vl = v_lds0 + (unsigned)slot * (unsigned)(TILE * 2);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int p = blk * 64 + i * 16 + lr;
            p = p < N ? p : N - 1;
            const unsigned row_b = (unsigned)row_of_position7(kind, p, T, HW, magic) * (unsigned)(D * 2);
            lds_dma16_base7(kb, row_b + kchunk_b, kl + i * 4096u);
            lds_dma16_base7(vb, row_b + vchunk_b, vl + i * 4096u);
        }
    };
    uint32_t ev = blist[lane];
    auto entry = [&](int idx) INL -> uint32_t { return (uint32_t)__builtin_amdgcn_readlane((int)ev, idx & 63); };

    // ---- LDS operand addresses (element offsets inside a tile), as in the ping-pong kernel
    const int kappa = (l32 & 0x13) | ((l32 & 4) << 1) | ((l32 & 8) >> 1);
    // K fragment of d-step st: row kappa, 16-byte chunk (2 st + hh) ^ (kappa & 15) = offset koff0 ^ (st << 4);
    // V^T fragment of d-tile dt: chunk (4 dt + c0) ^ ((vr & 3) << 2) = offset voff0 ^ (dt << 5)
    const int koff0 = kappa * D + ((hh ^ (kappa & 15)) << 3);
    const int vr = 8 * hh + ((l32 >> 2) & 3);
    const int voff0 = vr * D + (((2 * (l32 >> 4) + ((l32 & 3) >> 1)) ^ ((vr & 3) << 2)) << 3) + 4 * (l32 & 1);

    f32x16 o[NQ][NDT];
#pragma unroll
    for (int qt = 0; qt < NQ; ++qt)
#pragma unroll
        for (int i = 0; i < NDT; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[qt][i][r] = 0.f;
    float m_run[NQ] = {0.f, 0.f}, l_run[NQ] = {0.f, 0.f};
    bool have_ref[NQ] = {false, false};
    f32x16 s[NQ][2];
    Frag7 pf[NQ][4];

    // Operand fragments move through a ring of RING register quads: step i takes ring[i % RING] and the read of
    // fragment i + RING is issued right after it.  Steps 0..15: K fragment (kt = i & 1, st = i >> 1), two MFMAs
    // into S; steps 16..31: V^T fragment (kk = (i - 16) >> 2, dt = (i - 16) & 3), two MFMAs into O.
    constexpr int RING = 4;
    Frag7 ring[RING];
    auto read_frag = [&](int i, const u16 *Kt, const u16 *Vt, Frag7 &f) INL {
        if (i < 16) {
            f.v = *reinterpret_cast<const bf16x8 *>(Kt + (i & 1) * 32 * D + (koff0 ^ ((i >> 1) << 4)));
        } else {
            const int t = i - 16;
            const u16 *vp = Vt + (t >> 2) * 16 * D + (voff0 ^ ((t & 3) << 5));
            f.h[0] = TR_READ(vp);
            f.h[1] = TR_READ(vp + 4 * D);
        }
    };
    auto mfma_step = [&](int i, const Frag7 &f) INL {
        if (i < 16) {
            const int kt = i & 1, st = i >> 1;
#pragma unroll
            for (int qt = 0; qt < NQ; ++qt) {
                if (st == 0) {
                    f32x16 z;
#pragma unroll
                    for (int r = 0; r < 16; ++r) z[r] = 0.f;
                    s[qt][kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.v, qf[qt][st].v, z, 0, 0, 0);
                } else {
                    s[qt][kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.v, qf[qt][st].v, s[qt][kt], 0, 0, 0);
                }
            }
        } else {
            const int t = i - 16;
#pragma unroll
            for (int qt = 0; qt < NQ; ++qt)
                o[qt][t & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.v, pf[qt][t >> 2].v, o[qt][t & 3], 0, 0, 0);
        }
    };
    auto run_steps = [&](const u16 *Kt, const u16 *Vt, int first, int last) INL {
#pragma unroll
        for (int i = first; i < last; ++i) {
            mfma_step(i, ring[i % RING]);
            if (i + RING < last) read_frag(i + RING, Kt, Vt, ring[i % RING]);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    auto softmax = [&](int qt, int blk) INL {
        if (blk * 64 + 64 > N) {
            const int kbase = blk * 64 + hh * 8;
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (kbase + kt * 32 + 16 * (r >> 3) + (r & 7) >= N) s[qt][kt][r] = -INFINITY;
        }
        // P = 2^(S c2 - m) rounded to bf16; returns the lane's sum of the rounded values (what the PV product sees)
        auto exp_pack = [&]() INL -> float {
            float ps0 = 0.f, ps1 = 0.f;
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int r = 0; r < 16; r += 2) {
                    const uint32_t w = pack2e7(__builtin_amdgcn_exp2f(fmaf(s[qt][kt][r], c2, -m_run[qt])),
                                               __builtin_amdgcn_exp2f(fmaf(s[qt][kt][r + 1], c2, -m_run[qt])));
                    pf[qt][kt * 2 + (r >> 3)].w[(r & 7) >> 1] = w;
                    if (r & 2) ps1 = add_bf16_pair7(ps1, w); else ps0 = add_bf16_pair7(ps0, w);
                }
            asm volatile("s_nop 4" : "+v"(ps0), "+v"(ps1));
            return ps0 + ps1;
        };
        // lazy reference: the block maximum is computed only when no reference exists yet or the sums show that
        // some logit rose more than 13 binades above it (then the reference moves and the block is redone)
        float psum = 0.f;
        bool redo = !have_ref[qt];
        if (!redo) {
            psum = exp_pack();
            redo = __any(!(psum <= 8192.f));
        }
        if (redo) {
            float mx = s[qt][0][0];
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[qt][kt][r]);
            mx = fmaf(fmaxf(max_with_other_half7(mx), -1e30f), c2, -m_run[qt]);   // block maximum minus reference
            const float shift = have_ref[qt] ? fmaxf(mx, 0.f) : mx;
            if (have_ref[qt]) {
                const float alpha = __builtin_amdgcn_exp2f(-shift);
                l_run[qt] *= alpha;
#pragma unroll
                for (int i = 0; i < NDT; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o[qt][i][r] *= alpha;
            }
            m_run[qt] += shift;
            have_ref[qt] = true;
            psum = exp_pack();
        }
        l_run[qt] += psum;
    };

    const bool lin = a.use_linear && !a.write_sparse_only && !(a.drop && a.drop[bh / a.H]);   // pruned sample (Sec. 4.3): out = O_s
    const u16 *hf = a.hfrag + (size_t)bh * 2 * D * D;
    auto stage_state = [&]() INL {      // 64 KB of linear-state fragments (hi, lo) into the idle K slots
#pragma unroll
        for (int i = 0; i < 16; ++i) lds_dma16_7(hf + (size_t)(i * 256 + tid) * 8, lds_addr_of7(Kb + (i * 256 + wave * 64) * 8));
    };

    // ---- main loop over the union list.  Block b lives in slot b % NSLOT; iteration j: barrier, fetch of block
    // j + PD (into the slot read in iteration j - 1), S(j), softmax(j), PV(j).
    if (n > 0) {
#pragma unroll
        for (int b = 0; b < PD; ++b)
            if (b < n) fetch((int)(entry(b) & 0xffffffu), b);
        uint32_t eq[PD];
#pragma unroll
        for (int b = 0; b < PD; ++b) eq[b] = b < n ? entry(b) : 0u;
        int slot = 0;
        for (int j = 0; j < n; ++j) {
            {   // all fetches up to block j must have landed; newer ones (8 loads each) may stay in flight
                int newer = n - 1 - j;
                if (newer > PD - 1) newer = PD - 1;
                if (newer >= 2) WAIT_VM7(16);
                else if (newer == 1) WAIT_VM7(8);
                else WAIT_VM7(0);
            }
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            const int jf = j + PD;
            uint32_t e_f = 0u;
            if (jf < n) {
                if ((jf & 63) == 0) ev = blist[jf + lane];
                e_f = entry(jf);
                int slot_f = slot + PD; if (slot_f >= NSLOT) slot_f -= NSLOT;
                fetch((int)(e_f & 0xffffffu), slot_f);
            }
            const uint32_t e_cur = eq[0];
            if (e_cur & mybit) {
                const u16 *Kt = Kb + slot * TILE;
                const u16 *Vt = Vb + slot * TILE;
                const int blk = (int)(e_cur & 0xffffffu);
#pragma unroll
                for (int i = 0; i < RING; ++i) read_frag(i, Kt, Vt, ring[i]);
                run_steps(Kt, Vt, 0, 16);
#pragma unroll
                for (int i = 0; i < RING; ++i) read_frag(16 + i, Kt, Vt, ring[(16 + i) % RING]);   // land under the softmax
                softmax(0, blk);
                softmax(1, blk);
                run_steps(Kt, Vt, 16, 32);
            }
#pragma unroll
            for (int b = 0; b + 1 < PD; ++b) eq[b] = eq[b + 1];
            eq[PD - 1] = e_f;
            ++slot; if (slot >= NSLOT) slot = 0;
        }
    }
    WAIT_VM7(0);
    __syncthreads();          // every wave is done with the rings: they become staging space
    if (lin) stage_state();

    // ---- epilogue ---------------------------------------------------------------------------------
    float inv_l[NQ];
#pragma unroll
    for (int qt = 0; qt < NQ; ++qt) {
        const float l_tot = l_run[qt] + __shfl_xor(l_run[qt], 32);
        inv_l[qt] = l_tot > 0.f ? 1.f / l_tot : 0.f;
    }
    float lin_scale[NQ] = {0.f, 0.f}, inv_den[NQ] = {0.f, 0.f};
    if (lin) {
        const float *Zh = a.Z + (size_t)bh * D;
#pragma unroll
        for (int qt = 0; qt < NQ; ++qt) {
            float dpart = 0.f;
#pragma unroll
            for (int st = 0; st < NS; ++st) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    uint32_t w = relu2e7(qf[qt][st].w[j]);
                    qf[qt][st].w[j] = w;
                    dpart = fmaf(__uint_as_float(w << 16), Zh[st * 16 + hh * 8 + 2 * j], dpart);
                    dpart = fmaf(__uint_as_float(w & 0xffff0000u), Zh[st * 16 + hh * 8 + 2 * j + 1], dpart);
                }
            }
            const float den = dpart + __shfl_xor(dpart, 32) + a.eps;
            inv_den[qt] = 1.f / den;
            lin_scale[qt] = a.coef[bh] * inv_den[qt];
        }
        WAIT_VM7(0);
        __syncthreads();   // the staged fragments have landed in every wave's view
    }
    // results leave through a wave-private 8 KB of the V ring (free since the barrier above), one sub-tile at a
    // time, so that every global store is a run of full 256-byte rows
    unsigned char *stg = reinterpret_cast<unsigned char *>(Vb) + wave * 8192;
    u16 *obase_h = reinterpret_cast<u16 *>(a.out) + (size_t)bh * N * D;
#pragma unroll
    for (int qt = 0; qt < NQ; ++qt) {
        f32x16 num[NDT];
        if (lin) {
#pragma unroll
            for (int dt = 0; dt < NDT; ++dt) {
#pragma unroll
                for (int r = 0; r < 16; ++r) num[dt][r] = 0.f;
#pragma unroll
                for (int st = 0; st < NS; ++st) {
                    const int idx = ((dt * NS + st) * 64 + lane) * 8;
                    bf16x8 hi = *reinterpret_cast<const bf16x8 *>(Kb + idx);
                    bf16x8 lo = *reinterpret_cast<const bf16x8 *>(Kb + D * D + idx);
                    num[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lo, qf[qt][st].v, num[dt], 0, 0, 0);
                    num[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(hi, qf[qt][st].v, num[dt], 0, 0, 0);
                }
            }
        }
        const size_t orow = ((size_t)bh * N + qrow[qt]) * D;
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                float os[4], ol[4], ov[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    os[t] = o[qt][dt][g4 * 4 + t] * inv_l[qt];
                    ol[t] = lin ? num[dt][g4 * 4 + t] : 0.f;
                    ov[t] = lin ? fmaf(ol[t], lin_scale[qt], os[t]) : os[t];
                }
                uint2 pk;
                pk.x = pack2e7(ov[0], ov[1]);
                pk.y = pack2e7(ov[2], ov[3]);
                *reinterpret_cast<uint2 *>(stg + l32 * 256 + (((dt * 4 + g4) ^ (l32 & 15)) << 4) + hh * 8) = pk;
                if (DBG && qvalid[qt]) {
                    const int col = dt * 32 + 8 * g4 + 4 * hh;
                    if (a.o_sparse_dbg)
                        *reinterpret_cast<float4 *>(a.o_sparse_dbg + orow + col) = make_float4(os[0], os[1], os[2], os[3]);
                    if (a.o_linear_dbg && lin)
                        *reinterpret_cast<float4 *>(a.o_linear_dbg + orow + col) =
                            make_float4(ol[0] * inv_den[qt], ol[1] * inv_den[qt], ol[2] * inv_den[qt], ol[3] * inv_den[qt]);
                }
            }
        asm volatile("" ::: "memory");       // the wave's LDS operations execute in order
        const int dest_mine = qvalid[qt] ? qrow[qt] : -1;
        const int r4 = lane >> 4, c16 = lane & 15;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int r = 4 * i + r4;
            const uint4 v = *reinterpret_cast<const uint4 *>(stg + r * 256 + ((c16 ^ (r & 15)) << 4));
            const int dest = __shfl(dest_mine, r);
            if (dest >= 0) *reinterpret_cast<uint4 *>(obase_h + (size_t)dest * D + c16 * 8) = v;
        }
        asm volatile("" ::: "memory");
    }
}

template <int PD, bool DBG>
static hipError_t launch_v7(const AttnArgs &a, hipStream_t st)
{
    const int ntiles = (a.nb + 3) / 4;
    const int total = a.B * a.H * ntiles;
    const int per_xcd = (total + 7) / 8;
    const int list_cap = (a.nb + 63) & ~63;
    const size_t lds = (size_t)(2 * (PD + 1)) * 64 * 128 * 2 + (size_t)list_cap * 4;
    static_assert(PD + 1 >= 4, "the epilogue stages 64 KB of state fragments in the K ring");
    constexpr int kMaxDyn = 160 * 1024 - 2048;
    if (lds > (size_t)kMaxDyn) return hipErrorInvalidValue;
    auto kern = sparse_attn_v7_kernel<PD, DBG>;
    static bool attr_done[16] = {};
    if (hipError_t e = dyn_lds_attr_once(reinterpret_cast<const void *>(kern), kMaxDyn, attr_done); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(per_xcd * 8), dim3(256), lds, st, a, ntiles, total, per_xcd, list_cap);
    return hipGetLastError();
}

hipError_t launch_sparse_attn_v7(const AttnArgs &a, hipStream_t st)
{
    const bool dbg = a.o_sparse_dbg || a.o_linear_dbg;
    return dbg ? launch_v7<3, true>(a, st) : launch_v7<3, false>(a, st);
}

}  // namespace salad
