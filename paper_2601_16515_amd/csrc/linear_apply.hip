// Unfused form of the linear apply (Eq. (3) quotient) plus scale-and-sum (Alg. 1 residual
// integration) as one streaming kernel:  out <- out + coef[b,h] * relu(Q) Hs / (relu(Q).Z + eps),
// where `out` holds the sparse branch (bf16) on entry.  HBM-bound: reads Q and O_s, writes O
// (6*N*d bytes per head); the d x d product runs on bf16 MFMA with Hs rounded to bf16.
// One wave owns 32 stored rows at a time; the state fragments are staged in LDS once per workgroup.
// d = 128 (linear_apply128_kernel): every global access is a full 128-byte line segment (8 rows x 128 bytes
// per wave instruction); rows change between that layout and the MFMA operand / accumulator layouts
// through a wave-private 8 KB LDS buffer.  d = 64 keeps the direct-access kernel.
#include "salad_internal.h"

namespace salad {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef short s16x2 __attribute__((ext_vector_type(2)));

union Frag8a {
    bf16x8 v;
    uint4 u;
    uint32_t w[4];
};


template <int D>
__global__ __launch_bounds__(256) void linear_apply_kernel(ApplyArgs a, int rows_per_wg)
{
    constexpr int NS = D / 16, NDT = D / 32;
    __shared__ __attribute__((aligned(1024))) u16 hf_lds[D * D];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hh = lane >> 5;
    const int bh = blockIdx.y;
    if (a.drop && a.drop[bh / a.H]) return;            // pruned sample (Sec. 4.3): out already holds O_s
    {   // fragments are lane-linear in memory: copy as is (16 bytes per lane per load)
        const u16 *hf = a.hfrag + (size_t)bh * D * D;
        constexpr int LOADS = D * D / 8 / 256;
#pragma unroll
        for (int i = 0; i < LOADS; ++i)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(hf + (size_t)(i * 256 + tid) * 8),
                                             (__attribute__((address_space(3))) void *)(hf_lds + (i * 256 + wave * 64) * 8), 16, 0, 0);
    }
    const float *Zh = a.Z + (size_t)bh * D;
    float zr[NS][8];
#pragma unroll
    for (int st = 0; st < NS; ++st)
#pragma unroll
        for (int j = 0; j < 8; ++j) zr[st][j] = Zh[st * 16 + hh * 8 + j];
    const float coef = a.coef[bh];
    __syncthreads();
    const int row_end = min(a.N, (int)(blockIdx.x + 1) * rows_per_wg);
    for (int row0 = blockIdx.x * rows_per_wg + wave * 32; row0 < row_end; row0 += 128) {
        const int row = row0 + l32;
        const bool valid = row < a.N;
        const int rr = valid ? row : a.N - 1;
        const u16 *qrow = a.q + ((size_t)bh * a.N + rr) * D;
        Frag8a qf[NS];
        float dpart = 0.f;
#pragma unroll
        for (int st = 0; st < NS; ++st) qf[st].u = *reinterpret_cast<const uint4 *>(qrow + st * 16 + hh * 8);
        const size_t obase = ((size_t)bh * a.N + rr) * D;
        uint2 osv[NDT][4];
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) osv[dt][g4] = *reinterpret_cast<const uint2 *>(a.out + obase + dt * 32 + 8 * g4 + 4 * hh);
#pragma unroll
        for (int st = 0; st < NS; ++st) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                s16x2 v = __builtin_bit_cast(s16x2, qf[st].w[j]);
                s16x2 z = {0, 0};
                uint32_t w = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(v, z));
                qf[st].w[j] = w;
                dpart = fmaf(__uint_as_float(w << 16), zr[st][2 * j], dpart);
                dpart = fmaf(__uint_as_float(w & 0xffff0000u), zr[st][2 * j + 1], dpart);
            }
        }
        asm volatile("" ::: "memory");   // the wave's LDS operations execute in order; as above
        const float inv_den = 1.f / (dpart + __shfl_xor(dpart, 32) + a.eps);
        const float sc = coef * inv_den;
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt) {
            f32x16 num;
#pragma unroll
            for (int r = 0; r < 16; ++r) num[r] = 0.f;
#pragma unroll
            for (int st = 0; st < NS; ++st) {
                const int idx = ((dt * NS + st) * 64 + lane) * 8;
                bf16x8 hi = *reinterpret_cast<const bf16x8 *>(hf_lds + idx);
                num = __builtin_amdgcn_mfma_f32_32x32x16_bf16(hi, qf[st].v, num, 0, 0, 0);
            }
            if (valid) {
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) {
                    const int col = dt * 32 + 8 * g4 + 4 * hh;
                    const uint2 os = osv[dt][g4];
                    float o0 = fmaf(num[g4 * 4 + 0], sc, __uint_as_float(os.x << 16));
                    float o1 = fmaf(num[g4 * 4 + 1], sc, __uint_as_float(os.x & 0xffff0000u));
                    float o2 = fmaf(num[g4 * 4 + 2], sc, __uint_as_float(os.y << 16));
                    float o3 = fmaf(num[g4 * 4 + 3], sc, __uint_as_float(os.y & 0xffff0000u));
                    f32x2 x01 = {o0, o1}, x23 = {o2, o3};
                    uint2 pk;
                    pk.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(x01, bf16x2));
                    pk.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(x23, bf16x2));
                    *reinterpret_cast<uint2 *>(a.out + obase + col) = pk;
                    if (a.o_linear_dbg)
                        *reinterpret_cast<float4 *>(a.o_linear_dbg + obase + col) =
                            make_float4(num[g4 * 4 + 0] * inv_den, num[g4 * 4 + 1] * inv_den,
                                        num[g4 * 4 + 2] * inv_den, num[g4 * 4 + 3] * inv_den);
                }
            }
        }
    }
}

// d = 128.  Per wave and 32-row block: Q rows -> LDS -> B-operand fragments; relu, denominator; for each
// half of the 128 output columns 32 MFMAs against the hi + lo state fragments, scaled results (fp32) -> LDS ->
// row layout, added to O_s in fp32, one rounding to bf16, stored.
// EMIT: instead of adding to O_s, write the unscaled O_l (bf16) to a.emit (input of the full Level-1
// projection) in the order that kernel's MFMA B operand wants: [B][ceil(N/32)][H] blocks of 32 rows x 128
// channels, 16-byte chunk c (channels 8c .. 8c+7) of block row r at ((c/2 * 64 + (c%2) * 32 + r) * 16 bytes, so
// that one 16-byte load per lane fetches a whole 32 x 16 fragment from 1 KB of contiguous memory.  Rows past N
// in the last block are written too (from the clamped Q row): finite values nobody uses.
// ROPE: the rotary linear branch (Sec. 4.1).  The denominator is taken from the unrotated relu(Q); then the rows'
// (cos, sin) words (two fp16 values per channel pair, [N, 64] words: 256 bytes per row, the same geometry as a bf16
// Q row) go through the same LDS staging as Q, and channel pair (2p, 2p+1) of relu(Q) is rotated before it becomes
// the numerator's MFMA operand (the state fragments then hold the rotated state).
// MERGE: the regrouped Top-K path (App. A.1.2) leaves O_s as up to four partial results per query (normalised per
// key block, bf16, with a log2-domain log-sum-exp each).  Instead of reading a merged O_s back, every thread gathers
// the 16-byte pieces of the partial rows it adds to, weighs them by 2^(lse - max lse) / sum and keeps the merged
// piece in fp32: one pass over Q and the partial results, one rounding.  The slot numbers and the selection word
// of a pass are loaded one pass ahead, the pieces of the second half row while the first half's MFMAs run.
template <bool DBG, bool EMIT, bool ROPE = false, bool MERGE = false>
__global__ __launch_bounds__(512) void linear_apply128_kernel(ApplyArgs a, int rows_per_wg)
{
    static_assert(!MERGE || (!DBG && !EMIT && !ROPE), "the merging variant exists for the plain sum only");
    constexpr int D = 128, NS = 8;
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    u16 *hf_lds = reinterpret_cast<u16 *>(smem);                                  // [D*D] state fragments
    float *z_lds = reinterpret_cast<float *>(smem + D * D * 2);                   // [D]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    unsigned char *stage = smem + D * D * 2 + 1024 + wave * 8192;                 // wave-private, 8 KB
    const int l32 = lane & 31, hh = lane >> 5;
    // ROPE: sample-head index fastest (neighbours in the grid share the angle-table rows)
    const int bh = ROPE ? blockIdx.x : blockIdx.y, rblk = ROPE ? blockIdx.y : blockIdx.x;
    const bool pruned = a.drop && a.drop[bh / a.H];    // pruned sample (Sec. 4.3): out = O_s
    if (pruned && !MERGE) return;                      // out already holds O_s
    {   // fragments are lane-linear in memory: copy as is (16 bytes per lane per load)
        const u16 *hf = a.hfrag + (size_t)bh * D * D;
#pragma unroll
        for (int i = 0; i < D * D / 8 / 512; ++i)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(hf + (size_t)(i * 512 + tid) * 8),
                                             (__attribute__((address_space(3))) void *)(hf_lds + (i * 512 + wave * 64) * 8), 16, 0, 0);
        if (tid < D) z_lds[tid] = a.Z[(size_t)bh * D + tid];
    }
    const float coef = pruned ? 0.f : a.coef[bh];
    __syncthreads();
    const int N = a.N;
    const u16 *qh = a.q + (size_t)bh * N * D;
    u16 *oh = a.out + (size_t)bh * N * D;
    const int r8 = lane >> 3, c8 = lane & 7;          // row layout of a half: 8 rows x 8 chunks of 16 bytes per instruction
    const int r4 = lane >> 4, c16 = lane & 15;        // row layout of full rows: 4 rows x 16 chunks
    const int row_end = min(N, (rblk + 1) * rows_per_wg);
    // MERGE: per row 8 k + r8 of the pass (k < 4) the number of partial results and their slots, loaded a pass ahead
    const size_t mslots = MERGE ? (size_t)N * a.m_kk : 0;
    int mcnt[4] = {0, 0, 0, 0}, msl[4][4] = {};
    auto merge_slots = [&](int rb0) __attribute__((always_inline)) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int row = rb0 + 8 * k + r8;
            const bool ok = row < N;
            const size_t qi = (size_t)bh * N + (ok ? row : N - 1);
            const int pc = (int)__popcll(a.m_mask[qi]);
            mcnt[k] = ok ? min(a.m_kk, pc) : 0;        // only the ranks the regrouping pass filled in
#pragma unroll
            for (int r = 0; r < 4; ++r) msl[k][r] = r < a.m_kk ? a.m_slot_of[qi * a.m_kk + r] : 0;
        }
    };
    if (MERGE && rblk * rows_per_wg + wave * 32 < row_end) merge_slots(rblk * rows_per_wg + wave * 32);
    for (int rb = rblk * rows_per_wg + wave * 32; rb < row_end; rb += 256) {
        float mw[4][4], minv[4];                       // weight of partial result r of row k; 1 / their sum
        uint4 mx4[4][4];                               // the pieces of the half row in flight
        auto merge_issue = [&](int h) __attribute__((always_inline)) {
#pragma unroll
            for (int k = 0; k < 4; ++k)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (r < mcnt[k])
                        mx4[k][r] = *reinterpret_cast<const uint4 *>(a.m_po + ((size_t)bh * mslots + msl[k][r]) * D + h * 64 + c8 * 8);
        };
        if (MERGE) {
            float ml[4][4];
#pragma unroll
            for (int k = 0; k < 4; ++k)
#pragma unroll
                for (int r = 0; r < 4; ++r) ml[k][r] = r < mcnt[k] ? a.m_lse[(size_t)bh * mslots + msl[k][r]] : -INFINITY;
            merge_issue(0);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float mx = fmaxf(fmaxf(ml[k][0], ml[k][1]), fmaxf(ml[k][2], ml[k][3]));
                float den = 0.f;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    mw[k][r] = r < mcnt[k] ? __builtin_amdgcn_exp2f(ml[k][r] - mx) : 0.f;
                    den += mw[k][r];
                }
                minv[k] = den > 0.f ? 1.f / den : 0.f;
            }
        }
        // merged O_s pieces of the half row in flight (fp32): acc[k][j] = (sum_r mw[k][r] * piece r) * minv[k], in the
        // order of topk_merge_kernel, so that a pruned sample gets the bits that kernel would write
        auto merge_take = [&](float (&acc)[4][8]) __attribute__((always_inline)) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[k][j] = 0.f;
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (r < mcnt[k]) {
                        const uint32_t w4[4] = {mx4[k][r].x, mx4[k][r].y, mx4[k][r].z, mx4[k][r].w};
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            acc[k][2 * j] = fmaf(mw[k][r], __uint_as_float(w4[j] << 16), acc[k][2 * j]);
                            acc[k][2 * j + 1] = fmaf(mw[k][r], __uint_as_float(w4[j] & 0xffff0000u), acc[k][2 * j + 1]);
                        }
                    }
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[k][j] *= minv[k];
            }
        };
        // ---- Q: 8 coalesced loads, swizzled into LDS (chunk ^ (row & 15)), read back as B-operand fragments
        uint4 qc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int row = min(rb + 4 * i + r4, N - 1);
            qc[i] = *reinterpret_cast<const uint4 *>(qh + (size_t)row * D + c16 * 8);
        }
        // O_s in the half-row layout (half h, rows 8k + r8): issued now, consumed at the end
        uint4 os[2][4];
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int row = min(rb + 8 * k + r8, N - 1);
                os[h][k] = (EMIT || MERGE) ? make_uint4(0, 0, 0, 0) : *reinterpret_cast<const uint4 *>(oh + (size_t)row * D + h * 64 + c8 * 8);
            }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int lrow = 4 * i + r4;
            *reinterpret_cast<uint4 *>(stage + lrow * 256 + ((c16 ^ (lrow & 15)) << 4)) = qc[i];
        }
        asm volatile("" ::: "memory");   // the wave's LDS operations execute in order; keep the compiler from reordering them
        Frag8a qf[NS];
        float dpart = 0.f;
#pragma unroll
        for (int st = 0; st < NS; ++st) {
            qf[st].u = *reinterpret_cast<const uint4 *>(stage + l32 * 256 + (((2 * st + hh) ^ (l32 & 15)) << 4));
            const float4 z0 = *reinterpret_cast<const float4 *>(z_lds + st * 16 + hh * 8);
            const float4 z1 = *reinterpret_cast<const float4 *>(z_lds + st * 16 + hh * 8 + 4);
            const float zz[8] = {z0.x, z0.y, z0.z, z0.w, z1.x, z1.y, z1.z, z1.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                s16x2 v = __builtin_bit_cast(s16x2, qf[st].w[j]);
                s16x2 z = {0, 0};
                uint32_t w = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(v, z));
                qf[st].w[j] = w;
                dpart = fmaf(__uint_as_float(w << 16), zz[2 * j], dpart);
                dpart = fmaf(__uint_as_float(w & 0xffff0000u), zz[2 * j + 1], dpart);
            }
        }
        asm volatile("" ::: "memory");   // the wave's LDS operations execute in order; as above
        if (ROPE) {
            // (cos, sin) words of the rows, 256 bytes per row: staged like the Q rows, then 4 words per d-step per lane
            uint4 tc[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int row = min(rb + 4 * i + r4, N - 1);
                tc[i] = *reinterpret_cast<const uint4 *>(a.rope_tab + (size_t)row * (D / 2) + c16 * 4);
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int lrow = 4 * i + r4;
                *reinterpret_cast<uint4 *>(stage + lrow * 256 + ((c16 ^ (lrow & 15)) << 4)) = tc[i];
            }
            asm volatile("" ::: "memory");
#pragma unroll
            for (int st = 0; st < NS; ++st) {
                const uint4 t = *reinterpret_cast<const uint4 *>(stage + l32 * 256 + (((2 * st + hh) ^ (l32 & 15)) << 4));
                const uint32_t cw[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t w = qf[st].w[j];
                    const float x = __uint_as_float(w << 16), y = __uint_as_float(w & 0xffff0000u);
                    const f16x2 hcs = __builtin_bit_cast(f16x2, cw[j]);
                    const float cc = (float)hcs[0], ss = (float)hcs[1];
                    f32x2 r = {x * cc - y * ss, x * ss + y * cc};
                    qf[st].w[j] = __builtin_bit_cast(uint32_t, __builtin_convertvector(r, bf16x2));
                }
            }
            asm volatile("" ::: "memory");
        }
        const float inv_den = 1.f / (dpart + __shfl_xor(dpart, 32) + a.eps);
        const float sc = EMIT ? inv_den : coef * inv_den;
        const bool rvalid = rb + l32 < N;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            f32x16 num[2];
#pragma unroll
            for (int dl = 0; dl < 2; ++dl) {
                const int dt = 2 * h + dl;
#pragma unroll
                for (int r = 0; r < 16; ++r) num[dl][r] = 0.f;
#pragma unroll
                for (int st = 0; st < NS; ++st) {
                    const int idx = ((dt * NS + st) * 64 + lane) * 8;
                    bf16x8 hi = *reinterpret_cast<const bf16x8 *>(hf_lds + idx);
                    num[dl] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(hi, qf[st].v, num[dl], 0, 0, 0);
                }
            }
            // accumulator layout (lane = row l32; registers 4 g4 + t = column 32 dl + 8 g4 + 4 hh + t) -> LDS, fp32,
            // rows of 64 columns = 16 chunks of 16 bytes, chunk ^ (row & 15)
#pragma unroll
            for (int dl = 0; dl < 2; ++dl)
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) {
                    const int chunk = dl * 8 + 2 * g4 + hh;
                    *reinterpret_cast<float4 *>(stage + l32 * 256 + ((chunk ^ (l32 & 15)) << 4)) =
                        make_float4(num[dl][g4 * 4 + 0] * sc, num[dl][g4 * 4 + 1] * sc, num[dl][g4 * 4 + 2] * sc, num[dl][g4 * 4 + 3] * sc);
                    if (DBG) {
                        if (a.o_linear_dbg && rvalid)
                            *reinterpret_cast<float4 *>(a.o_linear_dbg + ((size_t)bh * N + rb + l32) * D + (2 * h + dl) * 32 + 8 * g4 + 4 * hh) =
                                make_float4(num[dl][g4 * 4 + 0] * inv_den, num[dl][g4 * 4 + 1] * inv_den,
                                            num[dl][g4 * 4 + 2] * inv_den, num[dl][g4 * 4 + 3] * inv_den);
                    }
                }
            asm volatile("" ::: "memory");
            float macc[4][8];
            if (MERGE) {
                merge_take(macc);
                if (h == 0) merge_issue(1);            // lands under the second half's MFMAs
                else if (rb + 256 < row_end) merge_slots(rb + 256);
            }
            // row layout: 8 rows x 8 chunks of 8 columns per instruction; out = O_s + scaled numerator, one rounding
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int lrow = 8 * k + r8;
                const float4 n0 = *reinterpret_cast<const float4 *>(stage + lrow * 256 + (((2 * c8) ^ (lrow & 15)) << 4));
                const float4 n1 = *reinterpret_cast<const float4 *>(stage + lrow * 256 + (((2 * c8 + 1) ^ (lrow & 15)) << 4));
                const uint4 o4 = os[h][k];
                uint4 pk;
                {
                    f32x2 x0, x1, x2, x3;
                    if (MERGE && pruned) {             // no state was computed for this sample: O_s alone
                        x0 = (f32x2){macc[k][0], macc[k][1]};
                        x1 = (f32x2){macc[k][2], macc[k][3]};
                        x2 = (f32x2){macc[k][4], macc[k][5]};
                        x3 = (f32x2){macc[k][6], macc[k][7]};
                    } else if (MERGE) {
                        x0 = (f32x2){macc[k][0] + n0.x, macc[k][1] + n0.y};
                        x1 = (f32x2){macc[k][2] + n0.z, macc[k][3] + n0.w};
                        x2 = (f32x2){macc[k][4] + n1.x, macc[k][5] + n1.y};
                        x3 = (f32x2){macc[k][6] + n1.z, macc[k][7] + n1.w};
                    } else {
                        x0 = (f32x2){__uint_as_float(o4.x << 16) + n0.x, __uint_as_float(o4.x & 0xffff0000u) + n0.y};
                        x1 = (f32x2){__uint_as_float(o4.y << 16) + n0.z, __uint_as_float(o4.y & 0xffff0000u) + n0.w};
                        x2 = (f32x2){__uint_as_float(o4.z << 16) + n1.x, __uint_as_float(o4.z & 0xffff0000u) + n1.y};
                        x3 = (f32x2){__uint_as_float(o4.w << 16) + n1.z, __uint_as_float(o4.w & 0xffff0000u) + n1.w};
                    }
                    pk.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(x0, bf16x2));
                    pk.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(x1, bf16x2));
                    pk.z = __builtin_bit_cast(uint32_t, __builtin_convertvector(x2, bf16x2));
                    pk.w = __builtin_bit_cast(uint32_t, __builtin_convertvector(x3, bf16x2));
                }
                const int row = rb + lrow;
                if (EMIT) {
                    const int c = h * 8 + c8;
                    u16 *blk = a.emit + ((((size_t)(bh / a.H) * ((N + 31) >> 5) + (rb >> 5)) * a.H + bh % a.H) << 12);
                    *reinterpret_cast<uint4 *>(blk + (((c >> 1) * 64 + (c & 1) * 32 + lrow) << 3)) = pk;
                } else if (row < N) *reinterpret_cast<uint4 *>(oh + (size_t)row * D + h * 64 + c8 * 8) = pk;
            }
            asm volatile("" ::: "memory");
        }
    }
}

hipError_t launch_linear_apply_bf16(const ApplyArgs &a, hipStream_t st)
{
    if (a.D == 128) {
        // one workgroup of 8 waves per CU (64 KB of state fragments + 8 x 8 KB of staging), about two
        // workgroup-sized row ranges per CU; 256 rows per pass of a workgroup
        long long rows = ((long long)a.N * a.BH + 511) / 512;
        int rows_per_wg = (int)((rows + 255) / 256) * 256;
        if (rows_per_wg < 256) rows_per_wg = 256;
        dim3 grid((a.N + rows_per_wg - 1) / rows_per_wg, a.BH), block(512);
        constexpr int lds = 128 * 128 * 2 + 1024 + 8 * 8192;
        if (a.m_po) {                                  // O_s still lies in partial results: merge them in the same pass
            if (a.emit || a.o_linear_dbg || a.rope_tab || a.m_kk < 1 || a.m_kk > 4) return hipErrorInvalidValue;
            static bool done_m[16] = {};
            if (hipError_t e = dyn_lds_attr_once(reinterpret_cast<const void *>(linear_apply128_kernel<false, false, false, true>), lds, done_m); e != hipSuccess) return e;
            launch_kernel((linear_apply128_kernel<false, false, false, true>), grid, block, lds, st, a, rows_per_wg);
            return take_launch_status();
        }
        static bool done[6][16] = {};
        // variant: 0 plain, 1 debug output, 2 emit; + 3 with the rotary tables
        const int var = (a.emit ? 2 : a.o_linear_dbg ? 1 : 0) + (a.rope_tab ? 3 : 0);
        const void *kerns[6] = {reinterpret_cast<const void *>(linear_apply128_kernel<false, false, false>),
                                reinterpret_cast<const void *>(linear_apply128_kernel<true, false, false>),
                                reinterpret_cast<const void *>(linear_apply128_kernel<false, true, false>),
                                reinterpret_cast<const void *>(linear_apply128_kernel<false, false, true>),
                                reinterpret_cast<const void *>(linear_apply128_kernel<true, false, true>),
                                reinterpret_cast<const void *>(linear_apply128_kernel<false, true, true>)};
        if (hipError_t e = dyn_lds_attr_once(kerns[var], lds, done[var]); e != hipSuccess) return e;
        const dim3 grid_r(grid.y, grid.x);     // rotary variants: sample-head index fastest
        switch (var) {
        case 0: launch_kernel((linear_apply128_kernel<false, false, false>), grid, block, lds, st, a, rows_per_wg); break;
        case 1: launch_kernel((linear_apply128_kernel<true, false, false>), grid, block, lds, st, a, rows_per_wg); break;
        case 2: launch_kernel((linear_apply128_kernel<false, true, false>), grid, block, lds, st, a, rows_per_wg); break;
        case 3: launch_kernel((linear_apply128_kernel<false, false, true>), grid_r, block, lds, st, a, rows_per_wg); break;
        case 4: launch_kernel((linear_apply128_kernel<true, false, true>), grid_r, block, lds, st, a, rows_per_wg); break;
        default: launch_kernel((linear_apply128_kernel<false, true, true>), grid_r, block, lds, st, a, rows_per_wg); break;
        }
        return take_launch_status();
    }
    // rows per workgroup (a multiple of 128): about two workgroups per CU, so that the 2*d*d*2 bytes of
    // state fragments staged in LDS are reused over many rows
    long long rows = ((long long)a.N * a.BH + 511) / 512;
    int rows_per_wg = (int)((rows + 127) / 128) * 128;
    if (rows_per_wg < 128) rows_per_wg = 128;
    dim3 grid((a.N + rows_per_wg - 1) / rows_per_wg, a.BH), block(256);
    launch_kernel(linear_apply_kernel<64>, grid, block, 0, st, a, rows_per_wg);
    return take_launch_status();
}

}  // namespace salad
