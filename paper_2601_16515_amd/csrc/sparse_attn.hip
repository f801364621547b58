// Block-sparse softmax attention (Eq. (2)) over a CSR of kept 64-token KV blocks, with the linear
// branch's apply (Eq. (3)) and the scale-and-sum of Alg. 1 fused into the epilogue.  gfx950 only.
//
// bf16 kernel, one workgroup = 4 waves = 128 query positions (two 64-token query blocks) of one
// (batch, head); each wave owns 32 query positions.  The workgroup walks the ascending union of
// its two CSR rows; a wave skips KV blocks its own query block does not keep.
//
// Everything is computed transposed so that one lane owns one query:
//   S^T = K Q^T   (A = K tile rows from LDS, B = Q fragments held in registers for the whole kernel)
//   O^T += V^T P^T (A = V^T from LDS, B = P^T taken straight from the S^T accumulators)
// With v_mfma_f32_32x32x16_bf16 the accumulator of lane (query j = lane%32, half hh = lane/32) holds
// rows 8g + 4hh + t (g = 0..3, t = 0..3).  K rows are read from LDS through the permutation
// kappa (swap bits 2 and 3 of the row index) so that those 16 registers are keys 8hh..8hh+7 and
// 16+8hh..16+8hh+7 of the 32-key tile - exactly the B-operand layout of the PV product, with no
// cross-lane movement.  The online softmax therefore needs one cross-lane exchange per KV block
// (the running maximum, between lanes j and j+32); row sums stay per lane until the end.
//
// Token orders (App. A.1.1): positions of a temporal head are gathered from / scattered to the
// stored [N, d] rows inside the global loads and stores (each row is one contiguous d*2 bytes), so
// no permuted copy of Q, K, V or O is ever written.
//
// LDS: K tile [64 keys][d + 8] (row-major, 16-byte operand reads hit distinct banks), V tile
// transposed [d][64 + 8] with the 8-key group XOR-swizzled by (row / 16).  Global loads of the next
// KV block are issued into registers before the current block is computed.
#include "salad_internal.h"

namespace salad {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef short s16x2 __attribute__((ext_vector_type(2)));

constexpr int XT_PITCH = 72;
__device__ inline int vt_off(int row, int tok)
{
    return row * XT_PITCH + ((((tok >> 3) ^ (row >> 4)) & 7) << 3) + (tok & 7);
}

__device__ inline int row_of_position(int kind, int p, int T, int HW)
{
    if (!kind) return p;
    int loc = p / T;
    return (p - loc * T) * HW + loc;
}

__device__ inline uint32_t pack_bf16x2(float a, float b)
{
    f32x2 x = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf16x2));
}

__device__ inline uint32_t relu2(uint32_t x)
{
    s16x2 v = __builtin_bit_cast(s16x2, x);
    s16x2 z = {0, 0};
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(v, z));
}

union Frag8 {
    bf16x8 v;
    uint4 u;
    uint32_t w[4];
};

template <int D, bool DBG>
__global__ __launch_bounds__(256, 2) void sparse_attn_bf16_kernel(AttnArgs a, int ntiles, int total, int per_xcd)
{
    constexpr int KP = D + 8;      // K tile pitch (elements)
    constexpr int CH = D / 8;      // 16-byte chunks per row
    constexpr int KROWS = 256 / CH;        // K rows covered by one pass of 256 threads
    constexpr int KPASS = 64 / KROWS;      // passes per K tile (4 for d=128, 2 for d=64)
    constexpr int TPT = D / 32;            // V tokens per thread per tile
    constexpr int NS = D / 16;             // MFMA k-steps over d
    constexpr int NDT = D / 32;            // 32-wide tiles of the head dimension
    __shared__ __attribute__((aligned(16))) u16 Ks[64 * KP];
    __shared__ __attribute__((aligned(16))) u16 Vt[D * XT_PITCH];

    // Workgroup ids are dealt round-robin to the 8 XCDs; give each XCD a contiguous range of
    // (head, query tile) so that neighbouring tiles share K/V in that XCD's L2.
    const int g = blockIdx.x;
    const int L = (g & 7) * per_xcd + (g >> 3);
    if (L >= total) return;
    const int bh = L / ntiles, tile = L - bh * ntiles;
    const int h = bh % a.H;
    const int kind = (int)((a.kind_mask >> h) & 1ull);
    const int N = a.N, T = a.T, HW = a.HW, nb = a.nb;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hh = lane >> 5;
    const u16 *qb = reinterpret_cast<const u16 *>(a.q) + (size_t)bh * N * D;
    const u16 *kb = reinterpret_cast<const u16 *>(a.k) + (size_t)bh * N * D;
    const u16 *vb = reinterpret_cast<const u16 *>(a.v) + (size_t)bh * N * D;

    const int qblk = tile * 2 + (wave >> 1);
    const int mybit = 1 << (wave >> 1);
    const int qpos = qblk * 64 + (wave & 1) * 32 + l32;
    const bool qvalid = (qblk < nb) && (qpos < N);
    const int qrow = row_of_position(kind, qvalid ? qpos : N - 1, T, HW);

    // Q fragments (B operand): lane holds Q[query][16 s + 8 hh .. +7]
    Frag8 qf[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s)
        qf[s].u = *reinterpret_cast<const uint4 *>(qb + (size_t)qrow * D + s * 16 + hh * 8);

    // CSR rows of the two query blocks
    const int rowA = h * nb + tile * 2;
    int pa = a.row_ptr[rowA], ea = a.row_ptr[rowA + 1];
    int pb = 0, eb = 0;
    if (tile * 2 + 1 < nb) { pb = ea; eb = a.row_ptr[rowA + 2]; }

    // loop-invariant LDS addresses
    const int kc = tid % CH, kr = tid / CH;              // K store: chunk, first row
    const int fg = tid % CH, tq = tid / CH;              // V store: feature group, token group
    const int kappa = (l32 & 0x13) | ((l32 & 4) << 1) | ((l32 & 8) >> 1);

    uint4 kreg[KPASS], vreg[TPT];
    auto gload = [&](int blk) {
#pragma unroll
        for (int i = 0; i < KPASS; ++i) {
            int p = blk * 64 + kr + i * KROWS;
            p = p < N ? p : N - 1;
            int n = row_of_position(kind, p, T, HW);
            kreg[i] = *reinterpret_cast<const uint4 *>(kb + (size_t)n * D + kc * 8);
        }
#pragma unroll
        for (int i = 0; i < TPT; ++i) {
            int p = blk * 64 + tq * TPT + i;
            p = p < N ? p : N - 1;
            int n = row_of_position(kind, p, T, HW);
            vreg[i] = *reinterpret_cast<const uint4 *>(vb + (size_t)n * D + fg * 8);
        }
    };
    auto lstore = [&]() {
#pragma unroll
        for (int i = 0; i < KPASS; ++i)
            *reinterpret_cast<uint4 *>(Ks + (kr + i * KROWS) * KP + kc * 8) = kreg[i];
        uint32_t w[TPT][4];
#pragma unroll
        for (int i = 0; i < TPT; ++i) { w[i][0] = vreg[i].x; w[i][1] = vreg[i].y; w[i][2] = vreg[i].z; w[i][3] = vreg[i].w; }
#pragma unroll
        for (int f = 0; f < 8; ++f) {
            const uint32_t sel = (f & 1) ? 0x07060302u : 0x05040100u;
            int off = vt_off(fg * 8 + f, tq * TPT);
            if (TPT == 4) {
                uint2 o;
                o.x = __builtin_amdgcn_perm(w[1][f >> 1], w[0][f >> 1], sel);
                o.y = __builtin_amdgcn_perm(w[3][f >> 1], w[2][f >> 1], sel);
                *reinterpret_cast<uint2 *>(Vt + off) = o;
            } else {
                *reinterpret_cast<uint32_t *>(Vt + off) = __builtin_amdgcn_perm(w[1][f >> 1], w[0][f >> 1], sel);
            }
        }
    };
    auto next_block = [&](int &blk, int &flags) -> bool {
        int ca = pa < ea ? a.col_idx[pa] : 0x7fffffff;
        int cb = pb < eb ? a.col_idx[pb] : 0x7fffffff;
        blk = ca < cb ? ca : cb;
        if (blk == 0x7fffffff) return false;
        flags = (ca == blk ? 1 : 0) | (cb == blk ? 2 : 0);
        pa += (ca == blk);
        pb += (cb == blk);
        return true;
    };

    f32x16 o[NDT];
#pragma unroll
    for (int i = 0; i < NDT; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[i][r] = 0.f;
    float m_run = -1e30f, l_run = 0.f;
    const float c2 = a.scale * 1.44269504088896340736f;   // logits are kept in the log2 domain

    int blk = 0, flags = 0, cur_blk = 0, cur_flags = 0;
    bool more = next_block(blk, flags);
    if (more) gload(blk);
    while (more) {
        lstore();
        __syncthreads();
        cur_blk = blk; cur_flags = flags;
        more = next_block(blk, flags);
        if (more) gload(blk);

        if ((cur_flags & mybit) && qblk < nb) {
            // S^T for the 64 keys of this block: two 32-key tiles
            f32x16 s[2];
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
                for (int r = 0; r < 16; ++r) s[kt][r] = 0.f;
#pragma unroll
                for (int st = 0; st < NS; ++st) {
                    bf16x8 kf = *reinterpret_cast<const bf16x8 *>(Ks + (kt * 32 + kappa) * KP + st * 16 + hh * 8);
                    s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[st].v, s[kt], 0, 0, 0);
                }
            }
            // register r of tile kt is key  kt*32 + 16*(r/8) + 8*hh + r%8  of the block
            const int kbase = cur_blk * 64 + hh * 8;
            if (cur_blk * 64 + 64 > N) {
#pragma unroll
                for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (kbase + kt * 32 + 16 * (r >> 3) + (r & 7) >= N) s[kt][r] = -INFINITY;
            }
            float mx = s[0][0];
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kt][r]);
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m_run, mx * c2);
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
            m_run = m_new;
            float psum = 0.f;
            Frag8 pf[4];   // pf[kt*2 + c]: keys kt*32 + 16c + 8hh + 0..7
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int r = 0; r < 16; r += 2) {
                    float p0 = __builtin_amdgcn_exp2f(fmaf(s[kt][r], c2, -m_new));
                    float p1 = __builtin_amdgcn_exp2f(fmaf(s[kt][r + 1], c2, -m_new));
                    psum += p0 + p1;
                    pf[kt * 2 + (r >> 3)].w[(r & 7) >> 1] = pack_bf16x2(p0, p1);
                }
            l_run = l_run * alpha + psum;
#pragma unroll
            for (int i = 0; i < NDT; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[i][r] *= alpha;
            // O^T += V^T P^T
#pragma unroll
            for (int kc16 = 0; kc16 < 4; ++kc16) {
#pragma unroll
                for (int dt = 0; dt < NDT; ++dt) {
                    bf16x8 vf = *reinterpret_cast<const bf16x8 *>(Vt + vt_off(dt * 32 + l32, kc16 * 16 + hh * 8));
                    o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[kc16].v, o[dt], 0, 0, 0);
                }
            }
        }
        __syncthreads();
    }

    // ---- epilogue: normalise, linear branch, scale and sum, store ---------------------------------
    float l_tot = l_run + __shfl_xor(l_run, 32);
    const float inv_l = l_tot > 0.f ? 1.f / l_tot : 0.f;
    f32x16 num[NDT];
    float lin_scale = 0.f, inv_den = 0.f;
    const bool lin = a.use_linear && !a.write_sparse_only && !(a.drop && a.drop[bh / a.H]);   // pruned sample (Sec. 4.3): out = O_s
    if (lin) {
        // phi(Q) = relu(Q) on the fragments already in registers
        float dpart = 0.f;
        const float *Zh = a.Z + (size_t)bh * D;
#pragma unroll
        for (int st = 0; st < NS; ++st) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                uint32_t w = relu2(qf[st].w[j]);
                qf[st].w[j] = w;
                dpart = fmaf(__uint_as_float(w << 16), Zh[st * 16 + hh * 8 + 2 * j], dpart);
                dpart = fmaf(__uint_as_float(w & 0xffff0000u), Zh[st * 16 + hh * 8 + 2 * j + 1], dpart);
            }
        }
        const float den = dpart + __shfl_xor(dpart, 32) + a.eps;
        inv_den = 1.f / den;
        lin_scale = a.coef[bh] * inv_den;
        // num^T = Hs^T phi(Q)^T with Hs rounded to bf16 (MFMA operand)
        const u16 *hf = a.hfrag + (size_t)bh * D * D;
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt) {
#pragma unroll
            for (int r = 0; r < 16; ++r) num[dt][r] = 0.f;
#pragma unroll
            for (int st = 0; st < NS; ++st) {
                size_t idx = ((size_t)(dt * NS + st) * 64 + lane) * 8;
                bf16x8 hi = *reinterpret_cast<const bf16x8 *>(hf + idx);
                num[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(hi, qf[st].v, num[dt], 0, 0, 0);
            }
        }
    }
    if (!qvalid) return;
    // accumulator register r of tile dt is column  dt*32 + 8*(r/4) + 4*hh + r%4  of this lane's query
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
            pk.x = pack_bf16x2(ov[0], ov[1]);
            pk.y = pack_bf16x2(ov[2], ov[3]);
            *reinterpret_cast<uint2 *>(outp + col) = pk;
            if (DBG) {
                if (a.o_sparse_dbg)
                    *reinterpret_cast<float4 *>(a.o_sparse_dbg + obase + col) = make_float4(os[0], os[1], os[2], os[3]);
                if (a.o_linear_dbg && lin)
                    *reinterpret_cast<float4 *>(a.o_linear_dbg + obase + col) =
                        make_float4(ol[0] * inv_den, ol[1] * inv_den, ol[2] * inv_den, ol[3] * inv_den);
            }
        }
    }
}

bool attn_takes_large_tile(const AttnArgs &a)
{
    if ((a.D != 128 && a.D != 64) || !a.tile_lists) return false;
    if (a.topk_mask) return a.D == 128;
    const bool temporal = a.kind_mask != 0 && a.T > 1;
    return a.variant == 0 && (size_t)tile_list_cap(a.nb) * 4 <= 24 * 1024 && (unsigned long long)a.N * 256ull < (1ull << 32) &&
           (!temporal || a.t_magic != 0);
}

hipError_t launch_sparse_attn_bf16(const AttnArgs &a, hipStream_t st)
{
    // d = 128: the large-tile ping-pong kernel unless its block list does not fit in LDS or a variant is
    // forced (a.variant: 0 = automatic, 1 = double-buffered 128-row kernel, 2 = first-generation kernel)
    const int variant = a.variant;
    if (a.topk_mask) {   // token-level mask: the large-tile kernel only (the host checks that the shape fits it)
        if (a.D != 128 || !a.tile_lists) return hipErrorInvalidValue;
        return launch_sparse_attn_v5(a, st);
    }
    if (variant != 2) {
        // the large-tile kernel addresses rows with 32-bit byte offsets and divides by T with a
        // multiply (t_magic); a T = 1 grid makes the temporal order the identity
        const bool temporal = a.kind_mask != 0 && a.T > 1;
        const bool fits = (size_t)tile_list_cap(a.nb) * 4 <= 24 * 1024 && (unsigned long long)a.N * 256ull < (1ull << 32) &&
                          (!temporal || a.t_magic != 0);
        if (variant == 0 && fits && a.tile_lists) return launch_sparse_attn_v5(a, st);
        if (a.D == 128) return launch_sparse_attn_v2(a, st);
    }
    const int ntiles = (a.nb + 1) / 2;
    const int total = a.B * a.H * ntiles;
    const int per_xcd = (total + 7) / 8;
    dim3 grid(per_xcd * 8), block(256);
    const bool dbg = a.o_sparse_dbg || a.o_linear_dbg;
    if (a.D == 128) {
        if (dbg) launch_kernel((sparse_attn_bf16_kernel<128, true>), grid, block, 0, st, a, ntiles, total, per_xcd);
        else launch_kernel((sparse_attn_bf16_kernel<128, false>), grid, block, 0, st, a, ntiles, total, per_xcd);
    } else {
        if (dbg) launch_kernel((sparse_attn_bf16_kernel<64, true>), grid, block, 0, st, a, ntiles, total, per_xcd);
        else launch_kernel((sparse_attn_bf16_kernel<64, false>), grid, block, 0, st, a, ntiles, total, per_xcd);
    }
    return take_launch_status();
}

// ------------------------------------------------------------------------------------------------
// fp32 path for small shapes: one wave per query position, online softmax in fp32, same fused epilogue.
// Per kept block the lanes are the block's 64 keys for the logits (every lane takes the whole dot product of its key
// with the query, which sits in LDS: independent row loads, one maximum and one sum across the wave per block) and
// the head dimension for the output (lane c owns channels c and c + 64; the key's weight comes from its lane).
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void sparse_attn_f32_kernel(AttnArgs a)
{
    __shared__ __attribute__((aligned(16))) float qs[4][128];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int D = a.D, N = a.N, nb = a.nb;
    const long long gw = (long long)blockIdx.x * 4 + wave;     // (bh, position)
    const long long totalq = (long long)a.B * a.H * N;
    if (gw >= totalq) return;                          // whole waves leave; nothing below synchronises across waves
    const int bh = (int)(gw / N), p = (int)(gw - (long long)bh * N);
    const int h = bh % a.H;
    const int kind = (int)((a.kind_mask >> h) & 1ull);
    const float *qb = reinterpret_cast<const float *>(a.q) + (size_t)bh * N * D;
    const float *kb = reinterpret_cast<const float *>(a.k) + (size_t)bh * N * D;
    const float *vb = reinterpret_cast<const float *>(a.v) + (size_t)bh * N * D;
    const int n = row_of_position(kind, p, a.T, a.HW);
    const int c0 = lane, c1 = lane + 64;
    const bool h1 = c1 < D, h0 = c0 < D;
    const float q0 = h0 ? qb[(size_t)n * D + c0] : 0.f, q1 = h1 ? qb[(size_t)n * D + c1] : 0.f;
    qs[wave][c0] = q0;
    qs[wave][c1] = q1;
    __builtin_amdgcn_wave_barrier();                   // the wave's own LDS writes, read back by its own lanes
    float m = -1e30f, l = 0.f, o0 = 0.f, o1 = 0.f;
    const int row = h * nb + p / 64;
    for (int e = a.row_ptr[row]; e < a.row_ptr[row + 1]; ++e) {
        const int j = a.col_idx[e];
        const int pk = j * 64 + lane;                  // this lane's key
        const bool kvalid = pk < N;
        const int nk = row_of_position(kind, kvalid ? pk : N - 1, a.T, a.HW);
        const float4 *kr = reinterpret_cast<const float4 *>(kb + (size_t)nk * D);
        float part = 0.f;
        for (int d4 = 0; d4 < D / 4; d4 += 8) {        // D is 64 or 128: 8 row loads in flight
            float4 kv[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) kv[u] = kr[d4 + u];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const float4 qv = *reinterpret_cast<const float4 *>(&qs[wave][(d4 + u) * 4]);
                part = fmaf(qv.x, kv[u].x, part); part = fmaf(qv.y, kv[u].y, part);
                part = fmaf(qv.z, kv[u].z, part); part = fmaf(qv.w, kv[u].w, part);
            }
        }
        const float logit = kvalid ? part * a.scale : -INFINITY;
        float mb = logit;
#pragma unroll
        for (int x = 32; x > 0; x >>= 1) mb = fmaxf(mb, __shfl_xor(mb, x));
        const float mn = fmaxf(m, mb);
        const float alpha = __expf(m - mn), pw = kvalid ? __expf(logit - mn) : 0.f;
        float ps = pw;
#pragma unroll
        for (int x = 32; x > 0; x >>= 1) ps += __shfl_xor(ps, x);
        l = l * alpha + ps;
        o0 *= alpha; o1 *= alpha;
        m = mn;
        const int cmax = min(64, N - j * 64);
        for (int c = 0; c < cmax; c += 16) {           // 16 value rows in flight; weights and rows past the block are zero / clamped
            float v0[16], v1[16], wc[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int cc = c + u < cmax ? c + u : cmax - 1;
                const int nv = __shfl(nk, cc);
                wc[u] = c + u < cmax ? __shfl(pw, cc) : 0.f;
                const float *vr = vb + (size_t)nv * D;
                v0[u] = h0 ? vr[c0] : 0.f;
                v1[u] = h1 ? vr[c1] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < 16; ++u) { o0 = fmaf(wc[u], v0[u], o0); o1 = fmaf(wc[u], v1[u], o1); }
        }
    }
    const float inv_l = l > 0.f ? 1.f / l : 0.f;
    float os0 = o0 * inv_l, os1 = o1 * inv_l;
    float ol0 = 0.f, ol1 = 0.f, r0 = os0, r1 = os1;
    const bool lin = a.use_linear && !(a.drop && a.drop[bh / a.H]);   // pruned sample (Sec. 4.3): out = O_s
    if (lin) {
        const float *Hh = a.Hs + (size_t)bh * D * D;
        const float *Zh = a.Z + (size_t)bh * D;
        const float f0 = fmaxf(q0, 0.f), f1 = fmaxf(q1, 0.f);
        float dpart = (h0 ? f0 * Zh[c0] : 0.f) + (h1 ? f1 * Zh[c1] : 0.f);
#pragma unroll
        for (int x = 32; x > 0; x >>= 1) dpart += __shfl_xor(dpart, x);
        const float inv_den = 1.f / (dpart + a.eps);
        float n0 = 0.f, n1 = 0.f;
        for (int aa = 0; aa < D; aa += 8) {            // D is a multiple of 8: 8 state rows in flight
            float x0[8], x1[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                x0[u] = h0 ? Hh[(size_t)(aa + u) * D + c0] : 0.f;
                x1[u] = h1 ? Hh[(size_t)(aa + u) * D + c1] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const float qa = fmaxf(qs[wave][aa + u], 0.f);
                n0 = fmaf(qa, x0[u], n0);
                n1 = fmaf(qa, x1[u], n1);
            }
        }
        ol0 = n0 * inv_den; ol1 = n1 * inv_den;
        const float cf = a.coef[bh];
        r0 = fmaf(cf, ol0, os0); r1 = fmaf(cf, ol1, os1);
    }
    const size_t ob = ((size_t)bh * N + n) * D;
    float *out = reinterpret_cast<float *>(a.out);
    if (h0) out[ob + c0] = r0;
    if (h1) out[ob + c1] = r1;
    if (a.o_sparse_dbg) { if (h0) a.o_sparse_dbg[ob + c0] = os0; if (h1) a.o_sparse_dbg[ob + c1] = os1; }
    if (a.o_linear_dbg && lin) { if (h0) a.o_linear_dbg[ob + c0] = ol0; if (h1) a.o_linear_dbg[ob + c1] = ol1; }
}

hipError_t launch_sparse_attn_f32(const AttnArgs &a, hipStream_t st)
{
    long long totalq = (long long)a.B * a.H * a.N;
    dim3 grid((unsigned)((totalq + 3) / 4)), block(256);
    launch_kernel(sparse_attn_f32_kernel, grid, block, 0, st, a);
    return take_launch_status();
}

}  // namespace salad
