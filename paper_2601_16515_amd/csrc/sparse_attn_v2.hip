// Block-sparse softmax attention (Eq. (2)) with the fused linear apply / scale / sum epilogue,
// second generation for d = 128:
//   * K and V tiles go from global memory straight into LDS (global_load_lds_dwordx4): no VGPR
//     staging, no LDS write instructions.  The LDS image of a tile is lane-linear, so the bank
//     swizzle is applied on the global side: LDS slot (row r, 16-byte chunk pc) receives logical
//     chunk pc ^ sigma(r).
//   * V stays row-major in LDS; the V^T operand of the PV product is read with
//     ds_read_b64_tr_b16 (each 16-lane group transposes a 4-key x 16-column patch).
//   * LDS is double buffered: one workgroup barrier per KV block.
//   * The running maximum is only raised (and O, l rescaled) when some query of the wave exceeds it
//     by more than 2^8; P stays <= 2^8, exact in the final quotient because O and l share the scale.
// Tiling, operand layouts and the epilogue are those of the first-generation kernel.
#include "salad_internal.h"

namespace salad {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef short s16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

#define LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))
#define GLB_PTR(p) ((const __attribute__((address_space(1))) void *)(p))

namespace {

// position in a head's order -> stored row.  magic = floor(2^32 / T) + 1 gives the exact quotient
// for p * T < 2^32 (checked on the host); magic == 0 selects the plain division.
__device__ inline int row_of_position2(int kind, int p, int T, int HW, unsigned magic)
{
    if (!kind) return p;
    int loc = magic ? (int)__umulhi((unsigned)p, magic) : p / T;
    return (p - loc * T) * HW + loc;
}

__device__ inline uint32_t pack2(float a, float b)
{
    f32x2 x = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf16x2));
}

__device__ inline uint32_t relu2b(uint32_t x)
{
    s16x2 v = __builtin_bit_cast(s16x2, x);
    s16x2 z = {0, 0};
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(v, z));
}

union Frag {
    bf16x8 v;
    uint4 u;
    uint32_t w[4];
    s16x4 h[2];
};

}  // namespace

template <bool DBG>
__global__ __launch_bounds__(256, 2) void sparse_attn_v2_kernel(AttnArgs a, int ntiles, int total, int per_xcd)
{
    constexpr int D = 128, NS = 8, NDT = 4;
    constexpr int TILE = 64 * D;                  // elements per K or V tile (16 KB)
    __shared__ __attribute__((aligned(1024))) u16 Kb[2 * TILE];
    __shared__ __attribute__((aligned(1024))) u16 Vb[2 * TILE];

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
    const int qrow = row_of_position2(kind, qvalid ? qpos : N - 1, T, HW, a.t_magic);

    Frag qf[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s)
        qf[s].u = *reinterpret_cast<const uint4 *>(qb + (size_t)qrow * D + s * 16 + hh * 8);

    // CSR rows of the two query blocks.  A two-entry window per list is kept in registers and
    // refilled one iteration ahead, so the merge never waits on a load.
    const int rowA = h * nb + tile * 2;
    int pa = a.row_ptr[rowA], ea = a.row_ptr[rowA + 1];
    int pb = 0, eb = 0;
    if (tile * 2 + 1 < nb) { pb = ea; eb = a.row_ptr[rowA + 2]; }
    constexpr int NONE = 0x7fffffff;
    int ca0 = pa < ea ? a.col_idx[pa] : NONE, ca1 = pa + 1 < ea ? a.col_idx[pa + 1] : NONE;
    int cb0 = pb < eb ? a.col_idx[pb] : NONE, cb1 = pb + 1 < eb ? a.col_idx[pb + 1] : NONE;

    // ---- global -> LDS: thread owns LDS slots (row 16 i + tid/16, chunk tid%16), i = 0..3
    const int lr = tid >> 4, pc = tid & 15;
    const int kchunk = pc ^ (lr & 15);                 // K: sigma(r) = r & 15
    const int vchunk = pc ^ ((lr & 3) << 2);           // V: sigma(r) = (r & 3) << 2
    auto issue = [&](int blk, int buf) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int p = blk * 64 + i * 16 + lr;
            p = p < N ? p : N - 1;
            const size_t n = (size_t)row_of_position2(kind, p, T, HW, a.t_magic);
            __builtin_amdgcn_global_load_lds(GLB_PTR(kb + n * D + kchunk * 8),
                                             LDS_PTR(Kb + buf * TILE + (i * 256 + wave * 64) * 8), 16, 0, 0);
            __builtin_amdgcn_global_load_lds(GLB_PTR(vb + n * D + vchunk * 8),
                                             LDS_PTR(Vb + buf * TILE + (i * 256 + wave * 64) * 8), 16, 0, 0);
        }
    };

    // ---- LDS read addresses (element offsets inside a tile), loop invariant
    const int kappa = (l32 & 0x13) | ((l32 & 4) << 1) | ((l32 & 8) >> 1);
    int koff[NS];   // K operand: row kappa (+32 kt), logical chunk 2 st + hh
#pragma unroll
    for (int st = 0; st < NS; ++st) koff[st] = kappa * D + (((2 * st + hh) ^ (kappa & 15)) << 3);
    // V operand through the transposing read: this lane supplies the address of keys
    // (8 hh + (l32%16)/4 [+16 c16 + 4 half]) x columns 32 dt + 16 (l32/16) + 4 (l32%4) .. +3
    const int vr = 8 * hh + ((l32 >> 2) & 3);
    int voff[NDT];
#pragma unroll
    for (int dt = 0; dt < NDT; ++dt) {
        int chunk = 4 * dt + 2 * (l32 >> 4) + ((l32 & 3) >> 1);
        voff[dt] = vr * D + ((chunk ^ ((vr & 3) << 2)) << 3) + 4 * (l32 & 1);
    }

    auto next_block = [&](int &blk, int &flags) -> bool {
        blk = ca0 < cb0 ? ca0 : cb0;
        if (blk == NONE) return false;
        const bool fa = ca0 == blk, fb = cb0 == blk;
        flags = (fa ? 1 : 0) | (fb ? 2 : 0);
        if (fa) { ca0 = ca1; ++pa; ca1 = pa + 1 < ea ? a.col_idx[pa + 1] : NONE; }
        if (fb) { cb0 = cb1; ++pb; cb1 = pb + 1 < eb ? a.col_idx[pb + 1] : NONE; }
        return true;
    };

    f32x16 o[NDT];
#pragma unroll
    for (int i = 0; i < NDT; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[i][r] = 0.f;
    float m_run = -1e30f, l_run = 0.f;
    const float c2 = a.scale * 1.44269504088896340736f;

    int blk = 0, flags = 0;
    bool more = next_block(blk, flags);
    if (more) issue(blk, 0);

    auto step = [&](const int buf) -> bool {
        __syncthreads();   // tile `buf` has landed (the fence waits for the LDS loads); buf^1 is free
        const int cur_blk = blk, cur_flags = flags;
        more = next_block(blk, flags);
        if (more) issue(blk, buf ^ 1);
        // the refilled list entries are scalar loads; retire them here so that the waits on LDS
        // data below can be counted instead of waiting for everything
        asm volatile("" ::"s"(ca1), "s"(cb1));
        if ((cur_flags & mybit) && qblk < nb) {
            const u16 *Kt = Kb + buf * TILE;
            const u16 *Vt = Vb + buf * TILE;
            f32x16 s[2];
            {
                // all 16 K fragments are requested before the first product so that LDS latency is
                // paid once per block instead of once per MFMA
                bf16x8 kf[2][NS];
#pragma unroll
                for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                    for (int st = 0; st < NS; ++st)
                        kf[kt][st] = *reinterpret_cast<const bf16x8 *>(Kt + kt * 32 * D + koff[st]);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) s[kt][r] = 0.f;
#pragma unroll
                for (int st = 0; st < NS; ++st) {
                    s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[0][st], qf[st].v, s[0], 0, 0, 0);
                    s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[1][st], qf[st].v, s[1], 0, 0, 0);
                }
            }
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
            mx = fmaxf(mx, __shfl_xor(mx, 32)) * c2;
            if (__any(mx > m_run + 8.0f)) {      // wave-uniform: raise the reference maximum
                const float m_new = fmaxf(m_run, mx);
                const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
                m_run = m_new;
                l_run *= alpha;
#pragma unroll
                for (int i = 0; i < NDT; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o[i][r] *= alpha;
            }
            float psum = 0.f;
            Frag pf[4];
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int r = 0; r < 16; r += 2) {
                    float p0 = __builtin_amdgcn_exp2f(fmaf(s[kt][r], c2, -m_run));
                    float p1 = __builtin_amdgcn_exp2f(fmaf(s[kt][r + 1], c2, -m_run));
                    psum += p0 + p1;
                    pf[kt * 2 + (r >> 3)].w[(r & 7) >> 1] = pack2(p0, p1);
                }
            l_run += psum;
            {
                // V^T fragments are requested a full 16-key group (4 fragments) ahead of their use
                Frag vf[2][NDT];
                auto vread = [&](int c16, Frag (&f)[NDT]) {
#pragma unroll
                    for (int dt = 0; dt < NDT; ++dt) {
                        const u16 *vp = Vt + c16 * 16 * D + voff[dt];
                        f[dt].h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)LDS_PTR(vp));
                        f[dt].h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)LDS_PTR(vp + 4 * D));
                    }
                };
                vread(0, vf[0]);
                vread(1, vf[1]);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int c16 = 0; c16 < 4; ++c16) {
#pragma unroll
                    for (int dt = 0; dt < NDT; ++dt)
                        o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[c16 & 1][dt].v, pf[c16].v, o[dt], 0, 0, 0);
                    if (c16 + 2 < 4) vread(c16 + 2, vf[c16 & 1]);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
        return more;
    };
    if (more) {
        while (true) {
            if (!step(0)) break;
            if (!step(1)) break;
        }
    }

    // ---- epilogue ---------------------------------------------------------------------------------
    float l_tot = l_run + __shfl_xor(l_run, 32);
    const float inv_l = l_tot > 0.f ? 1.f / l_tot : 0.f;
    f32x16 num[NDT];
    float lin_scale = 0.f, inv_den = 0.f;
    const bool lin = a.use_linear && !a.write_sparse_only && !(a.drop && a.drop[bh / a.H]);   // pruned sample (Sec. 4.3): out = O_s
    if (lin) {
        float dpart = 0.f;
        const float *Zh = a.Z + (size_t)bh * D;
#pragma unroll
        for (int st = 0; st < NS; ++st) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                uint32_t w = relu2b(qf[st].w[j]);
                qf[st].w[j] = w;
                dpart = fmaf(__uint_as_float(w << 16), Zh[st * 16 + hh * 8 + 2 * j], dpart);
                dpart = fmaf(__uint_as_float(w & 0xffff0000u), Zh[st * 16 + hh * 8 + 2 * j + 1], dpart);
            }
        }
        const float den = dpart + __shfl_xor(dpart, 32) + a.eps;
        inv_den = 1.f / den;
        lin_scale = a.coef[bh] * inv_den;
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
            pk.x = pack2(ov[0], ov[1]);
            pk.y = pack2(ov[2], ov[3]);
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

hipError_t launch_sparse_attn_v2(const AttnArgs &a, hipStream_t st)
{
    const int ntiles = (a.nb + 1) / 2;
    const int total = a.B * a.H * ntiles;
    const int per_xcd = (total + 7) / 8;
    dim3 grid(per_xcd * 8), block(256);
    const bool dbg = a.o_sparse_dbg || a.o_linear_dbg;
    if (dbg) launch_kernel((sparse_attn_v2_kernel<true>), grid, block, 0, st, a, ntiles, total, per_xcd);
    else launch_kernel((sparse_attn_v2_kernel<false>), grid, block, 0, st, a, ntiles, total, per_xcd);
    return take_launch_status();
}

}  // namespace salad
