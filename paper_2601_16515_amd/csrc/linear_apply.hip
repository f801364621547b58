// Unfused form of the linear apply (Eq. (3) quotient) plus scale-and-sum (Alg. 1 residual
// integration) as one streaming kernel:  out <- out + coef[b,h] * relu(Q) Hs / (relu(Q).Z + eps),
// where `out` holds the sparse branch (bf16) on entry.  HBM-bound: reads Q and O_s, writes O
// (6*N*d bytes per head); the d x d product runs on bf16 MFMA with Hs split into hi + lo parts.
// One wave owns 32 stored rows at a time; the state fragments are staged in LDS once per workgroup.
#include "salad_internal.h"

namespace salad {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
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
    __shared__ __attribute__((aligned(1024))) u16 hf_lds[2 * D * D];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hh = lane >> 5;
    const int bh = blockIdx.y;
    {   // fragments are lane-linear in memory: copy as is (16 bytes per lane per load)
        const u16 *hf = a.hfrag + (size_t)bh * 2 * D * D;
        constexpr int LOADS = 2 * D * D / 8 / 256;
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
                bf16x8 lo = *reinterpret_cast<const bf16x8 *>(hf_lds + D * D + idx);
                num = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lo, qf[st].v, num, 0, 0, 0);
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

hipError_t launch_linear_apply_bf16(const ApplyArgs &a, hipStream_t st)
{
    // rows per workgroup (a multiple of 128): about two workgroups per CU, so that the 2*d*d*2 bytes of
    // state fragments staged in LDS are reused over many rows
    long long rows = ((long long)a.N * a.BH + 511) / 512;
    int rows_per_wg = (int)((rows + 127) / 128) * 128;
    if (rows_per_wg < 128) rows_per_wg = 128;
    dim3 grid((a.N + rows_per_wg - 1) / rows_per_wg, a.BH), block(256);
    if (a.D == 128) hipLaunchKernelGGL(linear_apply_kernel<128>, grid, block, 0, st, a, rows_per_wg);
    else hipLaunchKernelGGL(linear_apply_kernel<64>, grid, block, 0, st, a, rows_per_wg);
    return hipGetLastError();
}

}  // namespace salad
