// Full Level-1 static projection (Alg. 1 "Proj", Sec. 4.2 layer-wise static scaling):
//   out[b, n, :] = O_s[b, n, :] + lambda s_b (O_l[b, n, :] W_p),   W_p [D x D], D = H d,
// O_l[b, n, :] being the heads' linear-attention outputs concatenated per token.  d = 128, bf16.
//
// A [N, D] x [D, D] GEMM per sample (0.155 TFLOP at the 480p shape) on bf16 MFMA with fp32 accumulation,
// fused with the residual sum.  Like the attention kernels it is computed transposed, C^T = W_p^T O_l^T, so
// that a lane owns one token row: the A operand is a 32 x 16 fragment of a 128 x 128 block of W_p (input head
// h_in, output head h_out), read from LDS; the B operand is 8 consecutive channels of the lane's own O_l row,
// loaded straight from global memory ([B,H,N,d] layout: a head's row is 256 contiguous bytes).
//
//   workgroup = 8 waves = 256 token rows x 2 output heads; a wave owns 64 rows x 128 columns (8 accumulator
//   tiles), so each W_p fragment read from LDS feeds two MFMAs;
//   loop over the H input heads: the two 32 KB blocks W_p[h_in, h_out0..1] are fetched into one half of a
//   128 KB double buffer while the previous pair is being used, and the O_l fragments of the next input head
//   replace the current ones d-step by d-step as they are consumed.
// W_p is static per layer; proj_pack_kernel rearranges it once per call into fragment order (a few
// microseconds for 4.7 MB) so that the GEMM's LDS reads are lane-linear.
#include "salad_internal.h"

namespace salad {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

namespace {
union FragP {
    bf16x8 v;
    uint4 u;
};
constexpr int BLK = 128 * 128;   // elements of one (h_in, h_out) block
}  // namespace

// wfrag[(h_in * H + h_out) * BLK + idx] = W_p[h_in*128 + a][h_out*128 + c] with
// idx = ((c/32 * 8 + a/16) * 64 + ((a%16)/8) * 32 + c%32) * 8 + a%8   (A-operand fragments of the block's transpose)
__global__ __launch_bounds__(256) void proj_pack_kernel(const u16 *__restrict__ w, int H, u16 *__restrict__ wfrag)
{
    const int hi = blockIdx.x, ho = blockIdx.y;
    const size_t D = (size_t)H * 128;
    u16 *dst = wfrag + ((size_t)hi * H + ho) * BLK;
    for (int idx = threadIdx.x; idx < BLK; idx += 256) {
        const int a8 = idx & 7, t = idx >> 3, c32 = t & 31, h2 = (t >> 5) & 1, u = t >> 6, s = u & 7, ct = u >> 3;
        const int a = s * 16 + h2 * 8 + a8, c = ct * 32 + c32;
        dst[idx] = w[((size_t)hi * 128 + a) * D + (size_t)ho * 128 + c];
    }
}

hipError_t launch_proj_pack(const u16 *w_proj, int H, u16 *wfrag, hipStream_t st)
{
    hipLaunchKernelGGL(proj_pack_kernel, dim3(H, H), dim3(256), 0, st, w_proj, H, wfrag);
    return hipGetLastError();
}

__global__ __launch_bounds__(512, 2) void proj_apply_kernel(ProjArgs a)
{
    constexpr int D = 128, NS = 8;
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    u16 *wl = reinterpret_cast<u16 *>(smem);           // [2 buffers][2 output heads][BLK]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hh = lane >> 5;
    const int rg = wave & 3, cg = wave >> 2;
    const int b = blockIdx.z, H = a.H, N = a.N;
    if (a.drop && a.drop[b]) return;                   // pruned sample (Sec. 4.3): out already holds O_s
    const int ho_first = 2 * blockIdx.y;
    const int ho = ho_first + cg;                      // may be == H for the last pair of an odd H
    const int row0 = blockIdx.x * 256 + rg * 64;
    const float coef = a.coef[(size_t)b * H];          // lambda * s_b (the per-head scale is 1 in this form)

    // this wave's O_l rows (clamped at the end of the sequence; the extra rows are never stored)
    const u16 *olrow[2];
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) {
        int row = row0 + rt * 32 + l32;
        row = row < N ? row : N - 1;
        olrow[rt] = a.ol + ((size_t)b * H * N + row) * D + hh * 8;      // + h_in * N * D + st * 16
    }
    FragP bf[2][NS];
    auto load_b = [&](int hi, int st) __attribute__((always_inline)) {
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
            bf[rt][st].u = *reinterpret_cast<const uint4 *>(olrow[rt] + (size_t)hi * N * D + st * 16);
    };
    // both W_p blocks of input head hi -> LDS buffer `buf` (fragment order is lane-linear: plain copy)
    auto stage_w = [&](int hi, int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int x = 0; x < 2; ++x) {
            const int hox = ho_first + x < H ? ho_first + x : H - 1;
            const u16 *src = a.wfrag + ((size_t)hi * H + hox) * BLK;
            u16 *dst = wl + (buf * 2 + x) * BLK;
#pragma unroll
            for (int i = 0; i < BLK / 8 / 512; ++i)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(src + (size_t)(i * 512 + tid) * 8),
                                                 (__attribute__((address_space(3))) void *)(dst + (i * 512 + wave * 64) * 8), 16, 0, 0);
        }
    };

    f32x16 acc[2][4];
#pragma unroll
    for (int rt = 0; rt < 2; ++rt)
#pragma unroll
        for (int ct = 0; ct < 4; ++ct)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[rt][ct][r] = 0.f;

    stage_w(0, 0);
#pragma unroll
    for (int st = 0; st < NS; ++st) load_b(0, st);
    for (int hi = 0; hi < H; ++hi) {
        __builtin_amdgcn_s_waitcnt(0x0F70);           // vmcnt(0): this thread's parts of W_p(hi) and its O_l fragments
        __syncthreads();                               // ... and everybody else's; the other buffer is free again
        if (hi + 1 < H) stage_w(hi + 1, (hi + 1) & 1);
        const u16 *wb = wl + ((hi & 1) * 2 + cg) * BLK;
#pragma unroll
        for (int st = 0; st < NS; ++st) {
#pragma unroll
            for (int ct = 0; ct < 4; ++ct) {
                const bf16x8 af = *reinterpret_cast<const bf16x8 *>(wb + ((ct * NS + st) * 64 + lane) * 8);
                acc[0][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bf[0][st].v, acc[0][ct], 0, 0, 0);
                acc[1][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bf[1][st].v, acc[1][ct], 0, 0, 0);
            }
            if (hi + 1 < H) load_b(hi + 1, st);        // the fragments of this d-step are consumed: fetch the next head's
        }
    }
    if (ho >= H) return;
    // out = O_s + coef * C, one rounding; accumulator register 4 g4 + t of lane (l32, hh) is column
    // 32 ct + 8 g4 + 4 hh + t of row l32
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) {
        const int row = row0 + rt * 32 + l32;
        if (row >= N) continue;
        u16 *orow = a.out + (((size_t)b * H + ho) * N + row) * D;
#pragma unroll
        for (int ct = 0; ct < 4; ++ct)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const int col = ct * 32 + 8 * g4 + 4 * hh;
                const uint2 os = *reinterpret_cast<const uint2 *>(orow + col);
                f32x2 x01 = {fmaf(acc[rt][ct][g4 * 4 + 0], coef, __uint_as_float(os.x << 16)),
                             fmaf(acc[rt][ct][g4 * 4 + 1], coef, __uint_as_float(os.x & 0xffff0000u))};
                f32x2 x23 = {fmaf(acc[rt][ct][g4 * 4 + 2], coef, __uint_as_float(os.y << 16)),
                             fmaf(acc[rt][ct][g4 * 4 + 3], coef, __uint_as_float(os.y & 0xffff0000u))};
                uint2 pk;
                pk.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(x01, bf16x2));
                pk.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(x23, bf16x2));
                *reinterpret_cast<uint2 *>(orow + col) = pk;
            }
    }
}

hipError_t launch_proj_apply(const ProjArgs &a, hipStream_t st)
{
    constexpr int lds = 4 * BLK * 2;                  // 128 KB
    static bool done[16] = {};
    if (hipError_t e = dyn_lds_attr_once(reinterpret_cast<const void *>(proj_apply_kernel), lds, done); e != hipSuccess) return e;
    dim3 grid((a.N + 255) / 256, (a.H + 1) / 2, a.B), block(512);
    hipLaunchKernelGGL(proj_apply_kernel, grid, block, lds, st, a);
    return hipGetLastError();
}

}  // namespace salad
