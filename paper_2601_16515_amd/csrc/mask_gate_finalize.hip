// Block-mask builder, gate (dynamic scale) pass 1, and the finalize kernel that reduces the
// partial linear states and partial gate sums.  gfx950 only.
#include "salad_internal.h"

namespace salad {

// ------------------------------------------------------------------------------------------------
// Sliding-window block mask (Sec. 3 sliding-window attention; App. A.1.1).  One thread per CSR row.
// Row (h, i) keeps kept[h] consecutive KV blocks starting at clamp(i - kept/2, 0, nb - kept).
// Integer work only; the output is a few MB at most and is built once per grid.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void block_mask_kernel(MaskArgs a)
{
    int row = blockIdx.x * blockDim.x + threadIdx.x;
    int rows = a.H * a.nb;
    if (row > rows) return;
    if (row == rows) {
        int h = a.H - 1;
        a.row_ptr[rows] = (int32_t)(a.base[h] + (int64_t)a.nb * a.kept[h]);
        return;
    }
    int h = row / a.nb;
    int i = row - h * a.nb;
    int k = a.kept[h];
    int start = i - k / 2;
    start = start < 0 ? 0 : start;
    start = start > a.nb - k ? a.nb - k : start;
    int64_t off = a.base[h] + (int64_t)i * k;
    a.row_ptr[row] = (int32_t)off;
    for (int j = 0; j < k; ++j) a.col_idx[off + j] = start + j;
}

hipError_t launch_block_mask(const MaskArgs &a, hipStream_t st)
{
    int rows = a.H * a.nb + 1;
    hipLaunchKernelGGL(block_mask_kernel, dim3((rows + 255) / 256), dim3(256), 0, st, a);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Gate pass 1 (Alg. 1 Level 2): sum over a strided set of tokens of sigmoid(x.w + bias).
// One wave per token at a time; a lane owns 8-element chunks lane, lane+64, ... of the row and the
// matching gate weights in registers.  HBM-bound: x_t is read exactly once, 16 bytes per lane per
// load for bf16 (32 for fp32).  Partial sums are written per workgroup and added up in a fixed
// order by the finalize kernel, so the result does not depend on scheduling.
// ------------------------------------------------------------------------------------------------
constexpr int GATE_MAX_CHUNKS = 10;   // D <= 8*64*10 = 5120

template <bool BF16>
__device__ inline void load8(const void *row, int chunk, float (&f)[8])
{
    if (BF16) {
        uint4 u = *reinterpret_cast<const uint4 *>(reinterpret_cast<const u16 *>(row) + chunk * 8);
        uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __uint_as_float(w[i] << 16);
            f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    } else {
        const float4 *p = reinterpret_cast<const float4 *>(reinterpret_cast<const float *>(row) + chunk * 8);
        float4 a = p[0], b = p[1];
        f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w;
        f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
    }
}

template <bool BF16>
__global__ __launch_bounds__(256) void gate_partial_kernel(const void *x_t, const float *__restrict__ w,
                                                           float bias, int N, int D,
                                                           float *__restrict__ partial, int nparts)
{
    __shared__ float wave_sum[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int b = blockIdx.y;
    const int nch = D >> 3;
    float wr[GATE_MAX_CHUNKS][8];
#pragma unroll
    for (int j = 0; j < GATE_MAX_CHUNKS; ++j) {
        int c = lane + 64 * j;
#pragma unroll
        for (int e = 0; e < 8; ++e) wr[j][e] = (c < nch) ? w[c * 8 + e] : 0.f;
    }
    const size_t esz = BF16 ? 2 : 4;
    const char *xb = reinterpret_cast<const char *>(x_t) + (size_t)b * N * D * esz;
    float acc = 0.f;
    for (int n = blockIdx.x * 4 + wave; n < N; n += nparts * 4) {
        const void *row = xb + (size_t)n * D * esz;
        float dot = 0.f;
#pragma unroll
        for (int j = 0; j < GATE_MAX_CHUNKS; ++j) {
            int c = lane + 64 * j;
            if (c < nch) {
                float f[8];
                load8<BF16>(row, c, f);
#pragma unroll
                for (int e = 0; e < 8; ++e) dot = fmaf(f[e], wr[j][e], dot);
            }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) dot += __shfl_xor(dot, o);
        float z = dot + bias;
        acc += 1.f / (1.f + __expf(-z));   // identical in every lane
    }
    if (lane == 0) wave_sum[wave] = acc;
    __syncthreads();
    if (threadIdx.x == 0)
        partial[(size_t)b * nparts + blockIdx.x] = (wave_sum[0] + wave_sum[1]) + (wave_sum[2] + wave_sum[3]);
}

int gate_num_parts(int N)
{
    int parts = (N + 3) / 4;            // at most one token per wave
    return parts < 1024 ? (parts < 1 ? 1 : parts) : 1024;
}

hipError_t launch_gate_partial(const void *x_t, const float *w, float bias, int B, int N, int D,
                               int is_bf16, float *partial, int nparts, hipStream_t st)
{
    dim3 grid(nparts, B), block(256);
    if (is_bf16)
        hipLaunchKernelGGL(gate_partial_kernel<true>, grid, block, 0, st, x_t, w, bias, N, D, partial, nparts);
    else
        hipLaunchKernelGGL(gate_partial_kernel<false>, grid, block, 0, st, x_t, w, bias, N, D, partial, nparts);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Finalize.  Workgroups [0, BH*ceil((D*D+D)/256)) add up the P partial states of one head in chunk
// order (fp32) and emit Hs, Z and the bf16 hi/lo split of Hs laid out as MFMA A-operand fragments
// of Hs^T:  element (a, c) -> ((c/32 * (D/16) + a/16) * 64 + ((a%16)/8)*32 + c%32) * 8 + a%8.
// The last workgroup reduces the gate partial sums (or takes the caller's s), writes s and the
// per-(b, h) coefficient lambda * a_h * s_b of the residual sum (Alg. 1, Sec. 4.2).
// ------------------------------------------------------------------------------------------------
__device__ inline u16 f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (u16)(u >> 16);
}

__global__ __launch_bounds__(256) void finalize_kernel(FinalizeArgs a, int state_blocks, int blocks_per_head)
{
    const int D = a.D;
    if ((int)blockIdx.x < state_blocks) {
        int bh = blockIdx.x / blocks_per_head;
        int e = (blockIdx.x - bh * blocks_per_head) * 256 + threadIdx.x;
        int per = D * D + D;
        if (e >= per) return;
        const float *p = a.state_partial + (size_t)bh * a.P * per + e;
        float s = 0.f;
        for (int c = 0; c < a.P; ++c) s += p[(size_t)c * per];
        if (e < D * D) {
            a.Hs[(size_t)bh * D * D + e] = s;
            if (a.hfrag) {
                int row = e / D, col = e - row * D;   // Hs[row = a][col = c]
                u16 hi = f32_to_bf16_rne(s);
                float rem = s - __uint_as_float((uint32_t)hi << 16);
                u16 lo = f32_to_bf16_rne(rem);
                int idx = ((col / 32 * (D / 16) + row / 16) * 64 + ((row % 16) / 8) * 32 + col % 32) * 8 + row % 8;
                a.hfrag[(size_t)bh * 2 * D * D + idx] = hi;
                a.hfrag[(size_t)bh * 2 * D * D + D * D + idx] = lo;
            }
        } else {
            a.Z[(size_t)bh * D + (e - D * D)] = s;
        }
        return;
    }
    // dynamic scale and coefficients: one workgroup, fixed summation order
    __shared__ float red[256];
    __shared__ float s_sh;
    for (int b = 0; b < a.B; ++b) {
        float s;
        if (a.nparts > 0) {
            float t = 0.f;
            for (int i = threadIdx.x; i < a.nparts; i += 256) t += a.gate_partial[(size_t)b * a.nparts + i];
            red[threadIdx.x] = t;
            __syncthreads();
            for (int o = 128; o > 0; o >>= 1) {
                if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
                __syncthreads();
            }
            if (threadIdx.x == 0) s_sh = red[0] / (float)a.N;
            __syncthreads();
            s = s_sh;
            __syncthreads();
        } else {
            s = a.s_dev[b];
        }
        if (threadIdx.x == 0) {
            a.s_ws[b] = s;
            if (a.s_out) a.s_out[b] = s;
        }
        if (a.coef)
            for (int h = threadIdx.x; h < a.H; h += 256)
                a.coef[b * a.H + h] = a.lambda * (a.head_scale ? a.head_scale[h] : 1.f) * s;
    }
}

hipError_t launch_finalize(const FinalizeArgs &a, hipStream_t st)
{
    int per = a.D * a.D + a.D;
    int blocks_per_head = (per + 255) / 256;
    int state_blocks = a.P > 0 ? a.B * a.H * blocks_per_head : 0;
    hipLaunchKernelGGL(finalize_kernel, dim3(state_blocks + (a.do_gate ? 1 : 0)), dim3(256), 0, st, a, state_blocks, blocks_per_head);
    return hipGetLastError();
}

}  // namespace salad
