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
        a.row_ptr[rows] = (int32_t)a.total;
        return;
    }
    int h = row / a.nb;
    int i = row - h * a.nb;
    int k = a.kept[h];
    if (a.truncated) {
        // the blocks of [i - l, i - l + k) that exist; rows before l miss l - r' blocks (r' the row), rows after
        // nb - 1 - r miss 1, 2, ... : the row's first entry follows in closed form
        const int l = k / 2, r = k - 1 - l;
        const int lo = i - l < 0 ? 0 : i - l, hi = i - l + k > a.nb ? a.nb : i - l + k;
        const int64_t m = i < l ? i : l, t = i - (a.nb - r) > 0 ? i - (a.nb - r) : 0;
        const int64_t off = a.base[h] + (int64_t)i * k - (m * l - m * (m - 1) / 2) - t * (t + 1) / 2;
        a.row_ptr[row] = (int32_t)off;
        for (int j = lo; j < hi; ++j) a.col_idx[off + (j - lo)] = j;
        return;
    }
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
    launch_kernel(block_mask_kernel, dim3((rows + 255) / 256), dim3(256), 0, st, a);
    return take_launch_status();
}

// ------------------------------------------------------------------------------------------------
// Gate pass 1 (Alg. 1 Level 2): sum over a strided set of tokens of sigmoid(x.w + bias).
// One wave per token at a time; a lane owns 8-element chunks lane, lane+64, ... of the row and the
// matching gate weights in registers.  HBM-bound: x_t is read exactly once, 16 bytes per lane per
// load for bf16 (32 for fp32).  Partial sums are written per workgroup and added up in a fixed
// order by the finalize kernel, so the result does not depend on scheduling.
// ------------------------------------------------------------------------------------------------
constexpr int GATE_MAX_CHUNKS = 10;   // D <= 8*64*10 = 5120

// Raw 8-element chunk of a row: 16 bytes (bf16) or 32 bytes (fp32) per lane.
template <bool BF16> struct Chunk8;
template <> struct Chunk8<true> {
    uint4 u;
    __device__ inline void load(const void *row, int chunk) { u = *reinterpret_cast<const uint4 *>(reinterpret_cast<const u16 *>(row) + chunk * 8); }
    __device__ inline void zero() { u = make_uint4(0, 0, 0, 0); }
    __device__ inline float dot(const float (&w)[8], float acc) const
    {
        const uint32_t v[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            acc = fmaf(__uint_as_float(v[i] << 16), w[2 * i], acc);
            acc = fmaf(__uint_as_float(v[i] & 0xffff0000u), w[2 * i + 1], acc);
        }
        return acc;
    }
};
template <> struct Chunk8<false> {
    float v[8];
    __device__ inline void load(const void *row, int chunk)
    {
        const float4 *p = reinterpret_cast<const float4 *>(reinterpret_cast<const float *>(row) + chunk * 8);
        const float4 a = p[0], b = p[1];
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    }
    __device__ inline void zero()
    {
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = 0.f;
    }
    __device__ inline float dot(const float (&w)[8], float acc) const
    {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc = fmaf(v[i], w[i], acc);
        return acc;
    }
};

// NCH: 8-element chunks per lane (D <= 512 * NCH); TOK: tokens a wave handles per step.  The loads of the
// next step are issued before the current step is reduced (two register buffers), so a wave always has
// TOK*NCH 16-byte loads per lane in flight while it runs the dot products, the wave reduction and the
// sigmoid of the previous tokens.
template <bool BF16, int NCH, int TOK>
__global__ __launch_bounds__(256) void gate_partial_kernel(const void *x_t, const float *__restrict__ w,
                                                           float bias, int N, int D,
                                                           float *__restrict__ partial, int nparts)
{
    __shared__ float wave_sum[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int b = blockIdx.y;
    const int nch = D >> 3;
    float wr[NCH][8];
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
        int c = lane + 64 * j;
#pragma unroll
        for (int e = 0; e < 8; ++e) wr[j][e] = (c < nch) ? w[c * 8 + e] : 0.f;
    }
    const size_t esz = BF16 ? 2 : 4;
    const char *xb = reinterpret_cast<const char *>(x_t) + (size_t)b * N * D * esz;
    const int stride = nparts * 4 * TOK;
    float acc = 0.f;
    Chunk8<BF16> bufA[TOK][NCH], bufB[TOK][NCH];
    auto issue = [&](Chunk8<BF16> (&buf)[TOK][NCH], int n0) __attribute__((always_inline)) {
#pragma unroll
        for (int t = 0; t < TOK; ++t) {
            const int n = n0 + t < N ? n0 + t : N - 1;
            const void *row = xb + (size_t)n * D * esz;
#pragma unroll
            for (int j = 0; j < NCH; ++j) {
                const int c = lane + 64 * j;
                if (c < nch) buf[t][j].load(row, c);
                else buf[t][j].zero();
            }
        }
    };
    auto consume = [&](const Chunk8<BF16> (&buf)[TOK][NCH], int n0) __attribute__((always_inline)) {
        float dot[TOK];
#pragma unroll
        for (int t = 0; t < TOK; ++t) {
            dot[t] = 0.f;
#pragma unroll
            for (int j = 0; j < NCH; ++j) dot[t] = buf[t][j].dot(wr[j], dot[t]);
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1)
#pragma unroll
            for (int t = 0; t < TOK; ++t) dot[t] += __shfl_xor(dot[t], o);
#pragma unroll
        for (int t = 0; t < TOK; ++t)
            if (n0 + t < N) acc += 1.f / (1.f + __expf(-(dot[t] + bias)));   // identical in every lane
    };
    int n0 = (blockIdx.x * 4 + wave) * TOK;
    if (n0 < N) issue(bufA, n0);
    while (n0 < N) {
        if (n0 + stride < N) issue(bufB, n0 + stride);
        consume(bufA, n0);
        n0 += stride;
        if (n0 >= N) break;
        if (n0 + stride < N) issue(bufA, n0 + stride);
        consume(bufB, n0);
        n0 += stride;
    }
    if (lane == 0) wave_sum[wave] = acc;
    __syncthreads();
    if (threadIdx.x == 0)
        partial[(size_t)b * nparts + blockIdx.x] = (wave_sum[0] + wave_sum[1]) + (wave_sum[2] + wave_sum[3]);
}

// Rows wider than the register-resident weights allow (5120 < D <= 8192, e.g. 64 heads of 128 channels): the gate
// weights live in LDS (32 KB) and every lane reads the 8 weights of a chunk from there; one token per wave step, the
// next token's chunks are requested before the current one is reduced.  Same partial sums, same reduce afterwards.
constexpr int GATE_WIDE_MAX_CHUNKS = 16;   // D <= 8*64*16 = 8192
template <bool BF16>
__global__ __launch_bounds__(256) void gate_partial_wide_kernel(const void *x_t, const float *__restrict__ w, float bias, int N, int D,
                                                                float *__restrict__ partial, int nparts)
{
    __shared__ __attribute__((aligned(16))) float wsh[GATE_WIDE_MAX_CHUNKS * 64 * 8];
    __shared__ float wave_sum[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int b = blockIdx.y;
    const int nch = D >> 3;
    for (int i = threadIdx.x; i < GATE_WIDE_MAX_CHUNKS * 64 * 8; i += 256) wsh[i] = i < D ? w[i] : 0.f;
    __syncthreads();
    const size_t esz = BF16 ? 2 : 4;
    const char *xb = reinterpret_cast<const char *>(x_t) + (size_t)b * N * D * esz;
    const int stride = nparts * 4;
    float acc = 0.f;
    Chunk8<BF16> bufA[GATE_WIDE_MAX_CHUNKS], bufB[GATE_WIDE_MAX_CHUNKS];
    auto issue = [&](Chunk8<BF16> (&buf)[GATE_WIDE_MAX_CHUNKS], int n) __attribute__((always_inline)) {
        const void *row = xb + (size_t)n * D * esz;
#pragma unroll
        for (int j = 0; j < GATE_WIDE_MAX_CHUNKS; ++j) {
            const int c = lane + 64 * j;
            if (c < nch) buf[j].load(row, c);
            else buf[j].zero();
        }
    };
    auto consume = [&](const Chunk8<BF16> (&buf)[GATE_WIDE_MAX_CHUNKS]) __attribute__((always_inline)) {
        float dot = 0.f;
#pragma unroll
        for (int j = 0; j < GATE_WIDE_MAX_CHUNKS; ++j) {
            const float4 w0 = *reinterpret_cast<const float4 *>(wsh + (lane + 64 * j) * 8);
            const float4 w1 = *reinterpret_cast<const float4 *>(wsh + (lane + 64 * j) * 8 + 4);
            const float wr[8] = {w0.x, w0.y, w0.z, w0.w, w1.x, w1.y, w1.z, w1.w};
            dot = buf[j].dot(wr, dot);
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) dot += __shfl_xor(dot, o);
        acc += 1.f / (1.f + __expf(-(dot + bias)));   // identical in every lane
    };
    int n = blockIdx.x * 4 + wave;
    if (n < N) issue(bufA, n);
    while (n < N) {
        if (n + stride < N) issue(bufB, n + stride);
        consume(bufA);
        n += stride;
        if (n >= N) break;
        if (n + stride < N) issue(bufA, n + stride);
        consume(bufB);
        n += stride;
    }
    if (lane == 0) wave_sum[wave] = acc;
    __syncthreads();
    if (threadIdx.x == 0)
        partial[(size_t)b * nparts + blockIdx.x] = (wave_sum[0] + wave_sum[1]) + (wave_sum[2] + wave_sum[3]);
}

constexpr int GATE_MAX_PARTS = 512;

int gate_num_parts(int N)
{
    int parts = (N + 15) / 16;          // a workgroup step covers 16 tokens (4 waves x up to 4 tokens)
    return parts < GATE_MAX_PARTS ? (parts < 1 ? 1 : parts) : GATE_MAX_PARTS;
}

static void gate_dispatch_bf16(dim3 grid, dim3 block, hipStream_t st, const void *x_t, const float *w, float bias, int N, int D,
                               float *partial, int nparts)
{
    const int nch = (D / 8 + 63) / 64;
    if (nch <= 1) launch_kernel((gate_partial_kernel<true, 1, 4>), grid, block, 0, st, x_t, w, bias, N, D, partial, nparts);
    else if (nch <= 2) launch_kernel((gate_partial_kernel<true, 2, 4>), grid, block, 0, st, x_t, w, bias, N, D, partial, nparts);
    else if (nch <= 3) launch_kernel((gate_partial_kernel<true, 3, 2>), grid, block, 0, st, x_t, w, bias, N, D, partial, nparts);
    else if (nch <= 5) launch_kernel((gate_partial_kernel<true, 5, 2>), grid, block, 0, st, x_t, w, bias, N, D, partial, nparts);
    else if (nch <= GATE_MAX_CHUNKS) launch_kernel((gate_partial_kernel<true, GATE_MAX_CHUNKS, 1>), grid, block, 0, st, x_t, w, bias, N, D, partial, nparts);
    else launch_kernel((gate_partial_wide_kernel<true>), grid, block, 0, st, x_t, w, bias, N, D, partial, nparts);
}

// fp32 inputs are the small-shape path: one token per wave step
static void gate_dispatch_f32(dim3 grid, dim3 block, hipStream_t st, const void *x_t, const float *w, float bias, int N, int D,
                              float *partial, int nparts)
{
    const int nch = (D / 8 + 63) / 64;
    if (nch <= 2) launch_kernel((gate_partial_kernel<false, 2, 1>), grid, block, 0, st, x_t, w, bias, N, D, partial, nparts);
    else if (nch <= 5) launch_kernel((gate_partial_kernel<false, 5, 1>), grid, block, 0, st, x_t, w, bias, N, D, partial, nparts);
    else if (nch <= GATE_MAX_CHUNKS) launch_kernel((gate_partial_kernel<false, GATE_MAX_CHUNKS, 1>), grid, block, 0, st, x_t, w, bias, N, D, partial, nparts);
    else launch_kernel((gate_partial_wide_kernel<false>), grid, block, 0, st, x_t, w, bias, N, D, partial, nparts);
}

hipError_t launch_gate_partial(const void *x_t, const float *w, float bias, int B, int N, int D,
                               int is_bf16, float *partial, int nparts, hipStream_t st)
{
    dim3 grid(nparts, B), block(256);
    if (is_bf16) gate_dispatch_bf16(grid, block, st, x_t, w, bias, N, D, partial, nparts);
    else gate_dispatch_f32(grid, block, st, x_t, w, bias, N, D, partial, nparts);
    return take_launch_status();
}

// ------------------------------------------------------------------------------------------------
// Finalize.  Workgroups [0, BH*ceil((D*D+D)/64)) add up the P partial states of one head in chunk
// order (fp32) and emit Hs, Z and Hs rounded to bf16 laid out as MFMA A-operand fragments
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
    __shared__ float part[4][64];
    if ((int)blockIdx.x < state_blocks) {
        // 64 state elements per workgroup; the P partials are split over 4 thread groups (more loads in
        // flight), each group adds its share in chunk order, the 4 sums are added in group order
        const int bh = blockIdx.x / blocks_per_head;
        if (a.drop && a.drop[bh / a.H]) return;        // pruned sample: its partial states were not computed
        const int le = threadIdx.x & 63, grp = threadIdx.x >> 6;
        const int e = (blockIdx.x - bh * blocks_per_head) * 64 + le;
        const int per = D * D + D;
        float s = 0.f;
        if (e < per) {
            const float *p = a.state_partial + (size_t)bh * a.P * per + e;
            const int c0 = (a.P * grp) / 4, c1 = (a.P * (grp + 1)) / 4;
            for (int c = c0; c < c1; ++c) s += p[(size_t)c * per];
        }
        part[grp][le] = s;
        __syncthreads();
        if (grp != 0 || e >= per) return;
        s = (part[0][le] + part[1][le]) + (part[2][le] + part[3][le]);
        if (e < D * D) {
            a.Hs[(size_t)bh * D * D + e] = s;
            if (a.hfrag) {
                int row = e / D, col = e - row * D;   // Hs[row = a][col = c]
                int idx = ((col / 32 * (D / 16) + row / 16) * 64 + ((row % 16) / 8) * 32 + col % 32) * 8 + row % 8;
                a.hfrag[(size_t)bh * D * D + idx] = f32_to_bf16_rne(s);
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
        const bool dropped = a.drop != nullptr && s < a.tau;      // Sec. 4.3: scale below the threshold
        if (threadIdx.x == 0) {
            a.s_ws[b] = s;
            if (a.s_out) a.s_out[b] = s;
            if (a.drop) a.drop[b] = dropped ? 1 : 0;
            if (a.dropped_out) a.dropped_out[b] = dropped ? 1 : 0;
        }
        if (a.coef)
            for (int h = threadIdx.x; h < a.H; h += 256)
                a.coef[b * a.H + h] = dropped ? 0.f : a.lambda * (a.head_scale ? a.head_scale[h] : 1.f) * s;
    }
}

hipError_t launch_finalize(const FinalizeArgs &a, hipStream_t st)
{
    int per = a.D * a.D + a.D;
    int blocks_per_head = (per + 63) / 64;
    int state_blocks = a.P > 0 ? a.B * a.H * blocks_per_head : 0;
    launch_kernel(finalize_kernel, dim3(state_blocks + (a.do_gate ? 1 : 0)), dim3(256), 0, st, a, state_blocks, blocks_per_head);
    return take_launch_status();
}

}  // namespace salad
