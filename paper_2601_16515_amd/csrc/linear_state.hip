// Linear-attention state, Eq. (3):  Hs = sum_j relu(K_j)^T V_j  (d x d),  Z = sum_j relu(K_j).
//
// bf16 kernel.  HBM-bound: K and V are each read once (4*N*d bytes per head) for 2*N*d*d flops,
// 64 flop/byte at d = 128 - below the MFMA ridge but above what plain FMAs sustain, so the outer
// products run on bf16 MFMA with fp32 accumulators.  The contraction runs over tokens, which is
// the row index of the stored [N, d] tensors, so both operands must be transposed on the way:
// each thread loads a (TPT tokens x 8 features) patch with 16-byte loads, transposes it in
// registers with byte permutes and writes token-contiguous vectors to LDS; MFMA operands are then
// single 16-byte LDS reads.  The LDS tile is [feature][64 tokens + 8 pad] with the 8-token group
// index XOR-ed by (feature / 16) so that both the 8-byte transposed writes and the 16-byte operand
// reads spread over all banks.
//
// One workgroup (4 waves) owns one d x d accumulator: wave w holds the (w/2, w%2) quadrant.
// The token range of a head is cut into chunks, one workgroup each; the fp32 partial states go to
// the workspace and are added in chunk order by the finalize kernel (no float atomics, so results
// are reproducible run to run).
#include "salad_internal.h"

namespace salad {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

int state_tiles_per_chunk(int BH, int N, int target_wgs)
{
    int tiles = (N + 63) / 64;
    int want = target_wgs / (BH > 0 ? BH : 1);
    if (want < 1) want = 1;
    if (want > tiles) want = tiles;
    return (tiles + want - 1) / want;
}

int state_num_chunks(int BH, int N, int target_wgs)
{
    int tiles = (N + 63) / 64;
    int tpc = state_tiles_per_chunk(BH, N, target_wgs);
    return (tiles + tpc - 1) / tpc;
}

constexpr int XT_PITCH = 72;   // 64 tokens + 8 pad, in bf16 elements (144 bytes)

// element offset of (row = feature, tok) in a transposed tile
__device__ inline int xt_off(int row, int tok)
{
    return row * XT_PITCH + ((((tok >> 3) ^ (row >> 4)) & 7) << 3) + (tok & 7);
}

__device__ inline uint32_t relu_bf16x2(uint32_t x)
{
    s16x2 v = __builtin_bit_cast(s16x2, x);
    s16x2 z = {0, 0};
    v = __builtin_elementwise_max(v, z);   // negative bf16 (sign bit set) is a negative int16
    return __builtin_bit_cast(uint32_t, v);
}

// ROPE: the rotary linear branch (Sec. 4.1): after the ReLU and the Z sums (which stay unrotated), channel pair
// (2p, 2p+1) of token n is rotated by the angle whose cosine and sine sit, as two fp16 values in one word, at
// rope_tab[n * D/2 + p], before it enters the outer products, so the state is sum_j (R_j relu(K_j))^T V_j.
template <int D, bool ROPE = false>
__global__ __launch_bounds__(256, 2) void state_partial_kernel(const u16 *__restrict__ k,
                                                               const u16 *__restrict__ v, int N,
                                                               int tiles_per_chunk, int P,
                                                               float *__restrict__ partial,
                                                               const int32_t *__restrict__ drop, int H,
                                                               const uint32_t *__restrict__ rope_tab = nullptr)
{
    // ROPE: the sample-head index runs fastest over the grid, so that the workgroups that read the same rows of the
    // angle tables (same token chunk, different heads) run at the same time and the tables come from HBM once
    const int bh = ROPE ? blockIdx.x : blockIdx.y, chunk = ROPE ? blockIdx.y : blockIdx.x;
    if (drop && drop[bh / H]) return;                  // pruned sample (Sec. 4.3): K, V are not read
    constexpr int CH = D / 8;          // 16-byte chunks per row
    constexpr int TPT = D / 32;        // tokens per thread per tile (4 for d=128, 2 for d=64)
    constexpr int QT = D / 64;         // 32x32 tiles per side of a wave's quadrant
    __shared__ __attribute__((aligned(16))) u16 KT[D * XT_PITCH];
    __shared__ __attribute__((aligned(16))) u16 VT[D * XT_PITCH];
    __shared__ float zred[4][D];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hh = lane >> 5;
    const int fg = tid % CH, tq = tid / CH;   // feature group (8 features), token group (TPT tokens)
    const u16 *kb = k + (size_t)bh * N * D;
    const u16 *vb = v + (size_t)bh * N * D;
    const int tile0 = chunk * tiles_per_chunk;
    int tile1 = tile0 + tiles_per_chunk;
    const int tiles = (N + 63) / 64;
    if (tile1 > tiles) tile1 = tiles;

    f32x16 acc[QT][QT];
#pragma unroll
    for (int i = 0; i < QT; ++i)
#pragma unroll
        for (int j = 0; j < QT; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    float zacc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) zacc[e] = 0.f;

    // two tiles of global loads are kept in flight per thread (register buffers 0 and 1)
    uint4 kreg[2][TPT], vreg[2][TPT];
    uint4 creg[2][ROPE ? TPT : 1];     // (cos, sin) of the patch's 4 channel pairs
    auto gload = [&](uint4 (&kr)[TPT], uint4 (&vr)[TPT], uint4 *cr, int tile) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < TPT; ++i) {
            int n = tile * 64 + tq * TPT + i;
            if (n < N) {
                kr[i] = *reinterpret_cast<const uint4 *>(kb + (size_t)n * D + fg * 8);
                vr[i] = *reinterpret_cast<const uint4 *>(vb + (size_t)n * D + fg * 8);
                if (ROPE) cr[i] = *reinterpret_cast<const uint4 *>(rope_tab + (size_t)n * (D / 2) + fg * 4);
            } else {
                kr[i] = make_uint4(0, 0, 0, 0);
                vr[i] = make_uint4(0, 0, 0, 0);
                if (ROPE) cr[i] = make_uint4(0x3c00u, 0x3c00u, 0x3c00u, 0x3c00u);   // cos = 1, sin = 0
            }
        }
    };
    // transposed store of a (TPT x 8) patch: for feature f, TPT consecutive tokens
    auto tstore = [&](u16 *dst, const uint4 (&r)[TPT]) __attribute__((always_inline)) {
        uint32_t w[TPT][4];
#pragma unroll
        for (int i = 0; i < TPT; ++i) { w[i][0] = r[i].x; w[i][1] = r[i].y; w[i][2] = r[i].z; w[i][3] = r[i].w; }
#pragma unroll
        for (int f = 0; f < 8; ++f) {
            const uint32_t sel = (f & 1) ? 0x07060302u : 0x05040100u;
            int off = xt_off(fg * 8 + f, tq * TPT);
            if (TPT == 4) {
                uint2 o;
                o.x = __builtin_amdgcn_perm(w[1][f >> 1], w[0][f >> 1], sel);
                o.y = __builtin_amdgcn_perm(w[3][f >> 1], w[2][f >> 1], sel);
                *reinterpret_cast<uint2 *>(dst + off) = o;
            } else {
                uint32_t o = __builtin_amdgcn_perm(w[1][f >> 1], w[0][f >> 1], sel);
                *reinterpret_cast<uint32_t *>(dst + off) = o;
            }
        }
    };

    const int wa = wave >> 1, wc = wave & 1;
    auto step = [&](uint4 (&kr)[TPT], uint4 (&vr)[TPT], uint4 *cr, int tile) __attribute__((always_inline)) {
        // ReLU on K, running sums for Z
#pragma unroll
        for (int i = 0; i < TPT; ++i) {
            kr[i].x = relu_bf16x2(kr[i].x); kr[i].y = relu_bf16x2(kr[i].y);
            kr[i].z = relu_bf16x2(kr[i].z); kr[i].w = relu_bf16x2(kr[i].w);
            uint32_t w4[4] = {kr[i].x, kr[i].y, kr[i].z, kr[i].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                zacc[2 * j] += __uint_as_float(w4[j] << 16);
                zacc[2 * j + 1] += __uint_as_float(w4[j] & 0xffff0000u);
            }
            if (ROPE) {
                const uint32_t cw[4] = {cr[i].x, cr[i].y, cr[i].z, cr[i].w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float x = __uint_as_float(w4[j] << 16), y = __uint_as_float(w4[j] & 0xffff0000u);
                    const f16x2 hcs = __builtin_bit_cast(f16x2, cw[j]);
                    const float cc = (float)hcs[0], ss = (float)hcs[1];
                    f32x2 r = {x * cc - y * ss, x * ss + y * cc};
                    w4[j] = __builtin_bit_cast(uint32_t, __builtin_convertvector(r, bf16x2));
                }
                kr[i] = make_uint4(w4[0], w4[1], w4[2], w4[3]);
            }
        }
        tstore(KT, kr);
        tstore(VT, vr);
        __syncthreads();
        if (tile + 2 < tile1) gload(kr, vr, cr, tile + 2);
#pragma unroll
        for (int s = 0; s < 4; ++s) {   // 16 tokens per MFMA
            bf16x8 af[QT], bfr[QT];
#pragma unroll
            for (int i = 0; i < QT; ++i) {
                int ra = (wa * QT + i) * 32 + l32;
                int rc = (wc * QT + i) * 32 + l32;
                af[i] = *reinterpret_cast<const bf16x8 *>(KT + xt_off(ra, s * 16 + hh * 8));
                bfr[i] = *reinterpret_cast<const bf16x8 *>(VT + xt_off(rc, s * 16 + hh * 8));
            }
#pragma unroll
            for (int i = 0; i < QT; ++i)
#pragma unroll
                for (int j = 0; j < QT; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
        }
        __syncthreads();
    };
    if (tile0 < tile1) gload(kreg[0], vreg[0], creg[0], tile0);
    if (tile0 + 1 < tile1) gload(kreg[1], vreg[1], creg[1], tile0 + 1);
    for (int tile = tile0; tile < tile1; tile += 2) {
        step(kreg[0], vreg[0], creg[0], tile);
        if (tile + 1 < tile1) step(kreg[1], vreg[1], creg[1], tile + 1);
    }

    // partial Hs: accumulator register r of lane (l32, hh) is row a = 8*(r/4) + 4*hh + r%4, col c = l32
    const int per = D * D + D;
    float *out = partial + ((size_t)bh * P + chunk) * per;
#pragma unroll
    for (int i = 0; i < QT; ++i)
#pragma unroll
        for (int j = 0; j < QT; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int a = (wa * QT + i) * 32 + 8 * (r >> 2) + 4 * hh + (r & 3);
                int c = (wc * QT + j) * 32 + l32;
                out[a * D + c] = acc[i][j][r];
            }
    // partial Z: threads with the same fg hold sums over different tokens.  Within a wave the lanes
    // with equal fg are CH apart; across waves go through LDS in wave order.
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        float zz = zacc[e];
        for (int o = CH; o < 64; o <<= 1) zz += __shfl_xor(zz, o);
        zacc[e] = zz;
    }
    if (lane < CH) {
#pragma unroll
        for (int e = 0; e < 8; ++e) zred[wave][lane * 8 + e] = zacc[e];
    }
    __syncthreads();
    if (tid < D) out[D * D + tid] = (zred[0][tid] + zred[1][tid]) + (zred[2][tid] + zred[3][tid]);
}

hipError_t launch_state_partial_bf16(const u16 *k, const u16 *v, int BH, int N, int D,
                                     float *partial, const int32_t *drop, int H, int target_wgs, hipStream_t st,
                                     const uint32_t *rope_tab)
{
    int tpc = state_tiles_per_chunk(BH, N, target_wgs);
    int P = state_num_chunks(BH, N, target_wgs);
    dim3 grid(P, BH), block(256);
    if (rope_tab) {
        if (D != 128) return hipErrorInvalidValue;
        launch_kernel((state_partial_kernel<128, true>), dim3(BH, P), block, 0, st, k, v, N, tpc, P, partial, drop, H, rope_tab);
        return take_launch_status();
    }
    if (D == 128)
        launch_kernel((state_partial_kernel<128, false>), grid, block, 0, st, k, v, N, tpc, P, partial, drop, H, nullptr);
    else
        launch_kernel((state_partial_kernel<64, false>), grid, block, 0, st, k, v, N, tpc, P, partial, drop, H, nullptr);
    return take_launch_status();
}

// (cos, sin) tables of the rotary linear branch, fp32 [n] each -> one word per angle: fp16 cos | fp16 sin << 16
__global__ __launch_bounds__(256) void rope_pack_kernel(const float *__restrict__ c, const float *__restrict__ s_, size_t n,
                                                        uint32_t *__restrict__ out)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    f16x2 h = {(_Float16)c[i], (_Float16)s_[i]};
    out[i] = __builtin_bit_cast(uint32_t, h);
}

hipError_t launch_rope_pack(const float *rope_cos, const float *rope_sin, size_t n, uint32_t *tab, hipStream_t st)
{
    launch_kernel(rope_pack_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, rope_cos, rope_sin, n, tab);
    return take_launch_status();
}

// ------------------------------------------------------------------------------------------------
// fp32 state for small shapes.  A workgroup owns 64 consecutive elements of [Hs | Z] of one head (for d = 64: one
// row a of Hs, so relu(K[n][a]) is one broadcast load and V[n][c] a coalesced one) and splits the tokens over 16
// thread groups (token n goes to group n mod 16); every thread adds its tokens in ascending order with 8 loads in
// flight, the 16 sums are added in group order through LDS: the same result whatever the launch looks like.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void state_f32_kernel(const float *__restrict__ k, const float *__restrict__ v,
                                                         int N, int D, float *__restrict__ Hs, float *__restrict__ Z,
                                                         const int32_t *__restrict__ drop, int H)
{
    __shared__ float part[16][64];
    const int bh = blockIdx.y;
    if (drop && drop[bh / H]) return;                  // pruned sample (Sec. 4.3)
    const int le = threadIdx.x & 63, g = threadIdx.x >> 6;
    const int e = blockIdx.x * 64 + le;
    const bool live = e < D * D + D;
    const bool is_z = e >= D * D;
    const int a = is_z ? e - D * D : e / D, c = is_z ? 0 : e - a * D;
    const float *kb = k + (size_t)bh * N * D + (live ? a : 0);
    const float *vb = v + (size_t)bh * N * D + c;
    float s = 0.f;
    if (live) {
        int n = g;
        for (; n + 7 * 16 < N; n += 8 * 16) {
            float kk[8], vv[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                kk[u] = kb[(size_t)(n + 16 * u) * D];
                vv[u] = is_z ? 1.f : vb[(size_t)(n + 16 * u) * D];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) s = fmaf(fmaxf(kk[u], 0.f), vv[u], s);
        }
        for (; n < N; n += 16) s = fmaf(fmaxf(kb[(size_t)n * D], 0.f), is_z ? 1.f : vb[(size_t)n * D], s);
    }
    part[g][le] = s;
    __syncthreads();
    if (g == 0 && live) {
        float t = part[0][le];
#pragma unroll
        for (int i = 1; i < 16; ++i) t += part[i][le];
        if (is_z) Z[(size_t)bh * D + a] = t;
        else Hs[(size_t)bh * D * D + e] = t;
    }
}

hipError_t launch_state_f32(const float *k, const float *v, int BH, int N, int D, float *Hs, float *Z,
                            const int32_t *drop, int H, hipStream_t st)
{
    dim3 grid((D * D + D + 63) / 64, BH), block(1024);
    launch_kernel(state_f32_kernel, grid, block, 0, st, k, v, N, D, Hs, Z, drop, H);
    return take_launch_status();
}

}  // namespace salad
