// Full Level-1 static projection (Alg. 1 "Proj", Sec. 4.2 layer-wise static scaling):
//   out[b, n, :] = O_s[b, n, :] + lambda s_b (O_l[b, n, :] W_p),   W_p [D x D], D = H d,
// O_l[b, n, :] being the heads' linear-attention outputs concatenated per token.  d = 128, bf16.
//
// A [N, D] x [D, D] GEMM per sample (0.155 TFLOP at the 480p shape) on bf16 MFMA with fp32 accumulation,
// fused with the residual sum.  Like the attention kernels it is computed transposed, C^T = W_p^T O_l^T, so
// that a lane owns one token row: the A operand is a 32 x 16 fragment of a 128 x 128 block of W_p (input head
// h_in, output head h_out) read from LDS, the B operand 8 consecutive channels of the lane's own O_l row,
// loaded from global memory into registers.
//
//   workgroup = 4 waves = 256 token rows x 1 output head, two workgroups per CU (one's epilogue and barrier
//   waits run under the other's MFMAs); a wave owns 64 rows x 128 columns (8 accumulator tiles), so each W_p
//   fragment read from LDS feeds two MFMAs;
//   the contraction runs in steps of 32 input channels: per step 8 KB of W_p fragments go
//   straight from global memory into one of four LDS stages and each wave's own four O_l fragments into
//   registers (the producer writes O_l in fragment order, so a fragment is 1 KB of contiguous memory), three
//   steps ahead of their use (counted waits, one barrier per step);
//   the epilogue turns the accumulators into row layout through LDS, so that O_s is read and the sum written
//   in full 128-byte segments.
// W_p is static per layer; proj_pack_kernel rearranges it once per call into fragment order (a few
// microseconds for 4.7 MB) so that the GEMM's LDS reads are lane-linear.
#include "salad_internal.h"
#include <type_traits>

namespace salad {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

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
    // a workgroup takes 32 input channels (two d-steps) of one (h_in, h_out) block: rows read in full 256-byte
    // segments into LDS, the 8 fragments written 16 bytes per lane in lane order
    __shared__ uint32_t tile[32][65];                  // [a - 32 j][c / 2], padded
    const int hi = blockIdx.x, ho = blockIdx.y, j = blockIdx.z;
    const size_t D = (size_t)H * 128;
    const u16 *src = w + ((size_t)hi * 128 + 32 * j) * D + (size_t)ho * 128;
#pragma unroll
    for (int i = threadIdx.x; i < 32 * 64; i += 256) {
        const int r = i >> 6, c2 = i & 63;
        tile[r][c2] = *reinterpret_cast<const uint32_t *>(src + (size_t)r * D + 2 * c2);
    }
    __syncthreads();
    u16 *dst = wfrag + ((size_t)hi * H + ho) * BLK;
#pragma unroll
    for (int q = threadIdx.x; q < 8 * 64; q += 256) {
        const int c32 = q & 31, h2 = (q >> 5) & 1, s2 = (q >> 6) & 1, ct = q >> 7;
        const int t = (ct * 8 + 2 * j + s2) * 64 + h2 * 32 + c32;   // 16-byte slot of the packed block
        const int a0 = s2 * 16 + h2 * 8, c = ct * 32 + c32;
        uint32_t v[8];
#pragma unroll
        for (int a8 = 0; a8 < 8; ++a8) v[a8] = (tile[a0 + a8][c >> 1] >> ((c & 1) * 16)) & 0xffffu;
        *reinterpret_cast<uint4 *>(dst + (size_t)t * 8) =
            make_uint4(v[0] | (v[1] << 16), v[2] | (v[3] << 16), v[4] | (v[5] << 16), v[6] | (v[7] << 16));
    }
}

hipError_t launch_proj_pack(const u16 *w_proj, int H, u16 *wfrag, hipStream_t st)
{
    launch_kernel(proj_pack_kernel, dim3(H, H, 4), dim3(256), 0, st, w_proj, H, wfrag);
    return take_launch_status();
}

// One 16-byte-per-lane global -> LDS load (lane i lands at lds_addr + 16 i), issued through inline assembly so
// that its completion is tracked by hand with counted waits (several stages stay in flight across barriers).
__device__ inline void proj_dma16(const void *base_uniform, unsigned lane_off, unsigned lds_addr_uniform)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(lds_addr_uniform), "v"(lane_off), "s"(base_uniform) : "memory", "m0");
}

template <int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (N > 0) {
        static_for<N - 1>(f);
        f(std::integral_constant<int, N - 1>{});
    }
}

__global__ __launch_bounds__(256, 2) void proj_apply_kernel(ProjArgs a)
{
    constexpr int D = 128;
    constexpr int NSTAGE = 4, PDIST = 3;              // stages; stages in flight ahead of the one in use
    constexpr int STAGE_B = 8 * 1024;                  // LDS per stage: 8 W_p fragments of 1 KB
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hh = lane >> 5;
    const int rg = wave;
    const int H = a.H, N = a.N;
    // Workgroup -> (sample, row tile, output head).  Consecutive workgroup ids go to the 8 XCDs in turn, each
    // with its own L2; the H workgroups that share a row tile (and so the same 256 x D slice of O_l, which each
    // of them reads completely) are given consecutive slots of ONE XCD, so that they run side by side and the
    // slice comes from HBM once and from that L2 for the rest.
    const int ny = H, nrt = (N + 255) >> 8, ngrp = (nrt + 7) >> 3;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int ho = slot % ny, grp = slot / ny;
    const int b = grp / ngrp, rtile = (grp % ngrp) * 8 + xcd;
    if (rtile >= nrt) return;
    if (a.drop && a.drop[b]) return;                   // pruned sample (Sec. 4.3): out already holds O_s
    const int tile_row0 = rtile * 256;
    const float coef = a.coef[(size_t)b * H];          // lambda * s_b (the per-head scale is 1 in this form)
    const unsigned lds0 = __builtin_amdgcn_readfirstlane((unsigned)(size_t)((__attribute__((address_space(3))) unsigned char *)smem));
    const unsigned wave_u = (unsigned)__builtin_amdgcn_readfirstlane(wave);

    // ---- stage kk (k = 32 kk .. 32 kk + 31 of the D_in = 128 H contraction), 6 loads per lane:
    //   W_p -> LDS buffer kk % NSTAGE: the 8 fragments (4 column tiles x 2 d-steps) of this k range, 1 KB each, in
    //        the order (ct, s'); the packed block keeps fragment (ct, st) at ((ct*8 + st)*64 + lane)*8.  Wave w
    //        copies the two fragments of column tile w.
    //   O_l -> registers: the wave's own 2 x 2 fragments (row tile rt, d-step s'), each 1 KB of contiguous memory.
    const unsigned lane16 = (unsigned)lane * 16u;
    const int nt32 = (N + 31) >> 5;
    const unsigned char *olb[2];
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) {
        int t32 = __builtin_amdgcn_readfirstlane(tile_row0 / 32 + rg * 2 + rt);
        t32 = t32 < nt32 ? t32 : nt32 - 1;             // rows past N: any valid block, the results are not stored
        olb[rt] = reinterpret_cast<const unsigned char *>(a.ol) + (((size_t)b * nt32 + t32) * H << 13);
    }
    const unsigned char *wsrc = reinterpret_cast<const unsigned char *>(a.wfrag) + (size_t)ho * (BLK * 2) + (size_t)wave_u * 8192;
    // load i (0..5) of stage kk; a whole stage is stage_load(kk, 0..5, ...) in this order
    auto stage_load = [&](int kk, int i, u32x4 (&bq)[2][2]) __attribute__((always_inline)) {
        const int hi = kk >> 2, q4 = kk & 3;           // input head, quarter of its 128 channels
        if (i < 2) {
            const unsigned buf = lds0 + (unsigned)(kk % NSTAGE) * STAGE_B + wave_u * 2048u;
            const size_t woff = (size_t)hi * H * (BLK * 2) + q4 * 2048;
            proj_dma16(wsrc + woff + i * 1024, lane16, buf + i * 1024u);
        } else {
            const int rt = (i - 2) >> 1;
            const unsigned char *src = olb[rt] + ((size_t)hi << 13) + q4 * 2048;
            if (i & 1) asm volatile("global_load_dwordx4 %0, %1, %2 offset:1024" : "=v"(bq[rt][1]) : "v"(lane16), "s"(src) : "memory");
            else asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(bq[rt][0]) : "v"(lane16), "s"(src) : "memory");
        }
    };
    auto stage = [&](int kk, u32x4 (&bq)[2][2]) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 6; ++i) stage_load(kk, i, bq);
    };

    f32x16 acc[2][4];
#pragma unroll
    for (int rt = 0; rt < 2; ++rt)
#pragma unroll
        for (int ct = 0; ct < 4; ++ct)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[rt][ct][r] = 0.f;

    const int nk = 4 * H;                              // a multiple of NSTAGE
    u32x4 bq[NSTAGE][2][2];                            // O_l fragments of the stages in flight
    stage(0, bq[0]);
    stage(1, bq[1]);
    stage(2, bq[2]);
    const unsigned aoff = lane16;                      // + (ct*2 + s') * 1024
    for (int kk0 = 0; kk0 < nk; kk0 += NSTAGE) {
        static_for<NSTAGE>([&](auto uc) __attribute__((always_inline)) {
            constexpr int u = decltype(uc)::value;
            const int kk = kk0 + u;
            // stage kk must have landed; up to PDIST - 1 newer stages (6 loads each) may stay in flight
            // (nk is a multiple of NSTAGE: only the last two steps of the last group have fewer behind them)
            constexpr int LPS = 6;                     // loads per stage
            if (u <= 1 || kk0 + NSTAGE < nk) __builtin_amdgcn_s_waitcnt(0x0F70 | (2 * LPS));
            else if (u == 2) __builtin_amdgcn_s_waitcnt(0x0F70 | LPS);
            else __builtin_amdgcn_s_waitcnt(0x0F70);
            // the fragment registers are defined from here on (the loads above complete asynchronously)
            asm volatile("" : "+v"(bq[u][0][0]), "+v"(bq[u][0][1]), "+v"(bq[u][1][0]), "+v"(bq[u][1][1]));
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            // 8 x (W_p fragment from LDS, one ahead; 2 MFMAs); the 6 loads of stage kk + PDIST (its LDS buffer was
            // read in step kk - 1, its registers too) go out one at a time between them, so that a full memory
            // queue never holds up a wave that has MFMAs to issue
            const bool more = kk + PDIST < nk;
            const unsigned char *buf = smem + u * STAGE_B + aoff;
            FragP af[2];
            auto read_a = [&](int i) __attribute__((always_inline)) {      // i = sp * 4 + ct
                af[i & 1].u = *reinterpret_cast<const uint4 *>(buf + ((i & 3) * 2 + (i >> 2)) * 1024);
            };
            read_a(0);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int sp = i >> 2, ct = i & 3;
                if (i + 1 < 8) read_a(i + 1);
                acc[0][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i & 1].v, __builtin_bit_cast(bf16x8, bq[u][0][sp]), acc[0][ct], 0, 0, 0);
                acc[1][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i & 1].v, __builtin_bit_cast(bf16x8, bq[u][1][sp]), acc[1][ct], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (more && i < 6) stage_load(kk + PDIST, i, bq[(u + PDIST) % NSTAGE]);
                __builtin_amdgcn_sched_barrier(0);
            }
        });
    }
    __builtin_amdgcn_s_barrier();                      // every wave is done with the stages: they become staging space
    asm volatile("" ::: "memory");
    // ---- out = O_s + coef * C, one rounding.  Accumulator layout (lane = row l32; register 4 g4 + t = column
    // 32 ct + 8 g4 + 4 hh + t) -> wave-private 8 KB of LDS (fp32, rows of 64 columns = 16 chunks of 16 bytes,
    // chunk ^ (row & 15)) -> row layout (8 rows x 8 chunks of 8 columns per instruction), so that O_s is read
    // and out written in full 128-byte segments.
    unsigned char *stg = smem + wave * 8192;
    const int r8 = lane >> 3, c8 = lane & 7;
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) {
        const int row_base = tile_row0 + rg * 64 + rt * 32;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            uint4 os[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                int row = row_base + 8 * k + r8;
                row = row < N ? row : N - 1;
                os[k] = *reinterpret_cast<const uint4 *>(a.out + (((size_t)b * H + ho) * N + row) * D + h * 64 + c8 * 8);
            }
#pragma unroll
            for (int dl = 0; dl < 2; ++dl)
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) {
                    const int chunk = dl * 8 + 2 * g4 + hh;
                    const f32x16 &c = acc[rt][2 * h + dl];
                    *reinterpret_cast<float4 *>(stg + l32 * 256 + ((chunk ^ (l32 & 15)) << 4)) =
                        make_float4(c[g4 * 4 + 0] * coef, c[g4 * 4 + 1] * coef, c[g4 * 4 + 2] * coef, c[g4 * 4 + 3] * coef);
                }
            asm volatile("" ::: "memory");             // the wave's LDS operations execute in order
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int lrow = 8 * k + r8;
                const float4 n0 = *reinterpret_cast<const float4 *>(stg + lrow * 256 + (((2 * c8) ^ (lrow & 15)) << 4));
                const float4 n1 = *reinterpret_cast<const float4 *>(stg + lrow * 256 + (((2 * c8 + 1) ^ (lrow & 15)) << 4));
                const uint4 o4 = os[k];
                f32x2 x0 = {__uint_as_float(o4.x << 16) + n0.x, __uint_as_float(o4.x & 0xffff0000u) + n0.y};
                f32x2 x1 = {__uint_as_float(o4.y << 16) + n0.z, __uint_as_float(o4.y & 0xffff0000u) + n0.w};
                f32x2 x2 = {__uint_as_float(o4.z << 16) + n1.x, __uint_as_float(o4.z & 0xffff0000u) + n1.y};
                f32x2 x3 = {__uint_as_float(o4.w << 16) + n1.z, __uint_as_float(o4.w & 0xffff0000u) + n1.w};
                uint4 pk;
                pk.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(x0, bf16x2));
                pk.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(x1, bf16x2));
                pk.z = __builtin_bit_cast(uint32_t, __builtin_convertvector(x2, bf16x2));
                pk.w = __builtin_bit_cast(uint32_t, __builtin_convertvector(x3, bf16x2));
                const int row = row_base + lrow;
                if (row < N) *reinterpret_cast<uint4 *>(a.out + (((size_t)b * H + ho) * N + row) * D + h * 64 + c8 * 8) = pk;
            }
            asm volatile("" ::: "memory");
        }
    }
}

hipError_t launch_proj_apply(const ProjArgs &a, hipStream_t st)
{
    constexpr int lds = 4 * 8 * 1024;                 // 4 stages of 8 KB; reused as 4 x 8 KB of epilogue staging
    static bool done[16] = {};
    const int ny = a.H, ngrp = ((a.N + 255) / 256 + 7) / 8;
    dim3 grid(8 * ny * ngrp * a.B), block(256);
    if (hipError_t e = dyn_lds_attr_once(reinterpret_cast<const void *>(proj_apply_kernel), lds, done); e != hipSuccess) return e;
    launch_kernel(proj_apply_kernel, grid, block, lds, st, a);
    return take_launch_status();
}

}  // namespace salad
