// Internal declarations shared by the host API file and the kernel files of libsalad.
// Not installed; the public interface is include/salad.h.
#pragma once
#include <hip/hip_runtime.h>
#include <tuple>
#include <type_traits>
#include <utility>
#include <stdint.h>

namespace salad {

typedef unsigned short u16;

// ---- block mask -------------------------------------------------------------------------------
struct MaskArgs {
    int32_t nb, H;
    int32_t truncated;  // window cut at the sequence ends instead of shifted inward
    int32_t kept[64];
    int64_t base[64];   // first col_idx entry of head h
    int64_t total;      // number of col_idx entries
    int32_t *row_ptr, *col_idx;
};
hipError_t launch_block_mask(const MaskArgs &a, hipStream_t st);

// ---- gate (Alg. 1 Level 2) ----------------------------------------------------------------------
// Pass 1: per-workgroup partial sums of sigmoid(x.w + b) -> partial[b * nparts + part].
hipError_t launch_gate_partial(const void *x_t, const float *w, float bias, int B, int N, int D,
                               int is_bf16, float *partial, int nparts, hipStream_t st);
int gate_num_parts(int N);

// ---- linear state (Eq. (3) sums) ----------------------------------------------------------------
// bf16: partial states over token chunks, MFMA.  partial[(bh*P + c)][D*D + D] fp32.
// target_wgs: workgroups the launch aims for (the caller reads the tuning knob once per call)
int state_tiles_per_chunk(int BH, int N, int target_wgs);
int state_num_chunks(int BH, int N, int target_wgs);
// drop (may be null): int32 [B], workgroups of a sample with drop[b] != 0 return at once (H heads per sample)
// rope_tab (d = 128 only): [N, d/2] words (fp16 cos | fp16 sin << 16) of the rotary linear branch, or null
hipError_t launch_state_partial_bf16(const u16 *k, const u16 *v, int BH, int N, int D,
                                     float *partial, const int32_t *drop, int H, int target_wgs, hipStream_t st,
                                     const uint32_t *rope_tab = nullptr);
hipError_t launch_rope_pack(const float *rope_cos, const float *rope_sin, size_t n, uint32_t *tab, hipStream_t st);
// fp32: direct evaluation, one thread per state element (small shapes).
hipError_t launch_state_f32(const float *k, const float *v, int BH, int N, int D,
                            float *Hs, float *Z, const int32_t *drop, int H, hipStream_t st);

// ---- finalize: reduce partials, dynamic scale, coefficients ---------------------------------------
struct FinalizeArgs {
    int B, H, D;
    // state (bf16 path only; P == 0 skips the state part)
    const float *state_partial; int P;
    float *Hs, *Z;       // [BH, D, D], [BH, D] fp32
    u16 *hfrag;          // [BH][D*D] Hs rounded to bf16, in MFMA A-operand fragment order of Hs^T (may be null)
    // gate
    const float *gate_partial; int nparts; int N;   // nparts == 0: take s from s_dev
    const float *s_dev;
    float lambda; const float *head_scale;
    float *s_out;        // [B] (may be null)
    float *s_ws;         // [B]
    float *coef;         // [BH] lambda * a_h * s_b (may be null)
    int do_gate;         // 0: state part only
    // branch dropping (Sec. 4.3): the gate part writes drop[b] = s_b < tau (and a zero coefficient), the
    // state part skips samples with drop[b] != 0.  drop == nullptr: no dropping.
    float tau;
    int32_t *drop;       // [B] in the workspace
    int32_t *dropped_out;// [B] caller's copy (may be null)
};
hipError_t launch_finalize(const FinalizeArgs &a, hipStream_t st);

// ---- sparse attention + fused linear apply / scale / sum -------------------------------------------
struct AttnArgs {
    const void *q, *k, *v;
    void *out;
    const int32_t *row_ptr, *col_idx;
    int B, H, N, nb, T, HW, D;
    unsigned long long kind_mask;   // bit h set: head h uses the temporal token order
    float scale;                    // softmax scale (natural-log domain)
    int use_linear;                 // 0: out = O_s
    const u16 *hfrag;               // bf16 path
    const float *Hs;                // fp32 path
    const float *Z;
    const float *coef;              // [BH]
    float eps;
    float *o_sparse_dbg, *o_linear_dbg;
    int write_sparse_only;          // bf16: store O_s (rounded) to out and skip the linear part
    unsigned t_magic;               // floor(2^32 / T) + 1 when N * T < 2^32, else 0
    // per (head, 4-query-block tile): ascending union of the 4 CSR rows, entry = block | keep-mask << 24
    const uint32_t *tile_lists;     // [H * ntiles4][list_cap]
    const int32_t *tile_counts;     // [H * ntiles4]
    int list_cap;
    const int32_t *drop;            // [B] or null: samples whose linear branch is pruned (out = O_s)
    // Top-K token-level mask (App. A.1.2), large-tile kernel only: bit J of topk_mask[(b*H + h)*N + n] = query n
    // keeps key block J; tile_lists / tile_counts are then per (b, h, tile) with entries
    // block | J << 16 | wave mask << 24.  null: block rows (CSR) as above.
    const unsigned long long *topk_mask;
    // Top-K regrouped by key block, large-tile kernel only (g_desc != null): query tile L < g_max_tiles is the run of
    // g_desc[L].w queries (none: the workgroup returns; g_desc[L] = sample-head, key block, first slot, queries) whose stored rows are
    // g_idx[bh * N * g_kk + slot], attending to the 64-token blocks of that one key block (g_bpb per key block);
    // results go to g_po [slot][128] (normalised, bf16) and g_lse [slot] (fp32, log2 domain), not to out.
    const uint4 *g_desc;
    const int32_t *g_idx;
    u16 *g_po; float *g_lse;
    int g_kk, g_bpb, g_max_tiles;
    const uint32_t *rope_tab;       // large-tile kernel, fused epilogue only: [N, 64] angle words (fp16 cos | fp16 sin << 16) of the
                                    // rotary linear branch (the state fragments then hold the rotated state), or null
    int variant;                    // 0: automatic choice of the d = 128 kernel; 1: 128-query tiles; 2: first-generation kernel
};
hipError_t launch_sparse_attn_bf16(const AttnArgs &a, hipStream_t st);
// whether launch_sparse_attn_bf16 will take the large-tile kernel for these arguments (the only one whose fused epilogue
// knows the rotary linear branch)
bool attn_takes_large_tile(const AttnArgs &a);
// union lists of the CSR rows of every 4-query-block tile (input of the large-tile attention kernel)
int tile_list_cap(int nb);
hipError_t launch_tile_lists(const int32_t *row_ptr, const int32_t *col_idx, int H, int nb, uint32_t *lists,
                             int32_t *counts, hipStream_t st);
hipError_t launch_sparse_attn_f32(const AttnArgs &a, hipStream_t st);
hipError_t launch_sparse_attn_v2(const AttnArgs &a, hipStream_t st);   // d = 128 only
hipError_t launch_sparse_attn_v5(const AttnArgs &a, hipStream_t st);   // d = 128 only

// ---- Top-K dynamic mask (App. A.1.2), d = 128 bf16 ---------------------------------------------------------
// means [BH][nbk][128] fp32: mean key of each run of key_block positions of the head's own order (bit h of kind_mask:
// temporal; sequential fp32 sum in position order / count)
hipError_t launch_kblock_mean(const u16 *k, int BH, int N, int key_block, int nbk, float *means, unsigned long long kind_mask,
                              int H, int T, int HW, hipStream_t st);
// mask [BH][N]: bit J set for the topk key blocks with the largest q.mean (fp32, channels in ascending order,
// fused multiply-add; ties to the lower index)
hipError_t launch_topk_select(const u16 *q, const float *means, int BH, int N, int nbk, int topk,
                              unsigned long long *mask, hipStream_t st);
// per (b, h, tile of 256 queries): the 64-token blocks of every key block some query of the tile keeps
// regrouping by key block: counts, slot plan and query-tile descriptors, gathered query rows, slot of every pair
int topk_max_tiles(int BH, int N, int kk, int nbk);
// (ccnt, cbase: [BH][ceil(N/1024)][64] per-chunk counts and first slots; desc: [topk_max_tiles])
hipError_t launch_topk_group(const unsigned long long *mask, int BH, int N, int nbk, int kk, int32_t *ccnt,
                             int32_t *cbase, uint4 *desc, int32_t *gidx, int32_t *slot_of, hipStream_t st);
// out = the kk partial results of every query combined by their log-sum-exp weights (bf16; o_dbg fp32 optional)
hipError_t launch_topk_merge(const u16 *po, const float *lse, const int32_t *slot_of, const unsigned long long *mask,
                             int BH, int N, int kk, u16 *out, float *o_dbg, hipStream_t st);
hipError_t launch_topk_tile_lists(const unsigned long long *mask, int BH, int N, int nb, int key_block, int nbk,
                                  uint32_t *lists, int32_t *counts, hipStream_t st);

// ---- unfused linear apply + scale + sum (bf16): out = out + coef * phi(Q) Hs / (phi(Q).Z + eps) ----
struct ApplyArgs {
    const u16 *q; u16 *out;     // out holds O_s on entry
    int BH, N, D;
    const u16 *hfrag; const float *Z; const float *coef; float eps;
    float *o_linear_dbg;
    const int32_t *drop; int H;     // [B] or null: pruned samples are left as they are (out = O_s)
    const uint32_t *rope_tab;       // d = 128: [N, 64] words (fp16 cos | fp16 sin << 16) of the rotary linear branch, or null
    u16 *emit;                      // d = 128: non-null -> write the unscaled O_l (bf16, [B][ceil(N/32)][H] fragment blocks) here, leave out alone
    // d = 128, non-null m_po: out does not hold O_s yet; O_s of a row is the merge of its m_kk <= 4 partial results
    // (regrouped Top-K path, App. A.1.2), taken here in fp32 instead of by topk_merge_kernel.  Arguments as there.
    const u16 *m_po; const float *m_lse; const int32_t *m_slot_of; const unsigned long long *m_mask; int m_kk;
};
hipError_t launch_linear_apply_bf16(const ApplyArgs &a, hipStream_t st);

// ---- full Level-1 projection (Alg. 1 "Proj"): out = out + coef[b] * (O_l W_p), d = 128, bf16 ------------------
struct ProjArgs {
    const u16 *ol;                  // unscaled linear branch (bf16) as [B][ceil(N/32)][H] blocks of 32 rows in B-operand fragment order
    u16 *out;                       // [B,H,N,128], holds O_s on entry
    const u16 *wfrag;               // [H_in][H_out][128*128] W_p blocks in MFMA A-operand fragment order
    const float *coef;              // [B*H]; entry b*H is lambda * s_b (0 for a pruned sample)
    const int32_t *drop;            // [B] or null
    int B, H, N;
};
hipError_t launch_proj_pack(const u16 *w_proj, int H, u16 *wfrag, hipStream_t st);
hipError_t launch_proj_apply(const ProjArgs &a, hipStream_t st);

// Kernel launch whose status is this launch's own.  The <<<>>> form reports a failed launch only through the thread's
// "last error" slot, which an earlier, unrelated call may have set; hipLaunchKernel returns the launch's status.
// A launcher issues its launches through launch_kernel and returns take_launch_status(): the first failure among them.
inline hipError_t &launch_status_slot()
{
    static thread_local hipError_t e = hipSuccess;
    return e;
}
inline hipError_t take_launch_status()
{
    const hipError_t e = launch_status_slot();
    launch_status_slot() = hipSuccess;
    return e;
}
template <class Tuple, size_t... I>
inline hipError_t launch_with(const void *kernel, dim3 grid, dim3 block, size_t lds, hipStream_t st, Tuple &vals, std::index_sequence<I...>)
{
    void *ptrs[] = {static_cast<void *>(&std::get<I>(vals))...};
    return hipLaunchKernel(kernel, grid, block, ptrs, lds, st);
}
template <class... P, class... A>
inline void launch_kernel(void (*kernel)(P...), dim3 grid, dim3 block, size_t lds, hipStream_t st, A &&...args)
{
    static_assert(sizeof...(P) == sizeof...(A), "every kernel parameter needs its argument");
    std::tuple<std::remove_cv_t<P>...> vals(static_cast<P>(std::forward<A>(args))...);   // copies in the parameter types
    const hipError_t e = launch_with(reinterpret_cast<const void *>(kernel), grid, block, lds, st, vals, std::index_sequence_for<P...>{});
    if (e != hipSuccess && launch_status_slot() == hipSuccess) launch_status_slot() = e;
}

// Raises a kernel's dynamic-LDS limit once per device (`done` is the caller's per-kernel flag array).
inline hipError_t dyn_lds_attr_once(const void *kernel, int bytes, bool (&done)[16])
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 16) return hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (done[dev]) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) done[dev] = true;
    return e;
}


}  // namespace salad
