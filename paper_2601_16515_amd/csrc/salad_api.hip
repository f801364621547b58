// Host side of libsalad: argument checks, workspace layout, launch order, error text, timing.
// Every check runs before the first HIP call so that bad arguments are reported without a GPU.
#include <hip/hip_runtime.h>

#include <array>
#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <vector>

#include "../../include/salad.h"
#include "salad_internal.h"

using namespace salad;

namespace {

thread_local char g_err[512] = "";

salad_status fail(salad_status st, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return st;
}

salad_status hip_fail(hipError_t e, const char *what)
{
    return fail(SALAD_EHIP, "%s: %s", what, hipGetErrorString(e));
}

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct WsLayout {
    size_t gate_partial, state_partial, Hs, Z, hfrag, s, coef, drop, tile_lists, tile_counts, ol, wfrag, kmeans, topk_mask, g_counts, g_ccnt, g_seg, g_total, g_desc, g_idx, g_slot, g_lse, g_po, rope_tab, total;
    int nparts, P;
};

// tuning knobs (salad_tune): atomics, read once at the top of an entry point and passed down by value, so that a
// concurrent salad_tune on another thread cannot change a call half way through
std::atomic<int> g_state_target_wgs{256};
std::atomic<int> g_topk_variant{0};
std::atomic<int> g_attn_variant{0};

WsLayout ws_layout(int B, int H, int N, int d, int dtype, int state_wgs, bool full_proj = false, int topk = 0, bool rope = false)
{
    WsLayout w{};
    const size_t BH = (size_t)B * H;
    w.nparts = gate_num_parts(N);
    w.P = dtype == SALAD_BF16 ? state_num_chunks((int)BH, N, state_wgs) : 0;
    size_t off = 0;
    w.gate_partial = off; off = align256(off + sizeof(float) * (size_t)B * w.nparts);
    w.state_partial = off; off = align256(off + sizeof(float) * BH * (size_t)w.P * ((size_t)d * d + d));
    w.Hs = off; off = align256(off + sizeof(float) * BH * d * d);
    w.Z = off; off = align256(off + sizeof(float) * BH * d);
    w.hfrag = off; off = align256(off + (dtype == SALAD_BF16 ? sizeof(u16) * BH * d * d : 0));
    w.s = off; off = align256(off + sizeof(float) * B);
    w.coef = off; off = align256(off + sizeof(float) * BH);
    w.drop = off; off = align256(off + sizeof(int32_t) * B);
    {   // union lists per (head, 4-block tile) for the large-tile attention kernel
        const int nb = (N + 63) / 64, ntiles = (nb + 3) / 4;
        const bool need = dtype == SALAD_BF16 && (d == 128 || (d == 64 && !topk)) && (size_t)tile_list_cap(nb) * 4 <= 24 * 1024;
        const size_t nl = topk ? BH : (size_t)H;       // Top-K masks differ between samples
        w.tile_lists = off; off = align256(off + (need ? sizeof(uint32_t) * nl * ntiles * tile_list_cap(nb) : 0));
        w.tile_counts = off; off = align256(off + (need ? sizeof(int32_t) * nl * ntiles : 0));
    }
    // full Level-1 projection: the unscaled linear branch (bf16, [B,H,N,d]) and W_p in fragment order
    w.ol = off; off = align256(off + (full_proj ? sizeof(u16) * BH * (size_t)((N + 31) / 32 * 32) * d : 0));   // whole 32-row tiles
    w.wfrag = off; off = align256(off + (full_proj ? sizeof(u16) * (size_t)H * d * H * d : 0));
    // Top-K mask: mean keys of up to 64 key blocks per head, and the per-query block masks
    w.kmeans = off; off = align256(off + (topk ? sizeof(float) * BH * 64 * (size_t)d : 0));
    w.topk_mask = off; off = align256(off + (topk ? sizeof(uint64_t) * BH * (size_t)N : 0));
    {   // regrouping by key block: one slot per kept (query, key block) pair
        const int kk = topk > 8 ? 8 : topk;
        const size_t pairs = BH * (size_t)N * kk;
        const size_t nch = ((size_t)N + 1023) / 1024;
        w.g_counts = off; off = align256(off + (topk ? sizeof(int32_t) * BH * 64 : 0));
        w.g_ccnt = off; off = align256(off + (topk ? sizeof(int32_t) * BH * nch * 64 : 0));
        w.g_seg = off; off = align256(off + (topk ? sizeof(int32_t) * BH * nch * 64 : 0));
        w.g_total = off; off = align256(off + (topk ? 256 : 0));
        w.g_desc = off; off = align256(off + (topk ? sizeof(uint4) * (size_t)topk_max_tiles((int)BH, N, kk, 64) : 0));
        w.g_idx = off; off = align256(off + (topk ? sizeof(int32_t) * pairs : 0));
        w.g_slot = off; off = align256(off + (topk ? sizeof(int32_t) * pairs : 0));
        w.g_lse = off; off = align256(off + (topk ? sizeof(float) * pairs : 0));
        w.g_po = off; off = align256(off + (topk ? sizeof(u16) * pairs * d : 0));
    }
    w.rope_tab = off; off = align256(off + (rope ? sizeof(uint32_t) * (size_t)N * (d / 2) : 0));
    w.total = off;
    return w;
}

bool shape_ok(int B, int H, int N, int d, int dtype)
{
    if (B < 1 || H < 1 || N < 1) return false;
    if (dtype != SALAD_BF16 && dtype != SALAD_F32) return false;
    if (d != 64 && d != 128) return false;
    if ((long long)B * H * N * d > (1ll << 40)) return false;
    return true;
}

// ---- timing -----------------------------------------------------------------------------------
std::mutex g_tmu;
int g_timing = 0;   // 0 off, 1 every stage, 2 the attention stage only
struct CallEvents { hipEvent_t e[8]; bool has_epilogue, has_linear, attn_only; };   // e[7]: end of the Top-K mask steps
std::vector<CallEvents> g_calls;
std::vector<hipEvent_t> g_free_events;

hipEvent_t get_event()
{
    if (!g_free_events.empty()) {
        hipEvent_t e = g_free_events.back();
        g_free_events.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

// ---- static scratch for the entry point that takes no workspace ----------------------------------
// Device memory that lives in the code object: one copy per GPU the library is loaded on, held until the
// process ends.  The array's name is only a host-side handle; the device address is asked for once per
// device and that pointer is what kernels and copies get.
}  // namespace

static __device__ __align__(256) unsigned char scratch[SALAD_STATIC_SCRATCH_BYTES];

namespace {

std::mutex g_smu;
void *g_scratch_ptr[64] = {};

salad_status static_scratch_ptr(void **out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= 64) return fail(SALAD_ENOTSUP, "static scratch: device ordinal %d outside 0..63", dev);
    std::lock_guard<std::mutex> lk(g_smu);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));     // the current device's copy of the array
        if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(scratch)");
        if (!ptr || ((uintptr_t)ptr & 255)) return fail(SALAD_EHIP, "static scratch: bad device address %p", ptr);
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return SALAD_OK;
}

}  // namespace

extern "C" {

const char *salad_last_error(void) { return g_err; }

int32_t salad_kept_from_sparsity(int32_t nb, double sparsity)
{
    if (nb < 1) return 0;
    double k = std::floor((1.0 - sparsity) * (double)nb + 0.5);
    if (!(k >= 1.0)) k = 1.0;
    if (k > (double)nb) k = (double)nb;
    return (int32_t)k;
}

int64_t salad_block_mask_nnz_mode(int32_t T, int32_t Hh, int32_t W, int32_t block, int32_t H, const int32_t *kept_host,
                                  int32_t window_mode)
{
    if (T < 1 || Hh < 1 || W < 1 || block < 1 || H < 1 || !kept_host) return -1;
    if (window_mode != SALAD_WINDOW_SHIFTED && window_mode != SALAD_WINDOW_TRUNCATED) return -1;
    const int64_t N = (int64_t)T * Hh * W;
    const int64_t nb = (N + block - 1) / block;
    int64_t nnz = 0;
    for (int h = 0; h < H; ++h) {
        const int64_t k = kept_host[h];
        if (k < 1 || k > nb) return -1;
        nnz += nb * k;
        if (window_mode == SALAD_WINDOW_TRUNCATED) {
            const int64_t l = k / 2, r = k - 1 - l;
            nnz -= l * (l + 1) / 2 + r * (r + 1) / 2;
        }
    }
    return nnz;
}

int64_t salad_block_mask_nnz(int32_t T, int32_t Hh, int32_t W, int32_t block, int32_t H, const int32_t *kept_host)
{
    return salad_block_mask_nnz_mode(T, Hh, W, block, H, kept_host, SALAD_WINDOW_SHIFTED);
}

salad_status salad_block_mask_mode(int32_t T, int32_t Hh, int32_t W, int32_t block, int32_t H,
                                   const int32_t *kept_host, int32_t window_mode, int32_t *row_ptr_dev, int32_t *col_idx_dev,
                                   int64_t col_capacity, void *hip_stream)
{
    if (T < 1 || Hh < 1 || W < 1) return fail(SALAD_EINVAL, "salad_block_mask: grid (%d,%d,%d) must be positive", T, Hh, W);
    if (block != 64) return fail(SALAD_ENOTSUP, "salad_block_mask: block %d not supported (64 only)", block);
    if (H < 1 || H > 64) return fail(SALAD_ENOTSUP, "salad_block_mask: H=%d outside 1..64", H);
    if (window_mode != SALAD_WINDOW_SHIFTED && window_mode != SALAD_WINDOW_TRUNCATED)
        return fail(SALAD_EINVAL, "salad_block_mask: window_mode %d is neither SALAD_WINDOW_SHIFTED nor SALAD_WINDOW_TRUNCATED", (int)window_mode);
    if (!kept_host || !row_ptr_dev || !col_idx_dev) return fail(SALAD_EINVAL, "salad_block_mask: null pointer");
    const int64_t N = (int64_t)T * Hh * W;
    if (N > (1ll << 30)) return fail(SALAD_EINVAL, "salad_block_mask: N=%lld too large", (long long)N);
    const int64_t nnz = salad_block_mask_nnz_mode(T, Hh, W, block, H, kept_host, window_mode);
    if (nnz < 0) return fail(SALAD_EINVAL, "salad_block_mask: kept[h] must lie in 1..nb");
    if (nnz > 0x7fffffffll) return fail(SALAD_ENOTSUP, "salad_block_mask: nnz=%lld exceeds int32", (long long)nnz);
    if (col_capacity < nnz) return fail(SALAD_ENOSPC, "salad_block_mask: col_capacity %lld < nnz %lld", (long long)col_capacity, (long long)nnz);
    MaskArgs a{};
    a.nb = (int32_t)((N + block - 1) / block);
    a.H = H;
    a.truncated = window_mode == SALAD_WINDOW_TRUNCATED;
    int64_t base = 0;
    for (int h = 0; h < H; ++h) {
        a.kept[h] = kept_host[h];
        a.base[h] = base;
        base += salad_block_mask_nnz_mode(T, Hh, W, block, 1, kept_host + h, window_mode);
    }
    a.total = base;
    a.row_ptr = row_ptr_dev;
    a.col_idx = col_idx_dev;
    hipError_t e = launch_block_mask(a, (hipStream_t)hip_stream);
    if (e != hipSuccess) return hip_fail(e, "salad_block_mask launch");
    return SALAD_OK;
}

salad_status salad_block_mask(int32_t T, int32_t Hh, int32_t W, int32_t block, int32_t H,
                              const int32_t *kept_host, int32_t *row_ptr_dev, int32_t *col_idx_dev,
                              int64_t col_capacity, void *hip_stream)
{
    return salad_block_mask_mode(T, Hh, W, block, H, kept_host, SALAD_WINDOW_SHIFTED, row_ptr_dev, col_idx_dev, col_capacity, hip_stream);
}

size_t salad_tile_lists_bytes(int32_t H, int32_t nb)
{
    if (H < 1 || H > 64 || nb < 1 || (size_t)tile_list_cap(nb) * 4 > 24 * 1024) return 0;
    const size_t ntiles = ((size_t)nb + 3) / 4;
    return align256(sizeof(uint32_t) * (size_t)H * ntiles * tile_list_cap(nb)) + align256(sizeof(int32_t) * (size_t)H * ntiles);
}

salad_status salad_tile_lists(const int32_t *row_ptr_dev, const int32_t *col_idx_dev, int32_t H, int32_t nb,
                              void *lists_dev, size_t lists_bytes, void *hip_stream)
{
    if (!row_ptr_dev || !col_idx_dev || !lists_dev) return fail(SALAD_EINVAL, "salad_tile_lists: null pointer");
    if (H < 1 || H > 64 || nb < 1) return fail(SALAD_EINVAL, "salad_tile_lists: H=%d nb=%d", (int)H, (int)nb);
    const size_t need = salad_tile_lists_bytes(H, nb);
    if (!need) return fail(SALAD_ENOTSUP, "salad_tile_lists: %d blocks per head are more than the large-tile kernel's list holds", (int)nb);
    if ((uintptr_t)lists_dev & 255) return fail(SALAD_EINVAL, "salad_tile_lists: buffer not 256-byte aligned");
    if (lists_bytes < need) return fail(SALAD_ENOSPC, "salad_tile_lists: buffer %zu < %zu bytes", lists_bytes, need);
    const size_t ntiles = ((size_t)nb + 3) / 4;
    char *b = (char *)lists_dev;
    hipError_t e = launch_tile_lists(row_ptr_dev, col_idx_dev, H, nb, (uint32_t *)b,
                                     (int32_t *)(b + align256(sizeof(uint32_t) * (size_t)H * ntiles * tile_list_cap(nb))), (hipStream_t)hip_stream);
    if (e != hipSuccess) return hip_fail(e, "tile list launch");
    return SALAD_OK;
}

size_t salad_proj_pack_bytes(int32_t H, int32_t d)
{
    if (H < 1 || H > 64 || d != 128) return 0;
    return align256(sizeof(u16) * (size_t)H * d * H * d);
}

salad_status salad_proj_pack(const void *w_proj_dev, int32_t H, int32_t d, void *packed_dev, size_t packed_bytes, void *hip_stream)
{
    if (!w_proj_dev || !packed_dev) return fail(SALAD_EINVAL, "salad_proj_pack: null pointer");
    const size_t need = salad_proj_pack_bytes(H, d);
    if (!need) return fail(SALAD_ENOTSUP, "salad_proj_pack: needs 1 <= H <= 64 and d = 128 (H=%d d=%d)", (int)H, (int)d);
    if ((uintptr_t)packed_dev & 255) return fail(SALAD_EINVAL, "salad_proj_pack: buffer not 256-byte aligned");
    if (packed_bytes < need) return fail(SALAD_ENOSPC, "salad_proj_pack: buffer %zu < %zu bytes", packed_bytes, need);
    hipError_t e = launch_proj_pack((const u16 *)w_proj_dev, H, (u16 *)packed_dev, (hipStream_t)hip_stream);
    if (e != hipSuccess) return hip_fail(e, "projection pack launch");
    return SALAD_OK;
}

size_t salad_fwd_workspace_bytes(const salad_fwd_params *p)
{
    if (!p || !shape_ok(p->B, p->H, p->N, p->d, p->dtype)) return 0;
    return ws_layout(p->B, p->H, p->N, p->d, p->dtype, g_state_target_wgs.load(), p->w_proj != nullptr || p->w_proj_packed != nullptr, p->topk > 0 ? p->topk : 0, p->rope_cos != nullptr).total;
}

salad_status salad_linear_state_fwd(const void *k, const void *v, int32_t B, int32_t H, int32_t N, int32_t d,
                                    int32_t dtype, float *Hs_out, float *Z_out, void *workspace,
                                    size_t workspace_bytes, void *hip_stream)
{
    if (!k || !v || !Hs_out || !Z_out) return fail(SALAD_EINVAL, "salad_linear_state_fwd: null pointer");
    if (!shape_ok(B, H, N, d, dtype)) return fail(SALAD_EINVAL, "salad_linear_state_fwd: unsupported shape B=%d H=%d N=%d d=%d dtype=%d", B, H, N, d, dtype);
    hipStream_t st = (hipStream_t)hip_stream;
    if (dtype == SALAD_F32) {
        hipError_t e = launch_state_f32((const float *)k, (const float *)v, B * H, N, d, Hs_out, Z_out, nullptr, H, st);
        if (e != hipSuccess) return hip_fail(e, "state_f32 launch");
        return SALAD_OK;
    }
    const int state_wgs = g_state_target_wgs.load();
    WsLayout w = ws_layout(B, H, N, d, dtype, state_wgs);
    if (!workspace || ((uintptr_t)workspace & 255)) return fail(SALAD_EINVAL, "salad_linear_state_fwd: workspace null or not 256-byte aligned");
    if (workspace_bytes < w.total) return fail(SALAD_ENOSPC, "salad_linear_state_fwd: workspace %zu < %zu bytes", workspace_bytes, w.total);
    char *ws = (char *)workspace;
    hipError_t e = launch_state_partial_bf16((const u16 *)k, (const u16 *)v, B * H, N, d, (float *)(ws + w.state_partial), nullptr, H, state_wgs, st);
    if (e != hipSuccess) return hip_fail(e, "state_partial launch");
    FinalizeArgs f{};
    f.B = B; f.H = H; f.D = d;
    f.state_partial = (const float *)(ws + w.state_partial); f.P = w.P;
    f.Hs = Hs_out; f.Z = Z_out; f.hfrag = nullptr;
    f.nparts = 0; f.N = N; f.do_gate = 0;
    e = launch_finalize(f, st);
    if (e != hipSuccess) return hip_fail(e, "finalize launch");
    return SALAD_OK;
}

// Shared by salad_gate_fwd and salad_gate_fwd_static: host checks, then gate pass 1 and the fixed-order reduce.
// `scratch` holds the per-workgroup partial sums and, 256-byte aligned behind them, the reduced s.
static size_t gate_scratch_bytes(int B, int N)
{
    return align256(sizeof(float) * (size_t)B * gate_num_parts(N)) + align256(sizeof(float) * (size_t)B);
}

static salad_status gate_check(const char *who, const void *x_t, const float *w_gate, int32_t B, int32_t N, int32_t D,
                               int32_t dtype, const float *s_out)
{
    if (!x_t || !w_gate || !s_out) return fail(SALAD_EINVAL, "%s: null pointer", who);
    if (B < 1 || N < 1 || D < 8 || (D & 7)) return fail(SALAD_EINVAL, "%s: need B,N >= 1 and D a positive multiple of 8 (got %d,%d,%d)", who, B, N, D);
    if (D > 8192) return fail(SALAD_ENOTSUP, "%s: D=%d above 8192", who, D);
    if (dtype != SALAD_BF16 && dtype != SALAD_F32) return fail(SALAD_EINVAL, "%s: dtype %d", who, dtype);
    return SALAD_OK;
}

static salad_status gate_run(const void *x_t, const float *w_gate, float b_gate, int B, int N, int D, int dtype,
                             float *s_out, void *scratch, hipStream_t st)
{
    const int nparts = gate_num_parts(N);
    float *partial = (float *)scratch;
    hipError_t e = launch_gate_partial(x_t, w_gate, b_gate, B, N, D, dtype == SALAD_BF16, partial, nparts, st);
    if (e != hipSuccess) return hip_fail(e, "gate launch");
    FinalizeArgs f{};
    f.B = B; f.H = 1; f.D = 64; f.P = 0;
    f.gate_partial = partial; f.nparts = nparts; f.N = N;
    f.s_out = s_out; f.s_ws = (float *)((char *)scratch + align256(sizeof(float) * (size_t)B * nparts));
    f.coef = nullptr; f.do_gate = 1;
    e = launch_finalize(f, st);
    if (e != hipSuccess) return hip_fail(e, "finalize launch");
    return SALAD_OK;
}

salad_status salad_gate_fwd(const void *x_t, const float *w_gate, float b_gate, int32_t B, int32_t N, int32_t D,
                            int32_t dtype, float *s_out, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (salad_status c = gate_check("salad_gate_fwd", x_t, w_gate, B, N, D, dtype, s_out); c != SALAD_OK) return c;
    const size_t need = gate_scratch_bytes(B, N);
    if (!workspace || ((uintptr_t)workspace & 255)) return fail(SALAD_EINVAL, "salad_gate_fwd: workspace null or not 256-byte aligned");
    if (workspace_bytes < need) return fail(SALAD_ENOSPC, "salad_gate_fwd: workspace %zu < %zu bytes", workspace_bytes, need);
    return gate_run(x_t, w_gate, b_gate, B, N, D, dtype, s_out, workspace, (hipStream_t)hip_stream);
}

salad_status salad_gate_fwd_static(const void *x_t, const float *w_gate, float b_gate, int32_t B, int32_t N, int32_t D,
                                   int32_t dtype, float *s_out, void *hip_stream)
{
    if (salad_status c = gate_check("salad_gate_fwd_static", x_t, w_gate, B, N, D, dtype, s_out); c != SALAD_OK) return c;
    const size_t need = gate_scratch_bytes(B, N);
    if (need > SALAD_STATIC_SCRATCH_BYTES)
        return fail(SALAD_ENOSPC, "salad_gate_fwd_static: B=%d needs %zu bytes of scratch, the static buffer holds %d", B, need, (int)SALAD_STATIC_SCRATCH_BYTES);
    void *ptr = nullptr;
    if (salad_status c = static_scratch_ptr(&ptr); c != SALAD_OK) return c;
    // every partial sum and s[b] the reduce reads is written by this call's own pass 1: nothing has to start at zero
    return gate_run(x_t, w_gate, b_gate, B, N, D, dtype, s_out, ptr, (hipStream_t)hip_stream);
}

salad_status salad_sparse_linear_attn_fwd(const salad_fwd_params *p)
{
    if (!p) return fail(SALAD_EINVAL, "salad_sparse_linear_attn_fwd: null params");
    if (p->B < 1 || p->H < 1 || p->N < 1) return fail(SALAD_EINVAL, "fwd: B=%d H=%d N=%d must be positive", p->B, p->H, p->N);
    if (p->dtype != SALAD_BF16 && p->dtype != SALAD_F32) return fail(SALAD_EINVAL, "fwd: dtype %d", p->dtype);
    if (p->d != 64 && p->d != 128) return fail(SALAD_ENOTSUP, "fwd: d=%d not supported (64 or 128)", p->d);
    if (p->block != 64) return fail(SALAD_ENOTSUP, "fwd: block=%d not supported (64 only)", p->block);
    if (p->H > 64) return fail(SALAD_ENOTSUP, "fwd: H=%d above 64", p->H);
    if (p->T < 1 || p->Hh < 1 || p->W < 1 || (long long)p->T * p->Hh * p->W != p->N)
        return fail(SALAD_EINVAL, "fwd: N=%d is not T*Hh*W = %d*%d*%d", p->N, p->T, p->Hh, p->W);
    if (!shape_ok(p->B, p->H, p->N, p->d, p->dtype)) return fail(SALAD_EINVAL, "fwd: tensor too large");
    if (!p->q || !p->k || !p->v || !p->out) return fail(SALAD_EINVAL, "fwd: q, k, v, out must be non-null");
    if (p->out == p->q || p->out == p->k || p->out == p->v) return fail(SALAD_EINVAL, "fwd: out aliases an input");
    const bool topk = p->topk > 0;
    if (p->topk < 0) return fail(SALAD_EINVAL, "fwd: topk must be >= 0");
    if (!topk && (!p->row_ptr || !p->col_idx)) return fail(SALAD_EINVAL, "fwd: CSR pointers must be non-null");
    int nbk = 0;
    if (topk) {
        if (p->dtype != SALAD_BF16 || p->d != 128) return fail(SALAD_ENOTSUP, "fwd: topk needs dtype bf16 and d = 128");
        if (p->topk > 8) return fail(SALAD_ENOTSUP, "fwd: topk = %d above 8", p->topk);
        if (p->topk_key_block < 64 || p->topk_key_block % 64) return fail(SALAD_EINVAL, "fwd: topk_key_block = %d must be a positive multiple of 64", p->topk_key_block);
        nbk = (p->N + p->topk_key_block - 1) / p->topk_key_block;
        if (nbk > 64) return fail(SALAD_ENOTSUP, "fwd: %d key blocks above 64 (raise topk_key_block)", nbk);
        if (p->head_kind_host && p->T > 1)
            for (int h = 0; h < p->H; ++h)
                if (p->head_kind_host[h] == SALAD_HEAD_TEMPORAL) {
                    // key blocks of a temporal head are runs of its own order; only the regrouped path gathers them
                    if (g_topk_variant.load() != 0) return fail(SALAD_ENOTSUP, "fwd: topk_variant 1 works on the stored token order (head %d is TEMPORAL)", h);
                    if ((unsigned long long)p->N * (unsigned long long)p->T >= (1ull << 32)) return fail(SALAD_ENOTSUP, "fwd: topk: N * T too large for a TEMPORAL head");
                }
        if ((size_t)tile_list_cap((p->N + 63) / 64) * 4 > 24 * 1024 || (unsigned long long)p->N * 256ull >= (1ull << 32))
            return fail(SALAD_ENOTSUP, "fwd: topk: N = %d too long for the large-tile kernel", p->N);
    }
    if (p->tile_lists && ((uintptr_t)p->tile_lists & 255)) return fail(SALAD_EINVAL, "fwd: tile_lists not 256-byte aligned");
    if (p->phi != SALAD_PHI_RELU) return fail(SALAD_ENOTSUP, "fwd: feature map %d not supported (ReLU only)", p->phi);
    if (!(p->eps >= 0.f)) return fail(SALAD_EINVAL, "fwd: eps must be >= 0");
    if (!(p->softmax_scale >= 0.f) || !std::isfinite(p->softmax_scale)) return fail(SALAD_EINVAL, "fwd: softmax_scale must be finite and >= 0");
    if (!std::isfinite(p->lambda)) return fail(SALAD_EINVAL, "fwd: lambda must be finite");
    if (std::isnan(p->drop_threshold)) return fail(SALAD_EINVAL, "fwd: drop_threshold must not be NaN");
    const bool use_linear = p->lambda != 0.f;
    const bool need_gate = use_linear && !p->s_dev;
    const int Dm = p->H * p->d;
    if (need_gate) {
        if (!p->x_t || !p->w_gate) return fail(SALAD_EINVAL, "fwd: lambda != 0 needs s_dev, or x_t and w_gate");
    }
    // with the full projection the sparse kernel always stores O_s alone and the linear branch follows in its own kernels
    // Top-K regrouped by key block (the default Top-K path): the sparse branch is assembled by a merge kernel, so the
    // linear branch follows in its own kernel as well
    const int state_wgs = g_state_target_wgs.load(), attn_variant = g_attn_variant.load();
    const bool topk_regroup = p->topk > 0 && g_topk_variant.load() == 0;
    // rotary linear branch (Sec. 4.1): the rotation lives in the state kernel and in whichever kernel applies the linear
    // branch: the large-tile attention kernel's epilogue, or the separate apply kernel
    const bool rope = p->rope_cos != nullptr || p->rope_sin != nullptr;
    if (rope) {
        if (!p->rope_cos || !p->rope_sin) return fail(SALAD_EINVAL, "fwd: rope_cos and rope_sin must be given together");
        if (p->dtype != SALAD_BF16 || p->d != 128) return fail(SALAD_ENOTSUP, "fwd: the rotary linear branch needs dtype bf16 and d = 128");
    }
    // will the sparse branch run on the large-tile kernel?  (the same conditions as the dispatcher's: see attn_takes_large_tile)
    bool temporal_any = false;
    if (p->head_kind_host && p->T > 1)
        for (int h = 0; h < p->H; ++h) temporal_any |= p->head_kind_host[h] == SALAD_HEAD_TEMPORAL;
    const bool large_tile = p->dtype == SALAD_BF16 && (p->d == 128 || p->d == 64) && attn_variant == 0 &&
                            (size_t)tile_list_cap((p->N + 63) / 64) * 4 <= 24 * 1024 && (unsigned long long)p->N * 256ull < (1ull << 32) &&
                            (!temporal_any || (unsigned long long)p->N * (unsigned long long)p->T < (1ull << 32));
    const bool has_proj = p->w_proj != nullptr || p->w_proj_packed != nullptr;
    const bool rope_fused = rope && large_tile && !topk && !has_proj && !(p->flags & SALAD_FLAG_UNFUSED_EPILOGUE);
    const bool unfused = (p->flags & SALAD_FLAG_UNFUSED_EPILOGUE) != 0 || (has_proj && p->lambda != 0.f) ||
                         (topk_regroup && p->lambda != 0.f) || (rope && !rope_fused && p->lambda != 0.f);
    if (unfused && p->dtype != SALAD_BF16) return fail(SALAD_ENOTSUP, "fwd: unfused epilogue is bf16 only");
    if (p->flags & ~SALAD_FLAG_UNFUSED_EPILOGUE) return fail(SALAD_EINVAL, "fwd: unknown flags 0x%x", p->flags);
    const bool full_proj = has_proj && p->lambda != 0.f;
    if (p->w_proj_packed && ((uintptr_t)p->w_proj_packed & 255)) return fail(SALAD_EINVAL, "fwd: w_proj_packed not 256-byte aligned");
    if (has_proj) {
        if (p->dtype != SALAD_BF16 || p->d != 128) return fail(SALAD_ENOTSUP, "fwd: w_proj needs dtype bf16 and d = 128");
        if (p->head_scale) return fail(SALAD_EINVAL, "fwd: w_proj and head_scale exclude each other");
    }
    const WsLayout w = ws_layout(p->B, p->H, p->N, p->d, p->dtype, state_wgs, has_proj, topk ? p->topk : 0, p->rope_cos != nullptr);
    const bool need_lists = p->dtype == SALAD_BF16 && (p->d == 128 || p->d == 64) && (size_t)tile_list_cap((p->N + 63) / 64) * 4 <= 24 * 1024;
    if (use_linear || need_lists) {
        if (!p->workspace || ((uintptr_t)p->workspace & 255)) return fail(SALAD_EINVAL, "fwd: workspace null or not 256-byte aligned");
        if (p->workspace_bytes < w.total) return fail(SALAD_ENOSPC, "fwd: workspace %zu < %zu bytes", p->workspace_bytes, w.total);
    }
    uint64_t kind_mask = 0;
    if (p->head_kind_host)
        for (int h = 0; h < p->H; ++h) {
            if (p->head_kind_host[h] > 1) return fail(SALAD_EINVAL, "fwd: head_kind[%d]=%d", h, (int)p->head_kind_host[h]);
            if (p->head_kind_host[h] == SALAD_HEAD_TEMPORAL) kind_mask |= 1ull << h;
        }

    hipStream_t st = (hipStream_t)p->hip_stream;
    char *ws = (char *)p->workspace;
    const int BH = p->B * p->H;
    const bool bf16 = p->dtype == SALAD_BF16;
    hipError_t e;

    CallEvents ev{};
    int timing;
    auto give_back = [&]() {                       // an error path returns the events it took to the pool
        std::lock_guard<std::mutex> lk(g_tmu);
        for (auto &x : ev.e)
            if (x) { g_free_events.push_back(x); x = nullptr; }
    };
    {
        std::lock_guard<std::mutex> lk(g_tmu);
        timing = g_timing;
        if (timing)
            for (int i = 0; i < 8; ++i) {
                if (timing == 2 && i != 7 && i != 4) continue;
                ev.e[i] = get_event();
                if (!ev.e[i]) {
                    for (auto &x : ev.e)
                        if (x) { g_free_events.push_back(x); x = nullptr; }
                    return fail(SALAD_EHIP, "fwd: hipEventCreate failed");
                }
            }
    }
    ev.has_linear = use_linear;
    ev.has_epilogue = unfused && use_linear;
    ev.attn_only = timing == 2;
    auto mark = [&](int i) { if (timing == 1 || (timing == 2 && (i == 7 || i == 4))) (void)hipEventRecord(ev.e[i], st); };

    // Post-tuning branch dropping (Sec. 4.3): the dynamic scale has to be known before the state kernel, so the
    // gate is reduced first (finalize in gate-only form) and the later kernels skip the pruned samples.
    const bool dropping = use_linear && p->drop_threshold > 0.f;
    int32_t *drop = dropping ? (int32_t *)(ws + w.drop) : nullptr;
    mark(0);
    if (use_linear) {
        if (need_gate) {
            e = launch_gate_partial(p->x_t, p->w_gate, p->b_gate, p->B, p->N, Dm, bf16, (float *)(ws + w.gate_partial), w.nparts, st);
            if (e != hipSuccess) return give_back(), hip_fail(e, "gate launch");
        }
        FinalizeArgs f{};
        f.B = p->B; f.H = p->H; f.D = p->d;
        f.state_partial = (const float *)(ws + w.state_partial); f.P = w.P;
        f.Hs = (float *)(ws + w.Hs); f.Z = (float *)(ws + w.Z);
        f.hfrag = bf16 ? (u16 *)(ws + w.hfrag) : nullptr;
        f.gate_partial = (const float *)(ws + w.gate_partial); f.nparts = need_gate ? w.nparts : 0; f.N = p->N;
        f.s_dev = p->s_dev; f.lambda = p->lambda; f.head_scale = p->head_scale;
        f.s_out = p->s_out; f.s_ws = (float *)(ws + w.s); f.coef = (float *)(ws + w.coef); f.do_gate = 1;
        f.tau = p->drop_threshold; f.drop = drop; f.dropped_out = dropping ? p->dropped_out : nullptr;
        if (dropping) {
            FinalizeArgs g = f;
            g.P = 0;                                   // gate part only: s, coefficients, drop flags
            e = launch_finalize(g, st);
            if (e != hipSuccess) return give_back(), hip_fail(e, "gate reduce launch");
            f.do_gate = 0;
        }
        mark(1);
        if (bf16)
        {
            if (rope) {     // the two fp32 tables -> one word per angle, read by the state and the apply kernels
                e = launch_rope_pack(p->rope_cos, p->rope_sin, (size_t)p->N * (p->d / 2), (uint32_t *)(ws + w.rope_tab), st);
                if (e != hipSuccess) return give_back(), hip_fail(e, "rotary table launch");
            }
            e = launch_state_partial_bf16((const u16 *)p->k, (const u16 *)p->v, BH, p->N, p->d, (float *)(ws + w.state_partial), drop, p->H, state_wgs, st,
                                          rope ? (const uint32_t *)(ws + w.rope_tab) : nullptr);
        }
        else
            e = launch_state_f32((const float *)p->k, (const float *)p->v, BH, p->N, p->d, (float *)(ws + w.Hs), (float *)(ws + w.Z), drop, p->H, st);
        if (e != hipSuccess) return give_back(), hip_fail(e, "state launch");
        mark(2);
        if (bf16 || f.do_gate) {                       // fp32: the state kernel wrote Hs, Z directly
            e = launch_finalize(f, st);
            if (e != hipSuccess) return give_back(), hip_fail(e, "finalize launch");
        }
    } else {
        mark(1);
        mark(2);
    }
    mark(3);

    AttnArgs a{};
    a.q = p->q; a.k = p->k; a.v = p->v; a.out = p->out;
    a.row_ptr = p->row_ptr; a.col_idx = p->col_idx;
    a.B = p->B; a.H = p->H; a.N = p->N; a.nb = (p->N + 63) / 64; a.T = p->T; a.HW = p->Hh * p->W; a.D = p->d;
    a.kind_mask = kind_mask;
    a.scale = p->softmax_scale > 0.f ? p->softmax_scale : 1.0f / std::sqrt((float)p->d);
    a.use_linear = use_linear;
    a.hfrag = use_linear && bf16 ? (const u16 *)(ws + w.hfrag) : nullptr;
    a.Hs = use_linear ? (const float *)(ws + w.Hs) : nullptr;
    a.Z = use_linear ? (const float *)(ws + w.Z) : nullptr;
    a.coef = use_linear ? (const float *)(ws + w.coef) : nullptr;
    a.eps = p->eps;
    a.o_sparse_dbg = p->o_sparse_dbg; a.o_linear_dbg = unfused ? nullptr : p->o_linear_dbg;
    a.write_sparse_only = unfused;
    a.drop = drop;
    a.variant = attn_variant;
    a.rope_tab = rope_fused && use_linear ? (const uint32_t *)(ws + w.rope_tab) : nullptr;
    if (topk) {
        // App. A.1.2: key-block means -> per-query selection -> per-tile visit lists; the mask never leaves the device
        float *means = (float *)(ws + w.kmeans);
        unsigned long long *mask = (unsigned long long *)(ws + w.topk_mask);
        e = launch_kblock_mean((const u16 *)p->k, BH, p->N, p->topk_key_block, nbk, means, kind_mask, p->H, p->T, p->Hh * p->W, st);
        if (e != hipSuccess) return give_back(), hip_fail(e, "key-block mean launch");
        e = launch_topk_select((const u16 *)p->q, means, BH, p->N, nbk, p->topk, mask, st);
        if (e != hipSuccess) return give_back(), hip_fail(e, "top-k selection launch");
        if (p->topk_mask_out) {
            e = hipMemcpyAsync(p->topk_mask_out, mask, sizeof(uint64_t) * (size_t)BH * p->N, hipMemcpyDeviceToDevice, st);
            if (e != hipSuccess) return give_back(), hip_fail(e, "top-k mask copy");
        }
        a.tile_lists = (const uint32_t *)(ws + w.tile_lists);
        a.tile_counts = (const int32_t *)(ws + w.tile_counts);
        a.list_cap = tile_list_cap(a.nb);
        a.topk_mask = mask;
        if (topk_regroup) {
            const int kk = p->topk < nbk ? p->topk : nbk;
            e = launch_topk_group(mask, BH, p->N, nbk, kk, (int32_t *)(ws + w.g_ccnt), (int32_t *)(ws + w.g_seg),
                                  (uint4 *)(ws + w.g_desc), (int32_t *)(ws + w.g_idx), (int32_t *)(ws + w.g_slot), st);
            if (e != hipSuccess) return give_back(), hip_fail(e, "top-k regrouping launch");
            a.g_desc = (const uint4 *)(ws + w.g_desc);
            a.g_idx = (const int32_t *)(ws + w.g_idx); a.g_po = (u16 *)(ws + w.g_po); a.g_lse = (float *)(ws + w.g_lse);
            a.g_kk = kk; a.g_bpb = p->topk_key_block / 64; a.g_max_tiles = topk_max_tiles(BH, p->N, kk, nbk);
        } else {
            e = launch_topk_tile_lists(mask, BH, p->N, a.nb, p->topk_key_block, nbk, (uint32_t *)(ws + w.tile_lists), (int32_t *)(ws + w.tile_counts), st);
            if (e != hipSuccess) return give_back(), hip_fail(e, "top-k tile list launch");
        }
        mark(7);
    } else if (need_lists) {
        mark(7);
        a.list_cap = tile_list_cap(a.nb);
        if (p->tile_lists) {      // built once for this CSR by salad_tile_lists
            const size_t ntiles = ((size_t)a.nb + 3) / 4;
            a.tile_lists = (const uint32_t *)p->tile_lists;
            a.tile_counts = (const int32_t *)((const char *)p->tile_lists + align256(sizeof(uint32_t) * (size_t)p->H * ntiles * a.list_cap));
        } else {
            a.tile_lists = (const uint32_t *)(ws + w.tile_lists);
            a.tile_counts = (const int32_t *)(ws + w.tile_counts);
            e = launch_tile_lists(p->row_ptr, p->col_idx, p->H, a.nb, (uint32_t *)(ws + w.tile_lists), (int32_t *)(ws + w.tile_counts), st);
            if (e != hipSuccess) return give_back(), hip_fail(e, "tile list launch");
        }
    }
    if (!topk && !need_lists) mark(7);
    a.t_magic = ((uint64_t)p->N * (uint64_t)p->T < (1ull << 32) && p->T > 1) ? (unsigned)((1ull << 32) / (uint64_t)p->T + 1) : 0u;
    e = bf16 ? launch_sparse_attn_bf16(a, st) : launch_sparse_attn_f32(a, st);
    if (e != hipSuccess) return give_back(), hip_fail(e, "sparse attention launch");
    // regrouped Top-K: the partial results of a query are merged by the linear-apply pass itself when that pass is the
    // plain sum (no debug outputs, no projection, no rotation, at most 4 partial results), else by a kernel of their own
    const bool merge_in_apply = a.g_desc && unfused && use_linear && !full_proj && !rope && !p->o_sparse_dbg &&
                                !p->o_linear_dbg && a.g_kk <= 4 && p->d == 128;
    if (a.g_desc && !merge_in_apply) {
        e = launch_topk_merge(a.g_po, a.g_lse, (const int32_t *)(ws + w.g_slot), a.topk_mask, BH, p->N, a.g_kk,
                              (u16 *)p->out, p->o_sparse_dbg, st);
        if (e != hipSuccess) return give_back(), hip_fail(e, "top-k merge launch");
    }
    mark(4);
    if (unfused && use_linear) {
        ApplyArgs ap{};
        ap.q = (const u16 *)p->q; ap.out = (u16 *)p->out; ap.BH = BH; ap.N = p->N; ap.D = p->d;
        ap.hfrag = (const u16 *)(ws + w.hfrag); ap.Z = (const float *)(ws + w.Z); ap.coef = (const float *)(ws + w.coef);
        ap.eps = p->eps; ap.o_linear_dbg = full_proj ? nullptr : p->o_linear_dbg;
        ap.drop = drop; ap.H = p->H;
        ap.emit = full_proj ? (u16 *)(ws + w.ol) : nullptr;
        ap.rope_tab = rope ? (const uint32_t *)(ws + w.rope_tab) : nullptr;
        if (merge_in_apply) {
            ap.m_po = a.g_po; ap.m_lse = a.g_lse; ap.m_slot_of = (const int32_t *)(ws + w.g_slot);
            ap.m_mask = a.topk_mask; ap.m_kk = a.g_kk;
        }
        e = launch_linear_apply_bf16(ap, st);
        if (e != hipSuccess) return give_back(), hip_fail(e, "linear apply launch");
        mark(5);
        if (full_proj) {
            // Alg. 1 "Proj" as one GEMM over the concatenated heads, fused with the residual sum
            if (!p->w_proj_packed) {      // W_p in fragment order: built here unless the caller did it once for the layer
                e = launch_proj_pack((const u16 *)p->w_proj, p->H, (u16 *)(ws + w.wfrag), st);
                if (e != hipSuccess) return give_back(), hip_fail(e, "projection pack launch");
            }
            ProjArgs pa{};
            pa.ol = (const u16 *)(ws + w.ol); pa.out = (u16 *)p->out;
            pa.wfrag = p->w_proj_packed ? (const u16 *)p->w_proj_packed : (const u16 *)(ws + w.wfrag);
            pa.coef = (const float *)(ws + w.coef); pa.drop = drop; pa.B = p->B; pa.H = p->H; pa.N = p->N;
            e = launch_proj_apply(pa, st);
            if (e != hipSuccess) return give_back(), hip_fail(e, "projection launch");
        }
    } else {
        mark(5);
    }
    mark(6);
    if (timing) {
        std::lock_guard<std::mutex> lk(g_tmu);
        g_calls.push_back(ev);
    }
    return SALAD_OK;
}

salad_status salad_timing_enable(int32_t on)
{
    std::lock_guard<std::mutex> lk(g_tmu);
    if (on < 0 || on > 2) return fail(SALAD_EINVAL, "salad_timing_enable: mode %d", (int)on);
    g_timing = on;
    return SALAD_OK;
}

salad_status salad_timing_read(salad_kernel_times *out, int32_t reset)
{
    if (!out) return fail(SALAD_EINVAL, "salad_timing_read: null output");
    std::lock_guard<std::mutex> lk(g_tmu);
    std::memset(out, 0, sizeof(*out));
    for (auto &c : g_calls) {
        if (c.attn_only) {
            hipError_t e = hipEventSynchronize(c.e[4]);
            if (e != hipSuccess) return hip_fail(e, "hipEventSynchronize");
            float ms_a = 0.f;
            e = hipEventElapsedTime(&ms_a, c.e[7], c.e[4]);
            if (e != hipSuccess) return hip_fail(e, "hipEventElapsedTime");
            out->attn_ms += ms_a;
            out->calls += 1;
            continue;
        }
        hipError_t e = hipEventSynchronize(c.e[6]);
        if (e != hipSuccess) return hip_fail(e, "hipEventSynchronize");
        float ms[6] = {0, 0, 0, 0, 0, 0};
        for (int i = 0; i < 6; ++i) {
            e = hipEventElapsedTime(&ms[i], c.e[i], c.e[i + 1]);
            if (e != hipSuccess) return hip_fail(e, "hipEventElapsedTime");
        }
        float topk_ms = 0.f;
        e = hipEventElapsedTime(&topk_ms, c.e[3], c.e[7]);
        if (e != hipSuccess) return hip_fail(e, "hipEventElapsedTime");
        ms[3] -= topk_ms;
        out->topk_ms += topk_ms;
        out->gate_ms += ms[0];
        out->state_ms += ms[1];
        out->finalize_ms += ms[2];
        out->attn_ms += ms[3];
        out->epilogue_ms += ms[4];
        out->proj_ms += ms[5];
        out->calls += 1;
    }
    if (reset) {
        for (auto &c : g_calls)
            for (auto &x : c.e)
                if (x) g_free_events.push_back(x);
        g_calls.clear();
    }
    return SALAD_OK;
}

/* Launch-shape knobs for experiments.  Every accepted key is declared in include/salad.h and range-checked here; the
 * values are atomics that an entry point reads once per call. */
salad_status salad_tune(const char *key, int32_t value)
{
    if (!key) return fail(SALAD_EINVAL, "salad_tune: null key");
    if (!std::strcmp(key, "state_wgs")) {
        if (value < 1 || value > 65536) return fail(SALAD_EINVAL, "salad_tune: state_wgs %d outside 1..65536", (int)value);
        g_state_target_wgs.store(value);
        return SALAD_OK;
    }
    if (!std::strcmp(key, "attn_variant")) {   // 0: automatic, 1: 128-query tiles, 2: first-generation kernel
        if (value < 0 || value > 2) return fail(SALAD_EINVAL, "salad_tune: attn_variant %d outside 0..2", (int)value);
        g_attn_variant.store(value);
        return SALAD_OK;
    }
    if (!std::strcmp(key, "topk_variant")) {   // 0: regrouped by key block (default), 1: token mask on query tiles
        if (value < 0 || value > 1) return fail(SALAD_EINVAL, "salad_tune: topk_variant %d outside 0..1", (int)value);
        g_topk_variant.store(value);
        return SALAD_OK;
    }
    return fail(SALAD_EINVAL, "salad_tune: unknown key %s", key);
}

}  // extern "C"
