// C-ABI entry points of libsvdp (see include/svdp.h): host-side validation,
// workspace carving and kernel launches.  No allocation, no synchronisation.
#include "../../include/svdp.h"

#include <hip/hip_runtime.h>

#include "svdp_kernels.h"
#include "svdp_fused.h"
#include "svdp_rows_mfma.h"
#include "svdp_rows_seq.h"
#include "svdp_calib.h"
#include "svdp_calib_stats.h"

#include <atomic>
#include <mutex>
#include <type_traits>
#include <vector>

namespace {

using namespace svdp;

constexpr int XP_MAX_BLOCKS = 128;    // stage-1 row slabs of P (d <= 16384)
constexpr int ROWS_BLOCKS = 256;      // k_rows blocks: one chunk of the row list and one partial y each (128 to
                                      // 512 were measured; 256 is best for every batch size)
constexpr size_t ALIGN = 256;

inline size_t align_up(size_t v) { return (v + ALIGN - 1) / ALIGN * ALIGN; }
inline int nb_of(int B) { return B <= 1 ? 1 : B <= 2 ? 2 : B <= 4 ? 4 : 8; }
inline int vec_of(int dt) { return dt == SVDP_F32 ? 4 : 8; }
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

svdp_status check_shape(int d, int D, int r, int dt)
{
    if (dt != SVDP_F32 && dt != SVDP_BF16) return SVDP_ERR_UNSUPPORTED;
    if (d <= 0 || D <= 0 || r <= 0) return SVDP_ERR_INVALID_ARG;
    const int e = vec_of(dt);
    if (D % 64 != 0 || d % e != 0 || r % e != 0) return SVDP_ERR_UNSUPPORTED;
    if (r > 2048 || d > 16384) return SVDP_ERR_UNSUPPORTED;
    return SVDP_OK;
}

svdp_status check_layer(const svdp_layer *L, bool need_pred, bool need_ffn)
{
    if (L == nullptr) return SVDP_ERR_INVALID_ARG;
    const svdp_status st = check_shape(L->d, L->D, L->r, L->wdtype);
    if (st != SVDP_OK) return st;
    if (need_pred && (!L->P || !L->Q || !L->b || !aligned16(L->P) || !aligned16(L->Q) ||
                      (reinterpret_cast<uintptr_t>(L->b) & 3u)))
        return SVDP_ERR_INVALID_ARG;
    if (need_ffn && (!L->W_gate || !L->W_up || !L->W_downT || !aligned16(L->W_gate) ||
                     !aligned16(L->W_up) || !aligned16(L->W_downT)))
        return SVDP_ERR_INVALID_ARG;
    if (L->flags & ~(uint32_t)(SVDP_FLAG_DRELU | SVDP_FLAG_REVALIDATE)) return SVDP_ERR_INVALID_ARG;
    return SVDP_OK;
}

// Workspace layout (all offsets 256-byte aligned):
//   tpart [XP_MAX_BLOCKS + 1][NB][r] f32 | mask [D/64] u64 | nnz i32 | ypart [ROWS_BLOCKS][NB][d] f32
struct Workspace {
    float *tpart;
    uint64_t *mask;
    int32_t *nnz;
    float *ypart;
    size_t bytes;
};

Workspace carve(void *base, int d, int D, int r, int NB)
{
    Workspace w;
    char *p = static_cast<char *>(base);
    size_t off = 0;
    w.tpart = reinterpret_cast<float *>(p + off);
    off += align_up((size_t)(XP_MAX_BLOCKS + 1) * NB * r * 4);     // partials, then the finished t
    w.mask = reinterpret_cast<uint64_t *>(p + off);
    off += align_up((size_t)D / 64 * 8);
    w.nnz = reinterpret_cast<int32_t *>(p + off);
    off += ALIGN;
    w.ypart = reinterpret_cast<float *>(p + off);
    off += align_up((size_t)ROWS_BLOCKS * NB * d * 4);
    w.bytes = off;
    return w;
}

svdp_status check_ws(const svdp_layer *L, int B, void *ws, size_t ws_bytes, Workspace *out)
{
    if (ws == nullptr || (reinterpret_cast<uintptr_t>(ws) & (ALIGN - 1))) return SVDP_ERR_WORKSPACE;
    *out = carve(ws, L->d, L->D, L->r, nb_of(B));
    if (ws_bytes < out->bytes) return SVDP_ERR_WORKSPACE;
    return SVDP_OK;
}

// Dynamic LDS above the default limit has to be enabled per kernel once.
template <typename K>
hipError_t allow_lds(K kernel, size_t bytes, int *granted)
{
    if ((int)bytes <= *granted) return hipSuccess;
    if (bytes > 160 * 1024) return hipErrorInvalidValue;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess) *granted = (int)bytes;
    return e;
}

inline svdp_status hip_status(hipError_t e)
{
    if (e == hipSuccess) e = hipGetLastError();
    else (void)hipGetLastError();
    return e == hipSuccess ? SVDP_OK : SVDP_ERR_HIP;
}

// ---- control blocks for launches whose blocks hand results to each other ----
// Control blocks live in static device memory (zero at load, zero again after every
// launch); one slot per workspace address seen by this process.
__device__ __align__(256) uint32_t g_step_ctrl[CTRL_SLOTS * CTRL_WORDS];

std::atomic<int> g_fused_mode{0};            // svdp_step_mode
std::atomic<int> g_spin_limit{400000};       // polls before a stage wait gives up
std::atomic<int> g_engine{0};           // svdp_engine
std::mutex g_slot_mutex;
std::vector<const void *> g_slots;
uint32_t *g_ctrl_base = nullptr;
int g_num_cus = 0;

bool fused_setup()
{
    if (g_ctrl_base != nullptr) return true;
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_step_ctrl)) != hipSuccess || p == nullptr) {
        (void)hipGetLastError();
        return false;
    }
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) {
        (void)hipGetLastError();
        return false;
    }
    g_num_cus = cus;
    g_ctrl_base = static_cast<uint32_t *>(p);
    return true;
}

// control block of a workspace, or nullptr when none is free
uint32_t *ctrl_for(const void *ws)
{
    std::lock_guard<std::mutex> lock(g_slot_mutex);
    if (!fused_setup()) return nullptr;
    for (size_t i = 0; i < g_slots.size(); ++i)
        if (g_slots[i] == ws) return g_ctrl_base + i * CTRL_WORDS;
    if (g_slots.size() >= (size_t)CTRL_SLOTS) return nullptr;
    g_slots.push_back(ws);
    return g_ctrl_base + (g_slots.size() - 1) * CTRL_WORDS;
}

// ---- launch helpers, one per kernel, templated on storage type and batch capacity ----

// The stacked benchmark's glue folded into the first kernel of a step (svdp_ffn_step_glued).
struct GlueArgs {
    const float *y_prev;
    const float *shift;
    float eps;
    void *x_out;
};

template <typename W, int NB>
svdp_status launch_xP(const svdp_layer *L, const void *x, int B, float *tpart, int *nt_out, hipStream_t st,
                      const GlueArgs *glue = nullptr)
{
    constexpr int VEC = Elem<W>::VEC;
    const int d = L->d, r = L->r;
    const int nt = (d + XP_ROWS - 1) / XP_ROWS;           // <= XP_MAX_BLOCKS since d <= 16384
    const int ncs = (r + XP_COLS - 1) / XP_COLS;
    const size_t outs = (size_t)NB * XP_COLS;
    const size_t parts = XP_THREADS / outs >= 1 ? XP_THREADS / outs : 1;
    const size_t nsub = XP_THREADS / (XP_COLS / VEC);
    const size_t lds = ((size_t)NB * XP_ROWS + nsub * (outs + 1) + parts * outs) * 4;
    static int granted = 64 * 1024, granted_g = 64 * 1024;
    if (glue != nullptr) {
        if (allow_lds(k_xP<W, NB, true>, lds, &granted_g) != hipSuccess) return SVDP_ERR_UNSUPPORTED;
        hipLaunchKernelGGL((k_xP<W, NB, true>), dim3(nt, ncs), dim3(XP_THREADS), lds, st, static_cast<const W *>(L->P),
                           static_cast<const W *>(x), B, d, r, tpart, glue->y_prev, glue->shift, glue->eps,
                           static_cast<W *>(glue->x_out));
    } else {
        if (allow_lds(k_xP<W, NB, false>, lds, &granted) != hipSuccess) return SVDP_ERR_UNSUPPORTED;
        hipLaunchKernelGGL((k_xP<W, NB, false>), dim3(nt, ncs), dim3(XP_THREADS), lds, st,
                           static_cast<const W *>(L->P), static_cast<const W *>(x), B, d, r, tpart, nullptr, nullptr,
                           0.f, nullptr);
    }
    *nt_out = nt;
    return hip_status(hipSuccess);
}

template <typename W, int NB, int LPR_LOG2, int THREADS>
svdp_status launch_scores_thr(const svdp_layer *L, const float *tpart, int nt, int B, float *s_out,
                              uint64_t *mask_out, hipStream_t st)
{
    const size_t tsp = (size_t)NB * L->r > (size_t)THREADS * 4 ? (size_t)NB * L->r : (size_t)THREADS * 4;
    const size_t lds = ((size_t)NB * L->r + (size_t)NB * SC_SLAB + tsp) * 4;
    static int granted = 64 * 1024;
    if (allow_lds(k_scores<W, NB, LPR_LOG2, THREADS>, lds, &granted) != hipSuccess) return SVDP_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((k_scores<W, NB, LPR_LOG2, THREADS>), dim3(L->D / SC_SLAB), dim3(THREADS), lds, st,
                       static_cast<const W *>(L->Q), L->b, tpart, nt, B, L->D, L->r, s_out, mask_out);
    return hip_status(hipSuccess);
}

template <typename W, int NB, int LPR_LOG2>
svdp_status launch_scores_lpr(const svdp_layer *L, const float *tpart, int nt, int B, float *s_out,
                              uint64_t *mask_out, hipStream_t st)
{
    // block size: 512 threads for one or two tokens (short critical path), 256 for larger batches
    // (fewer wavefronts repeating the per-wave overhead); measured on the 7B and Mistral shapes
    if (NB <= 2) return launch_scores_thr<W, NB, LPR_LOG2, 512>(L, tpart, nt, B, s_out, mask_out, st);
    return launch_scores_thr<W, NB, LPR_LOG2, 256>(L, tpart, nt, B, s_out, mask_out, st);
}

// Whether the score kernel on the matrix cores takes this layer and batch capacity.
template <typename W, int NB>
bool scores_on_matrix(const svdp_layer *L)
{
    if (!std::is_same<W, bf16>::value) return false;
    const int engine = g_engine.load();
    const bool want = engine == SVDP_ENGINE_MATRIX || (engine == SVDP_ENGINE_AUTO && NB >= 4);
    return want && L->r % 32 == 0 && L->r <= 32 * SCM_KB;
}

template <typename W, int NB>
svdp_status launch_scores(const svdp_layer *L, const float *tpart, int nt, int B, float *s_out,
                          uint64_t *mask_out, hipStream_t st)
{
    if constexpr (std::is_same<W, bf16>::value) {
        if (scores_on_matrix<W, NB>(L)) {
            const size_t lds = (size_t)3 * NB * L->r * 2;
            hipLaunchKernelGGL((k_scores_mfma<NB>), dim3(L->D / SC_SLAB), dim3(SCM_THREADS), lds, st,
                               static_cast<const bf16 *>(L->Q), L->b, tpart, nt, B, L->D, L->r, s_out, mask_out);
            return hip_status(hipSuccess);
        }
    }
    const int cg = L->r / Elem<W>::VEC;       // 16-byte column groups per row of Q
    if (cg <= 8) return launch_scores_lpr<W, NB, 3>(L, tpart, nt, B, s_out, mask_out, st);
    if (cg <= 16) return launch_scores_lpr<W, NB, 4>(L, tpart, nt, B, s_out, mask_out, st);
    if (cg <= 32) return launch_scores_lpr<W, NB, 5>(L, tpart, nt, B, s_out, mask_out, st);
    return launch_scores_lpr<W, NB, 6>(L, tpart, nt, B, s_out, mask_out, st);
}

// The row kernel on the matrix cores, if this layer and batch qualify: launches it and
// returns true (status in *out); false when the vector kernel has to do the work.
template <typename W, int NB, int MODE>
bool launch_rows_matrix(const svdp_layer *L, const void *x, int B, const uint64_t *mask, const int32_t *idx_in,
                        const int32_t *nnz_in, int32_t *idx_out, int32_t *nnz_out, const Workspace &w, hipStream_t st,
                        svdp_status *out)
{
    if constexpr (!std::is_same<W, bf16>::value) {
        return false;
    } else {
        const int engine = g_engine.load();
        // measured on the Mistral shape: ahead of the vector kernel only at the largest batch capacity
        if (engine == SVDP_ENGINE_VECTOR || (engine == SVDP_ENGINE_AUTO && NB < 8)) return false;
        if (L->d % 512 != 0 || (L->flags & SVDP_FLAG_REVALIDATE) != 0) return false;
        const int d = L->d, D = L->D, grid = ROWS_BLOCKS;
        const int max_chunk = ((D + grid - 1) / grid + MF_ROWS - 1) / MF_ROWS * MF_ROWS;
        const size_t lds = (size_t)NB * d * 2 +
                           ((size_t)ROWS_WAVES * max_chunk * 2 * NB + (size_t)max_chunk * MF_TOK + max_chunk) * 4;
        static int granted = 64 * 1024;
        if (lds > 160 * 1024 || allow_lds(k_rows_mfma<NB, MODE>, lds, &granted) != hipSuccess) return false;
        hipLaunchKernelGGL((k_rows_mfma<NB, MODE>), dim3(grid), dim3(ROWS_THREADS), lds, st,
                           static_cast<const bf16 *>(L->W_gate), static_cast<const bf16 *>(L->W_up),
                           static_cast<const bf16 *>(L->W_downT), static_cast<const bf16 *>(x), B, d, D, mask, idx_in,
                           nnz_in, idx_out, nnz_out, w.nnz, max_chunk, L->flags, w.ypart);
        *out = hip_status(hipSuccess);
        return true;
    }
}

// The row kernel of the sequential pipeline (SVDP_FLAG_REVALIDATE), launched in place of k_rows.
template <typename W, int NB, int MODE>
svdp_status launch_rows_seq(const svdp_layer *L, const void *x, int B, const uint64_t *mask, const int32_t *idx_in,
                            const int32_t *nnz_in, int32_t *idx_out, int32_t *nnz_out, const Workspace &w,
                            hipStream_t st)
{
    const int d = L->d, D = L->D, grid = ROWS_BLOCKS;
    const int max_chunk = ((D + grid - 1) / grid + ROWS_UB - 1) / ROWS_UB * ROWS_UB;
    const size_t lds = (size_t)NB * d * sizeof(W) + ((size_t)2 * NB * max_chunk + (size_t)3 * max_chunk) * 4;
    static int granted = 64 * 1024;
    if (allow_lds(k_rows_seq<W, NB, MODE>, lds, &granted) != hipSuccess) return SVDP_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((k_rows_seq<W, NB, MODE>), dim3(grid), dim3(ROWS_THREADS), lds, st,
                       static_cast<const W *>(L->W_gate), static_cast<const W *>(L->W_up),
                       static_cast<const W *>(L->W_downT), static_cast<const W *>(x), B, d, D, mask, idx_in, nnz_in,
                       idx_out, nnz_out, w.nnz, max_chunk, L->flags, w.ypart);
    return hip_status(hipSuccess);
}

template <typename W, int NB, int MODE>
svdp_status launch_rows(const svdp_layer *L, const void *x, int B, const uint64_t *mask, const int32_t *idx_in,
                        const int32_t *nnz_in, int32_t *idx_out, int32_t *nnz_out, const Workspace &w, void *ws_base,
                        float *y, hipStream_t st)
{
    const int d = L->d, D = L->D;
    const int grid = ROWS_BLOCKS;
    const int max_chunk = ((D + grid - 1) / grid + ROWS_UB - 1) / ROWS_UB * ROWS_UB;
    size_t lds = (size_t)NB * d * sizeof(W) + ((size_t)NB * max_chunk + max_chunk) * 4;
    const size_t lds_tail = (size_t)ROWS_THREADS * 16;          // the in-launch reduction's tree
    const W *Wg = static_cast<const W *>(L->W_gate), *Wu = static_cast<const W *>(L->W_up);
    const W *Wd = static_cast<const W *>(L->W_downT), *xs = static_cast<const W *>(x);

    // Variant that also finishes y inside the launch (needs every block resident at once).
    if (g_fused_mode.load() == SVDP_STEP_MERGED_REDUCE) {
        uint32_t *ctrl = ctrl_for(ws_base);
        const size_t lds_f = lds > lds_tail ? lds : lds_tail;
        static int granted_f = 64 * 1024;
        static int resident = -1;
        if (ctrl != nullptr && allow_lds(k_rows<W, NB, MODE, true>, lds_f, &granted_f) == hipSuccess) {
            if (resident < 0) {
                int nb = 0;
                if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, k_rows<W, NB, MODE, true>, ROWS_THREADS,
                                                                 160 * 1024 / 2) != hipSuccess) {
                    (void)hipGetLastError();
                    nb = 0;
                }
                resident = nb;      // with half the LDS of a CU per block: a lower bound for smaller requests
            }
            const bool fits = lds_f <= 160 * 1024 / 2 ? resident * g_num_cus >= grid : g_num_cus >= grid;
            if (fits && lds_f <= 160 * 1024) {
                hipLaunchKernelGGL((k_rows<W, NB, MODE, true>), dim3(grid), dim3(ROWS_THREADS), lds_f, st, Wg, Wu, Wd,
                                   xs, B, d, D, mask, idx_in, nnz_in, idx_out, nnz_out, w.nnz, max_chunk, L->flags,
                                   w.ypart, y, ctrl, g_spin_limit.load());
                return hip_status(hipSuccess);
            }
        }
    }
    svdp_status s;
    if ((L->flags & SVDP_FLAG_REVALIDATE) != 0) {
        s = launch_rows_seq<W, NB, MODE>(L, x, B, mask, idx_in, nnz_in, idx_out, nnz_out, w, st);
    } else if (!launch_rows_matrix<W, NB, MODE>(L, x, B, mask, idx_in, nnz_in, idx_out, nnz_out, w, st, &s)) {
        static int granted = 64 * 1024;
        if (allow_lds(k_rows<W, NB, MODE, false>, lds, &granted) != hipSuccess) return SVDP_ERR_UNSUPPORTED;
        hipLaunchKernelGGL((k_rows<W, NB, MODE, false>), dim3(grid), dim3(ROWS_THREADS), lds, st, Wg, Wu, Wd, xs, B, d,
                           D, mask, idx_in, nnz_in, idx_out, nnz_out, w.nnz, max_chunk, L->flags, w.ypart, y, nullptr,
                           0);
        s = hip_status(hipSuccess);
    }
    if (s != SVDP_OK) return s;
    const int vpt = d / 4;
    const int blocks = B * ((vpt + RED_COLS - 1) / RED_COLS);
    hipLaunchKernelGGL(k_reduce_y, dim3(blocks), dim3(RED_COLS * RED_SEGS), 0, st, w.ypart,
                       MODE == ROWS_DENSE ? nullptr : w.nnz, D, D, grid, NB, B, d, y);
    return hip_status(hipSuccess);
}

svdp_status launch_compact(const uint64_t *mask, int D, int32_t *idx, int32_t *nnz, hipStream_t st)
{
    hipLaunchKernelGGL(k_compact_scan, dim3(1), dim3(SCAN_THREADS), 0, st, mask, D / 64, idx, nnz);
    return hip_status(hipSuccess);
}

inline int fused_max_chunk(int D, int G) { return ((D + G - 1) / G + ROWS_UB - 1) / ROWS_UB * ROWS_UB; }

template <typename W, int NB>
size_t fused_lds_bytes(const svdp_layer *L, int G)
{
    constexpr int VEC = Elem<W>::VEC;
    const size_t s1 = (size_t)(256 / (XP_COLS / VEC)) * NB * XP_COLS * 4;
    const size_t tsp = (size_t)NB * L->r > (size_t)FUSED_THREADS * 4 ? (size_t)NB * L->r : (size_t)FUSED_THREADS * 4;
    const size_t s2 = ((size_t)NB * L->r + (size_t)NB * SC_SLAB + tsp) * 4;
    const int mc = fused_max_chunk(L->D, G);
    const size_t s3 = ((size_t)L->D / 64 + 2) * 8 + ((size_t)NB * mc + mc) * 4;
    const size_t s4 = (size_t)FUSED_THREADS * 16;
    size_t scratch = s1 > s2 ? s1 : s2;
    scratch = scratch > s3 ? scratch : s3;
    scratch = scratch > s4 ? scratch : s4;
    return (size_t)NB * L->d * sizeof(W) + scratch;
}

// SVDP_ERR_UNSUPPORTED means "use the kernel sequence instead"
template <typename W, int NB>
svdp_status run_step_fused(const svdp_layer *L, const void *x, int B, float *y, uint64_t *mask_out, int32_t *idx_out,
                           int32_t *nnz_out, const Workspace &w, void *ws_base, hipStream_t st)
{
    constexpr int VEC = Elem<W>::VEC;
    uint32_t *ctrl = ctrl_for(ws_base);
    if (ctrl == nullptr) return SVDP_ERR_UNSUPPORTED;
    const int G = g_num_cus < ROWS_BLOCKS ? g_num_cus : ROWS_BLOCKS;
    if (L->D / 64 > 4096) return SVDP_ERR_UNSUPPORTED;
    const size_t lds = fused_lds_bytes<W, NB>(L, G);
    if (lds > 160 * 1024) return SVDP_ERR_UNSUPPORTED;
    static int granted = 64 * 1024;
    if (allow_lds(k_step_fused<W, NB>, lds, &granted) != hipSuccess) return SVDP_ERR_UNSUPPORTED;
    static int resident = -1;      // blocks of this kernel one CU can hold (1024 threads each)
    if (resident < 0) {
        int nb = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, k_step_fused<W, NB>, FUSED_THREADS, lds) != hipSuccess) {
            (void)hipGetLastError();
            nb = 0;
        }
        resident = nb;
    }
    if (resident < 1) return SVDP_ERR_UNSUPPORTED;
    const int cg = L->r / VEC;
    int lpr_log2 = 3;
    while ((1 << lpr_log2) < cg && lpr_log2 < 6) ++lpr_log2;
    hipLaunchKernelGGL((k_step_fused<W, NB>), dim3(G), dim3(FUSED_THREADS), lds, st, static_cast<const W *>(L->P),
                       static_cast<const W *>(L->Q), L->b, static_cast<const W *>(L->W_gate),
                       static_cast<const W *>(L->W_up), static_cast<const W *>(L->W_downT), static_cast<const W *>(x),
                       B, L->d, L->D, L->r, lpr_log2, L->flags, w.tpart, w.mask, w.ypart, fused_max_chunk(L->D, G), y,
                       mask_out, idx_out, nnz_out, ctrl, g_spin_limit.load());
    return hip_status(hipSuccess);
}

// dispatch on (dtype, batch capacity)
#define SVDP_DISPATCH(dt, NBv, CALL)                                                         \
    do {                                                                                     \
        if ((dt) == SVDP_F32) {                                                              \
            using W = float;                                                                 \
            switch (NBv) {                                                                   \
            case 1: { constexpr int NB = 1; return CALL; }                                   \
            case 2: { constexpr int NB = 2; return CALL; }                                   \
            case 4: { constexpr int NB = 4; return CALL; }                                   \
            default: { constexpr int NB = 8; return CALL; }                                  \
            }                                                                                \
        } else {                                                                             \
            using W = bf16;                                                                  \
            switch (NBv) {                                                                   \
            case 1: { constexpr int NB = 1; return CALL; }                                   \
            case 2: { constexpr int NB = 2; return CALL; }                                   \
            case 4: { constexpr int NB = 4; return CALL; }                                   \
            default: { constexpr int NB = 8; return CALL; }                                  \
            }                                                                                \
        }                                                                                    \
    } while (0)

template <typename W, int NB>
svdp_status run_predict(const svdp_layer *L, const void *x, int B, float *s, uint64_t *mask, const Workspace &w,
                        hipStream_t st, const GlueArgs *glue = nullptr)
{
    int nt = 0;
    svdp_status e = launch_xP<W, NB>(L, x, B, w.tpart, &nt, st, glue);
    if (e != SVDP_OK) return e;
    if (NB >= 4 && nt > 1 && !scores_on_matrix<W, NB>(L)) {
        // finish t once instead of in every score block (the vector score kernel splits the
        // partial list over threads through LDS, which costs more than a launch from 4 tokens up)
        const int count = NB * L->r;
        float *t = w.tpart + (size_t)XP_MAX_BLOCKS * NB * L->r;
        hipLaunchKernelGGL(k_tsum, dim3((count + 255) / 256), dim3(256), 0, st, w.tpart, nt, count, t);
        e = hip_status(hipSuccess);
        if (e != SVDP_OK) return e;
        return launch_scores<W, NB>(L, t, 1, B, s, mask, st);
    }
    return launch_scores<W, NB>(L, w.tpart, nt, B, s, mask, st);
}

template <typename W, int NB>
svdp_status run_step(const svdp_layer *L, const void *x, int B, float *y, uint64_t *mask_out, int32_t *idx_out,
                     int32_t *nnz_out, const Workspace &w, void *ws_base, hipStream_t st,
                     const GlueArgs *glue = nullptr)
{
    if (glue != nullptr) {
        // x is made by the first kernel (from x_prev = x); the row kernel reads it from x_out
        uint64_t *mask = mask_out ? mask_out : w.mask;
        svdp_status e = run_predict<W, NB>(L, x, B, nullptr, mask, w, st, glue);
        if (e != SVDP_OK) return e;
        return launch_rows<W, NB, ROWS_MASK>(L, glue->x_out, B, mask, nullptr, nullptr, idx_out, nnz_out, w, ws_base, y,
                                             st);
    }
    if (g_fused_mode.load() == SVDP_STEP_PERSISTENT) {
        const svdp_status f = run_step_fused<W, NB>(L, x, B, y, mask_out, idx_out, nnz_out, w, ws_base, st);
        if (f != SVDP_ERR_UNSUPPORTED) return f;
    }
    uint64_t *mask = mask_out ? mask_out : w.mask;
    svdp_status e = run_predict<W, NB>(L, x, B, nullptr, mask, w, st);
    if (e != SVDP_OK) return e;
    return launch_rows<W, NB, ROWS_MASK>(L, x, B, mask, nullptr, nullptr, idx_out, nnz_out, w, ws_base, y, st);
}

svdp_status dispatch_predict(const svdp_layer *L, const void *x, int B, float *s, const Workspace &w, hipStream_t st)
{
    SVDP_DISPATCH(L->wdtype, nb_of(B), (run_predict<W, NB>(L, x, B, s, nullptr, w, st)));
}
svdp_status dispatch_sparse(const svdp_layer *L, const void *x, int B, const int32_t *idx, const int32_t *nnz,
                            float *y, const Workspace &w, void *ws_base, hipStream_t st)
{
    SVDP_DISPATCH(L->wdtype, nb_of(B),
                  (launch_rows<W, NB, ROWS_LIST>(L, x, B, nullptr, idx, nnz, nullptr, nullptr, w, ws_base, y, st)));
}
svdp_status dispatch_dense(const svdp_layer *L, const void *x, int B, float *y, const Workspace &w, void *ws_base,
                           hipStream_t st)
{
    SVDP_DISPATCH(L->wdtype, nb_of(B),
                  (launch_rows<W, NB, ROWS_DENSE>(L, x, B, nullptr, nullptr, nullptr, nullptr, nullptr, w, ws_base, y, st)));
}
template <typename W, int NB>
svdp_status launch_rows_only(const svdp_layer *L, const void *x, int B, const uint64_t *mask, const Workspace &w,
                             hipStream_t st)
{
    const int d = L->d, D = L->D;
    const int grid = ROWS_BLOCKS;
    const int max_chunk = ((D + grid - 1) / grid + ROWS_UB - 1) / ROWS_UB * ROWS_UB;
    const size_t lds = (size_t)NB * d * sizeof(W) + ((size_t)NB * max_chunk + max_chunk) * 4;
    if ((L->flags & SVDP_FLAG_REVALIDATE) != 0)
        return launch_rows_seq<W, NB, ROWS_MASK>(L, x, B, mask, nullptr, nullptr, nullptr, nullptr, w, st);
    svdp_status sm;
    if (launch_rows_matrix<W, NB, ROWS_MASK>(L, x, B, mask, nullptr, nullptr, nullptr, nullptr, w, st, &sm)) return sm;
    static int granted = 64 * 1024;
    if (allow_lds(k_rows<W, NB, ROWS_MASK, false>, lds, &granted) != hipSuccess) return SVDP_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((k_rows<W, NB, ROWS_MASK, false>), dim3(grid), dim3(ROWS_THREADS), lds, st,
                       static_cast<const W *>(L->W_gate), static_cast<const W *>(L->W_up),
                       static_cast<const W *>(L->W_downT), static_cast<const W *>(x), B, d, D, mask, nullptr, nullptr,
                       nullptr, nullptr, w.nnz, max_chunk, L->flags, w.ypart, nullptr, nullptr, 0);
    return hip_status(hipSuccess);
}
svdp_status dispatch_rows_only(const svdp_layer *L, const void *x, int B, const uint64_t *mask, const Workspace &w,
                               hipStream_t st)
{
    SVDP_DISPATCH(L->wdtype, nb_of(B), (launch_rows_only<W, NB>(L, x, B, mask, w, st)));
}
svdp_status dispatch_step(const svdp_layer *L, const void *x, int B, float *y, uint64_t *mask_out,
                          int32_t *idx_out, int32_t *nnz_out, const Workspace &w, void *ws_base, hipStream_t st,
                          const GlueArgs *glue = nullptr)
{
    SVDP_DISPATCH(L->wdtype, nb_of(B),
                  (run_step<W, NB>(L, x, B, y, mask_out, idx_out, nnz_out, w, ws_base, st, glue)));
}

inline bool bad_batch(int B) { return B < 1 || B > SVDP_MAX_BATCH; }

}  // namespace

extern "C" {

size_t svdp_workspace_bytes(const svdp_layer *layer, int32_t max_batch)
{
    if (layer == nullptr || bad_batch(max_batch)) return 0;
    if (check_shape(layer->d, layer->D, layer->r, layer->wdtype) != SVDP_OK) return 0;
    return carve(nullptr, layer->d, layer->D, layer->r, nb_of(max_batch)).bytes;
}

svdp_status svdp_predict(const svdp_layer *layer, const void *x, int32_t B, float *s, void *ws, size_t ws_bytes,
                         void *stream)
{
    svdp_status st = check_layer(layer, true, false);
    if (st != SVDP_OK) return st;
    if (x == nullptr || s == nullptr || bad_batch(B) || !aligned16(x)) return SVDP_ERR_INVALID_ARG;
    Workspace w;
    st = check_ws(layer, B, ws, ws_bytes, &w);
    if (st != SVDP_OK) return st;
    return dispatch_predict(layer, x, B, s, w, static_cast<hipStream_t>(stream));
}

svdp_status svdp_compact(const float *s, int32_t B, int32_t D, uint64_t *mask, int32_t *idx, int32_t *nnz,
                         void *stream)
{
    if (s == nullptr || mask == nullptr || idx == nullptr || nnz == nullptr || bad_batch(B) || D <= 0) return SVDP_ERR_INVALID_ARG;
    if (D % 64 != 0) return SVDP_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(k_mask_from_scores, dim3((D / 64 + 3) / 4), dim3(256), 0, st, s, B, D, mask);
    svdp_status e = hip_status(hipSuccess);
    if (e != SVDP_OK) return e;
    return launch_compact(mask, D, idx, nnz, st);
}

svdp_status svdp_sparse_ffn(const svdp_layer *layer, const void *x, int32_t B, const int32_t *idx,
                            const int32_t *nnz, float *y, void *ws, size_t ws_bytes, void *stream)
{
    svdp_status st = check_layer(layer, false, true);
    if (st != SVDP_OK) return st;
    if (x == nullptr || y == nullptr || idx == nullptr || nnz == nullptr || bad_batch(B) || !aligned16(x) ||
        !aligned16(y))
        return SVDP_ERR_INVALID_ARG;
    Workspace w;
    st = check_ws(layer, B, ws, ws_bytes, &w);
    if (st != SVDP_OK) return st;
    return dispatch_sparse(layer, x, B, idx, nnz, y, w, ws, static_cast<hipStream_t>(stream));
}

svdp_status svdp_dense_ffn(const svdp_layer *layer, const void *x, int32_t B, float *y, void *ws, size_t ws_bytes,
                           void *stream)
{
    svdp_status st = check_layer(layer, false, true);
    if (st != SVDP_OK) return st;
    if (x == nullptr || y == nullptr || bad_batch(B) || !aligned16(x) || !aligned16(y)) return SVDP_ERR_INVALID_ARG;
    Workspace w;
    st = check_ws(layer, B, ws, ws_bytes, &w);
    if (st != SVDP_OK) return st;
    return dispatch_dense(layer, x, B, y, w, ws, static_cast<hipStream_t>(stream));
}

svdp_status svdp_ffn_step(const svdp_layer *layer, const void *x, int32_t B, float *y, uint64_t *mask_out,
                          int32_t *idx_out, int32_t *nnz_out, void *ws, size_t ws_bytes, void *stream)
{
    svdp_status st = check_layer(layer, true, true);
    if (st != SVDP_OK) return st;
    if (x == nullptr || y == nullptr || bad_batch(B) || !aligned16(x) || !aligned16(y)) return SVDP_ERR_INVALID_ARG;
    Workspace w;
    st = check_ws(layer, B, ws, ws_bytes, &w);
    if (st != SVDP_OK) return st;
    return dispatch_step(layer, x, B, y, mask_out, idx_out, nnz_out, w, ws, static_cast<hipStream_t>(stream));
}

svdp_status svdp_ffn_step_glued(const svdp_layer *layer, const void *x_prev, const float *y_prev, const float *shift,
                                float eps, void *x_out, int32_t B, float *y, uint64_t *mask_out, int32_t *idx_out,
                                int32_t *nnz_out, void *ws, size_t ws_bytes, void *stream)
{
    svdp_status st = check_layer(layer, true, true);
    if (st != SVDP_OK) return st;
    if (x_prev == nullptr || y_prev == nullptr || shift == nullptr || x_out == nullptr || y == nullptr ||
        bad_batch(B) || !aligned16(x_prev) || !aligned16(x_out) || !aligned16(y) || !(eps >= 0.f))
        return SVDP_ERR_INVALID_ARG;
    Workspace w;
    st = check_ws(layer, B, ws, ws_bytes, &w);
    if (st != SVDP_OK) return st;
    const GlueArgs glue{y_prev, shift, eps, x_out};
    return dispatch_step(layer, x_prev, B, y, mask_out, idx_out, nnz_out, w, ws, static_cast<hipStream_t>(stream), &glue);
}

svdp_status svdp_active_rows(const svdp_layer *layer, const void *x, int32_t B, const uint64_t *mask, void *ws,
                             size_t ws_bytes, void *stream)
{
    svdp_status st = check_layer(layer, false, true);
    if (st != SVDP_OK) return st;
    if (x == nullptr || mask == nullptr || bad_batch(B) || !aligned16(x)) return SVDP_ERR_INVALID_ARG;
    Workspace w;
    st = check_ws(layer, B, ws, ws_bytes, &w);
    if (st != SVDP_OK) return st;
    return dispatch_rows_only(layer, x, B, mask, w, static_cast<hipStream_t>(stream));
}

svdp_status svdp_stack_glue(const void *x, const float *y, const float *shift, int32_t d, int32_t dtype, float eps,
                            void *x_next, void *stream)
{
    if (x == nullptr || y == nullptr || shift == nullptr || x_next == nullptr || d <= 0) return SVDP_ERR_INVALID_ARG;
    if (dtype != SVDP_F32 && dtype != SVDP_BF16) return SVDP_ERR_UNSUPPORTED;
    // whole 16-byte vectors of x, as for a layer's d
    if (d % (dtype == SVDP_BF16 ? 8 : 4) != 0) return SVDP_ERR_UNSUPPORTED;
    if (!aligned16(x) || !aligned16(y) || !aligned16(shift) || !aligned16(x_next)) return SVDP_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dtype == SVDP_F32)
        hipLaunchKernelGGL(k_stack_glue<float>, dim3(1), dim3(256), 0, st, static_cast<const float *>(x), y, shift,
                           d, eps, static_cast<float *>(x_next));
    else if (dtype == SVDP_BF16)
        hipLaunchKernelGGL(k_stack_glue<bf16>, dim3(1), dim3(256), 0, st, static_cast<const bf16 *>(x), y, shift, d,
                           eps, static_cast<bf16 *>(x_next));
    else
        return SVDP_ERR_UNSUPPORTED;
    return hip_status(hipSuccess);
}

const char *svdp_status_string(svdp_status st)
{
    switch (st) {
    case SVDP_OK: return "ok";
    case SVDP_ERR_INVALID_ARG: return "invalid argument";
    case SVDP_ERR_UNSUPPORTED: return "unsupported shape or dtype";
    case SVDP_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case SVDP_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

size_t svdp_calib_workspace_bytes(int32_t D, int32_t T, int32_t eta)
{
    if (D < 1 || T < 1 || T > CAL_MAX_T || eta < 1) return 0;
    const size_t MS = ((size_t)T + eta - 1) / eta;
    return align_up((size_t)D * MS * 4) + 2 * align_up((size_t)D * (MS + 1) * 4) + align_up((size_t)D * 4) +
           align_up(sizeof(SelectState)) + align_up((size_t)SEL_BINS * 8) + 2 * align_up((size_t)D * 4);
}

svdp_status svdp_calib_bias(const float *w, const float *s, int32_t D, int32_t T, int32_t eta, int64_t need,
                            float *b, int32_t *k, int32_t *steps, float *kendall, void *ws, size_t ws_bytes,
                            void *stream)
{
    if (w == nullptr || s == nullptr || b == nullptr || D < 1 || T < 1 || eta < 1 || need < 0)
        return SVDP_ERR_INVALID_ARG;
    if (T > CAL_MAX_T) return SVDP_ERR_UNSUPPORTED;
    const size_t bytes = svdp_calib_workspace_bytes(D, T, eta);
    if (ws == nullptr || (reinterpret_cast<uintptr_t>(ws) & (ALIGN - 1)) || ws_bytes < bytes) return SVDP_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int MS = (T + eta - 1) / eta;
    char *p = static_cast<char *>(ws);
    float *key = reinterpret_cast<float *>(p);
    p += align_up((size_t)D * MS * 4);
    int32_t *drop = reinterpret_cast<int32_t *>(p);
    p += align_up((size_t)D * (MS + 1) * 4);
    float *tauc = reinterpret_cast<float *>(p);
    p += align_up((size_t)D * (MS + 1) * 4);
    int32_t *k0 = reinterpret_cast<int32_t *>(p);
    int n2 = 1;
    while (n2 < T) n2 <<= 1;
    const size_t lds = (size_t)n2 * 8 + (size_t)T * 8 + (size_t)(MS + 1) * 8;
    static int granted = 64 * 1024;
    if (allow_lds(k_calib_sort, lds, &granted) != hipSuccess) return SVDP_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(k_calib_sort, dim3(D), dim3(CAL_THREADS), lds, st, w, s, T, n2, eta, MS, key, drop, tauc, k0,
                       kendall);
    svdp_status e = hip_status(hipSuccess);
    if (e != SVDP_OK) return e;
    p += align_up((size_t)D * 4);
    SelectState *state = reinterpret_cast<SelectState *>(p);
    p += align_up(sizeof(SelectState));
    long long *hist = reinterpret_cast<long long *>(p);
    const size_t items = (size_t)D * MS;
    const int hb = (int)((items + 256 * 8 - 1) / (256 * 8) < 2048 ? (items + 256 * 8 - 1) / (256 * 8) : 2048);
    hipLaunchKernelGGL(k_select_init, dim3(1), dim3(SEL_THREADS), 0, st, drop, D, MS, (long long)need, state, hist);
    hipLaunchKernelGGL((k_select_hist<23, 8>), dim3(hb), dim3(256), 0, st, key, drop, D, MS, state, hist);
    hipLaunchKernelGGL((k_select_pick<23, true>), dim3(1), dim3(64), 0, st, state, hist);
    hipLaunchKernelGGL((k_select_hist<15, 8>), dim3(hb), dim3(256), 0, st, key, drop, D, MS, state, hist);
    hipLaunchKernelGGL((k_select_pick<15, false>), dim3(1), dim3(64), 0, st, state, hist);
    hipLaunchKernelGGL((k_select_hist<7, 8>), dim3(hb), dim3(256), 0, st, key, drop, D, MS, state, hist);
    hipLaunchKernelGGL((k_select_pick<7, false>), dim3(1), dim3(64), 0, st, state, hist);
    hipLaunchKernelGGL((k_select_hist<0, 7>), dim3(hb), dim3(256), 0, st, key, drop, D, MS, state, hist);
    hipLaunchKernelGGL((k_select_pick<0, false>), dim3(1), dim3(64), 0, st, state, hist);
    p += align_up((size_t)SEL_BINS * 8);
    int32_t *lo = reinterpret_cast<int32_t *>(p);
    p += align_up((size_t)D * 4);
    int32_t *up = reinterpret_cast<int32_t *>(p);
    hipLaunchKernelGGL(k_select_bounds, dim3((D + 255) / 256), dim3(256), 0, st, key, D, MS, state, lo, up);
    hipLaunchKernelGGL(k_select_finish, dim3(1), dim3(SEL_THREADS), 0, st, lo, up, drop, tauc, k0, D, T, eta, MS, state, b,
                       k, steps);
    return hip_status(hipSuccess);
}

size_t svdp_calib_stats_workspace_bytes(const svdp_layer *layer, int32_t T)
{
    if (check_layer(layer, true, true) != SVDP_OK || layer->wdtype != SVDP_BF16 || T < 1) return 0;
    return align_up((size_t)layer->r * layer->d * 2) + align_up((size_t)layer->D * 4) +
           align_up((size_t)T * 3 * layer->r * 2);
}

svdp_status svdp_calib_stats(const svdp_layer *layer, const void *X, int32_t T, float *w, float *s, void *ws,
                             size_t ws_bytes, void *stream)
{
    svdp_status e = check_layer(layer, true, true);
    if (e != SVDP_OK) return e;
    if (X == nullptr || w == nullptr || s == nullptr || T < 1) return SVDP_ERR_INVALID_ARG;
    if (layer->wdtype != SVDP_BF16) return SVDP_ERR_UNSUPPORTED;
    const size_t bytes = svdp_calib_stats_workspace_bytes(layer, T);
    if (ws == nullptr || (reinterpret_cast<uintptr_t>(ws) & (ALIGN - 1)) || ws_bytes < bytes) return SVDP_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int d = layer->d, D = layer->D, r = layer->r;
    char *p = static_cast<char *>(ws);
    bf16 *Pt = reinterpret_cast<bf16 *>(p);                      // [r][d]
    p += align_up((size_t)r * d * 2);
    float *cn = reinterpret_cast<float *>(p);                    // [D] squared column norms of W_down
    p += align_up((size_t)D * 4);
    uint16_t *tp = reinterpret_cast<uint16_t *>(p);              // [T][3r]: t = x P as three bf16 terms
    const bf16 *Wg = static_cast<const bf16 *>(layer->W_gate), *Wu = static_cast<const bf16 *>(layer->W_up);
    const bf16 *Xb = static_cast<const bf16 *>(X);
    auto tiles = [](int n, int b) { return (n + b - 1) / b; };

    hipLaunchKernelGGL(k_row_norm2, dim3(tiles(D, 4)), dim3(256), 0, st, static_cast<const bf16 *>(layer->W_downT), D, d,
                       cn);
    hipLaunchKernelGGL(k_transpose16, dim3(tiles(r, 32), tiles(d, 32)), dim3(256), 0, st,
                       static_cast<const uint16_t *>(layer->P), d, r, reinterpret_cast<uint16_t *>(Pt));
    // w = (ReLU(W_gate X^T) * (W_up X^T))^2 * cn
    hipLaunchKernelGGL((k_gemm_nt<2, EPI_DAMAGE>), dim3(tiles(T, GM_BN), tiles(D, GM_BM)), dim3(GM_THREADS), 0, st, Wg,
                       Wu, d, d, Xb, d, D, T, d, cn, w, nullptr, T);
    // t = X P, split
    hipLaunchKernelGGL((k_gemm_nt<1, EPI_SPLIT3>), dim3(tiles(r, GM_BN), tiles(T, GM_BM)), dim3(GM_THREADS), 0, st, Xb,
                       nullptr, d, d, Pt, d, T, r, d, nullptr, nullptr, tp, 3 * r);
    // s = Q t^T over the three terms
    hipLaunchKernelGGL((k_gemm_nt<1, EPI_PLAIN>), dim3(tiles(T, GM_BN), tiles(D, GM_BM)), dim3(GM_THREADS), 0, st,
                       static_cast<const bf16 *>(layer->Q), nullptr, r, r, reinterpret_cast<const bf16 *>(tp), 3 * r, D,
                       T, 3 * r, nullptr, s, nullptr, T);
    return hip_status(hipSuccess);
}

const char *svdp_version(void) { return "0.3"; }

void svdp_set_step_mode(int32_t mode, int32_t spin_limit)
{
    if (mode >= SVDP_STEP_SEQUENCE && mode <= SVDP_STEP_MERGED_REDUCE) g_fused_mode.store(mode);
    if (spin_limit > 0) g_spin_limit.store(spin_limit);
}

void svdp_set_engine(int32_t engine)
{
    if (engine >= SVDP_ENGINE_AUTO && engine <= SVDP_ENGINE_MATRIX) g_engine.store(engine);
}

svdp_status svdp_step_timeouts(int32_t *count)
{
    if (count == nullptr) return SVDP_ERR_INVALID_ARG;
    *count = 0;
    std::lock_guard<std::mutex> lock(g_slot_mutex);
    if (g_ctrl_base == nullptr) return SVDP_OK;          // the persistent kernel never ran
    if (hipDeviceSynchronize() != hipSuccess) return SVDP_ERR_HIP;
    for (size_t i = 0; i < g_slots.size(); ++i) {
        uint32_t flag = 0;
        uint32_t *p = g_ctrl_base + i * CTRL_WORDS + CTRL_ERROR;
        if (hipMemcpy(&flag, p, sizeof(flag), hipMemcpyDeviceToHost) != hipSuccess) return SVDP_ERR_HIP;
        if (flag != 0) {
            *count += 1;
            flag = 0;
            if (hipMemcpy(p, &flag, sizeof(flag), hipMemcpyHostToDevice) != hipSuccess) return SVDP_ERR_HIP;
        }
    }
    return SVDP_OK;
}

#ifdef SVDP_TRACE
// Debug builds only: copy the phase time stamps to the host (synchronises).
int svdp_debug_read_trace(unsigned long long *host, size_t count)
{
    const size_t total = sizeof(svdp::g_trace) / sizeof(svdp::g_trace[0]);
    if (count > total) count = total;
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(svdp::g_trace), count * sizeof(unsigned long long), 0,
                                    hipMemcpyDeviceToHost);
}
#endif

}  // extern "C"
