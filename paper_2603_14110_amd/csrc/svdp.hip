// C-ABI entry points of libsvdp (see include/svdp.h): host-side validation,
// workspace carving and kernel launches.  No allocation, no synchronisation,
// no state kept between calls (everything follows from a call's arguments).
#include "../../include/svdp.h"

#include <hip/hip_runtime.h>

#include "svdp_kernels.h"
#include "svdp_rows_mfma.h"
#include "svdp_rows_seq.h"
#include "svdp_calib.h"
#include "svdp_calib_stats.h"
#include "svdp_whiten.h"

#include <algorithm>
#include <atomic>
#include <cmath>
#include <numeric>
#include <mutex>
#include <type_traits>
#include <vector>

namespace {

using namespace svdp;

constexpr int XP_MAX_BLOCKS = 128;    // stage-1 row slabs of P (d <= 16384)
constexpr int ROWS_BLOCKS = 256;      // row-kernel blocks: one chunk of the row list and one partial y each (128 to
                                      // 512 were measured; 256 is best for every batch size)
constexpr size_t ALIGN = 256;
constexpr size_t LDS_DEFAULT = 64 * 1024;     // dynamic LDS a kernel may use without asking
constexpr size_t LDS_MAX = 160 * 1024;        // LDS of one gfx950 compute unit
constexpr int MAX_DEVICES = 64;

inline size_t align_up(size_t v) { return (v + ALIGN - 1) / ALIGN * ALIGN; }
inline int nb_of(int B) { return B <= 1 ? 1 : B <= 2 ? 2 : B <= 4 ? 4 : 8; }
inline int vec_of(int dt) { return dt == SVDP_F32 ? 4 : 8; }
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int round_up(int v, int m) { return (v + m - 1) / m * m; }
inline bool bad_batch(int B) { return B < 1 || B > SVDP_MAX_BATCH; }

constexpr uint32_t ALL_FLAGS =
    SVDP_FLAG_DRELU | SVDP_FLAG_REVALIDATE | SVDP_FLAG_ENGINE_VECTOR | SVDP_FLAG_ENGINE_MATRIX;

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
    if (L->flags & ~ALL_FLAGS) return SVDP_ERR_INVALID_ARG;
    if ((L->flags & SVDP_FLAG_ENGINE_VECTOR) && (L->flags & SVDP_FLAG_ENGINE_MATRIX)) return SVDP_ERR_INVALID_ARG;
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

inline svdp_status hip_status(hipError_t e)
{
    if (e == hipSuccess) e = hipGetLastError();
    else (void)hipGetLastError();
    return e == hipSuccess ? SVDP_OK : SVDP_ERR_HIP;
}

// Dynamic LDS above the default limit has to be enabled per kernel and device once.  What was
// enabled is remembered per kernel (the template parameter is the kernel itself) and device;
// the driver call is made under a lock, so that the remembered size never runs ahead of it.
std::mutex g_grant_mutex;
template <auto Kernel>
bool grant_lds(size_t bytes)
{
    static std::atomic<int> granted[MAX_DEVICES];
    if (bytes <= LDS_DEFAULT) return true;
    if (bytes > LDS_MAX) return false;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) {
        (void)hipGetLastError();
        return false;
    }
    if ((int)bytes <= granted[dev].load(std::memory_order_acquire)) return true;
    std::lock_guard<std::mutex> lock(g_grant_mutex);
    if ((int)bytes <= granted[dev].load(std::memory_order_relaxed)) return true;
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(Kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)bytes) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    granted[dev].store((int)bytes, std::memory_order_release);
    return true;
}

// ---- which kernels a call uses and how much LDS they need: pure host arithmetic ----

enum Engine { ENGINE_AUTO = 0, ENGINE_VECTOR = 1, ENGINE_MATRIX = 2 };
inline Engine engine_of(const svdp_layer *L)
{
    return (L->flags & SVDP_FLAG_ENGINE_VECTOR) ? ENGINE_VECTOR
                                                : (L->flags & SVDP_FLAG_ENGINE_MATRIX) ? ENGINE_MATRIX : ENGINE_AUTO;
}

template <typename W, int NB>
size_t xp_lds(const svdp_layer *)
{
    constexpr int VEC = Elem<W>::VEC;
    const size_t outs = (size_t)NB * XP_COLS;
    const size_t parts = XP_THREADS / outs >= 1 ? XP_THREADS / outs : 1;
    const size_t nsub = XP_THREADS / (XP_COLS / VEC);
    return ((size_t)NB * XP_ROWS + nsub * (outs + 1) + parts * outs) * 4;
}

// Whether the score kernel on the matrix cores takes this layer and batch capacity.
template <typename W, int NB>
bool scores_on_matrix(const svdp_layer *L)
{
    if (!std::is_same<W, bf16>::value) return false;
    const Engine engine = engine_of(L);
    const bool want = engine == ENGINE_MATRIX || (engine == ENGINE_AUTO && NB >= 4);
    return want && L->r % 32 == 0 && L->r <= 32 * SCM_KB;
}
template <int NB>
constexpr int scores_threads() { return NB <= 2 ? 512 : 256; }
template <typename W, int NB>
size_t scores_lds(const svdp_layer *L)
{
    if (scores_on_matrix<W, NB>(L)) return (size_t)3 * NB * L->r * 2;
    const size_t thr = scores_threads<NB>();
    const size_t tsp = (size_t)NB * L->r > thr * 4 ? (size_t)NB * L->r : thr * 4;
    return ((size_t)NB * L->r + (size_t)NB * SC_SLAB + tsp) * 4;
}

enum RowsKind { ROWS_VECTOR = 0, ROWS_SEQ = 1, ROWS_MATRIX = 2 };
struct RowsPlan {
    RowsKind kind;
    int max_chunk;      // LDS row capacity of a block
    int min_chunk;      // fewest rows a block takes (short lists use fewer blocks)
    size_t lds;
    bool split;         // gate/up kernel, then the down projection over column slices (k_down_slices)
};

// Split organisation: parts of the list per column slice, fewest rows of a part, and where its buffers lie
// inside the workspace's partial-y region [ROWS_BLOCKS][NB][d]: the RG partial y's, then h [D][NB], then the list [D].
constexpr int DOWN_RG = 8;
constexpr int DOWN_MIN_CHUNK = 64;
inline size_t split_h_offset(int d, int NB) { return align_up((size_t)DOWN_RG * NB * d * 4); }
inline size_t split_list_offset(int d, int D, int NB) { return split_h_offset(d, NB) + align_up((size_t)D * NB * 4); }
inline bool split_fits(int d, int D, int NB)
{
    return (D + DOWN_RG - 1) / DOWN_RG <= DS_MAX_CHUNK && d % DS_SW == 0 &&
           split_list_offset(d, D, NB) + (size_t)D * 4 <= (size_t)ROWS_BLOCKS * NB * d * 4;
}

template <typename W, int NB>
RowsPlan plan_rows(const svdp_layer *L)
{
    const int d = L->d, D = L->D, G = ROWS_BLOCKS;
    const int per = (D + G - 1) / G;
    RowsPlan p;
    p.split = false;
    if ((L->flags & SVDP_FLAG_REVALIDATE) != 0) {
        p.kind = ROWS_SEQ;
        p.min_chunk = 4;
        p.max_chunk = round_up(per > p.min_chunk ? per : p.min_chunk, ROWS_UB);
        p.lds = (size_t)NB * d * sizeof(W) + ((size_t)2 * NB * p.max_chunk + (size_t)3 * p.max_chunk) * 4;
        return p;
    }
    if (std::is_same<W, bf16>::value) {
        const Engine engine = engine_of(L);
        // measured on the Mistral shape: ahead of the vector kernel only at the largest batch capacity
        const bool want = engine == ENGINE_MATRIX || (engine == ENGINE_AUTO && NB >= 8);
        if (want && d % 512 == 0) {
            p.kind = ROWS_MATRIX;
            p.min_chunk = MF_ROWS;
            p.max_chunk = round_up(per > p.min_chunk ? per : p.min_chunk, MF_ROWS);
            p.lds = (size_t)NB * d * 2 + ((size_t)ROWS_WAVES * p.max_chunk * 2 * NB + p.max_chunk) * 4;
            p.split = true;
            if (p.lds <= LDS_MAX && split_fits(d, D, NB)) return p;
            p.split = false;
        }
    }
    p.kind = ROWS_VECTOR;
    p.min_chunk = 4;
    p.max_chunk = round_up(per > p.min_chunk ? per : p.min_chunk, ROWS_UB);
    p.lds = (size_t)NB * d * sizeof(W) + ((size_t)NB * p.max_chunk + p.max_chunk) * 4;
    return p;
}

// dispatch on (dtype, batch capacity): f(W tag, NB constant)
template <typename T>
struct Tag {
    using type = T;
};
template <typename F>
auto dispatch(int dt, int NBv, F &&f)
{
    auto on_nb = [&](auto wtag) {
        switch (NBv) {
        case 1: return f(wtag, std::integral_constant<int, 1>{});
        case 2: return f(wtag, std::integral_constant<int, 2>{});
        case 4: return f(wtag, std::integral_constant<int, 4>{});
        default: return f(wtag, std::integral_constant<int, 8>{});
        }
    };
    return dt == SVDP_F32 ? on_nb(Tag<float>{}) : on_nb(Tag<bf16>{});
}

// Everything every kernel of the layer needs fits the LDS of a compute unit (pure).
bool layer_fits(const svdp_layer *L, int NBv)
{
    return dispatch(L->wdtype, NBv, [&](auto wt, auto nb) {
        using W = typename decltype(wt)::type;
        constexpr int NB = decltype(nb)::value;
        return xp_lds<W, NB>(L) <= LDS_MAX && scores_lds<W, NB>(L) <= LDS_MAX && plan_rows<W, NB>(L).lds <= LDS_MAX;
    });
}

svdp_status check_ws(const svdp_layer *L, int B, void *ws, size_t ws_bytes, Workspace *out)
{
    if (!layer_fits(L, nb_of(B))) return SVDP_ERR_UNSUPPORTED;
    if (ws == nullptr || (reinterpret_cast<uintptr_t>(ws) & (ALIGN - 1))) return SVDP_ERR_WORKSPACE;
    *out = carve(ws, L->d, L->D, L->r, nb_of(B));
    if (ws_bytes < out->bytes) return SVDP_ERR_WORKSPACE;
    return SVDP_OK;
}

// ---- preparation (LDS grants; nothing is enqueued) and launch, per kernel ----

// The stacked benchmark's glue folded into the first kernel of a step (svdp_ffn_step_glued).
struct GlueArgs {
    const float *y_prev;
    const float *shift;
    float eps;
    void *x_out;
};

template <typename W, int NB>
bool prepare_xP(const svdp_layer *L, bool glue)
{
    const size_t lds = xp_lds<W, NB>(L);
    return glue ? grant_lds<k_xP<W, NB, true>>(lds) : grant_lds<k_xP<W, NB, false>>(lds);
}

template <typename W, int NB>
svdp_status launch_xP(const svdp_layer *L, const void *x, int B, float *tpart, int *nt_out, hipStream_t st,
                      const GlueArgs *glue)
{
    const int d = L->d, r = L->r;
    const int nt = (d + XP_ROWS - 1) / XP_ROWS;           // <= XP_MAX_BLOCKS since d <= 16384
    const int ncs = (r + XP_COLS - 1) / XP_COLS;
    const size_t lds = xp_lds<W, NB>(L);
    if (glue != nullptr) {
        hipLaunchKernelGGL((k_xP<W, NB, true>), dim3(nt, ncs), dim3(XP_THREADS), lds, st, static_cast<const W *>(L->P),
                           static_cast<const W *>(x), B, d, r, tpart, glue->y_prev, glue->shift, glue->eps,
                           static_cast<W *>(glue->x_out));
    } else {
        hipLaunchKernelGGL((k_xP<W, NB, false>), dim3(nt, ncs), dim3(XP_THREADS), lds, st,
                           static_cast<const W *>(L->P), static_cast<const W *>(x), B, d, r, tpart, nullptr, nullptr,
                           0.f, nullptr);
    }
    *nt_out = nt;
    return hip_status(hipSuccess);
}

// lanes per row of the vector score kernel: 2^k >= 16-byte column groups per row of Q, 8..64
template <typename W>
int scores_lpr_log2(const svdp_layer *L)
{
    const int cg = L->r / Elem<W>::VEC;
    return cg <= 8 ? 3 : cg <= 16 ? 4 : cg <= 32 ? 5 : 6;
}

template <typename W, int NB, typename F>
auto with_scores_kernel(const svdp_layer *L, F &&f)
{
    constexpr int THR = scores_threads<NB>();
    switch (scores_lpr_log2<W>(L)) {
    case 3: return f(std::integral_constant<decltype(&k_scores<W, NB, 3, THR>), &k_scores<W, NB, 3, THR>>{});
    case 4: return f(std::integral_constant<decltype(&k_scores<W, NB, 4, THR>), &k_scores<W, NB, 4, THR>>{});
    case 5: return f(std::integral_constant<decltype(&k_scores<W, NB, 5, THR>), &k_scores<W, NB, 5, THR>>{});
    default: return f(std::integral_constant<decltype(&k_scores<W, NB, 6, THR>), &k_scores<W, NB, 6, THR>>{});
    }
}

template <typename W, int NB>
bool prepare_scores(const svdp_layer *L)
{
    const size_t lds = scores_lds<W, NB>(L);
    if constexpr (std::is_same<W, bf16>::value) {
        if (scores_on_matrix<W, NB>(L)) return grant_lds<k_scores_mfma<NB>>(lds);
    }
    return with_scores_kernel<W, NB>(L, [&](auto k) { return grant_lds<decltype(k)::value>(lds); });
}

template <typename W, int NB>
svdp_status launch_scores(const svdp_layer *L, const float *tpart, int nt, int B, float *s_out, uint64_t *mask_out,
                          hipStream_t st)
{
    const size_t lds = scores_lds<W, NB>(L);
    if constexpr (std::is_same<W, bf16>::value) {
        if (scores_on_matrix<W, NB>(L)) {
            hipLaunchKernelGGL((k_scores_mfma<NB>), dim3(L->D / SC_SLAB), dim3(SCM_THREADS), lds, st,
                               static_cast<const bf16 *>(L->Q), L->b, tpart, nt, B, L->D, L->r, s_out, mask_out);
            return hip_status(hipSuccess);
        }
    }
    // block size: 512 threads for one or two tokens (short critical path), 256 for larger batches
    // (fewer wavefronts repeating the per-wave overhead); measured on the 7B and Mistral shapes
    with_scores_kernel<W, NB>(L, [&](auto k) {
        hipLaunchKernelGGL(decltype(k)::value, dim3(L->D / SC_SLAB), dim3(scores_threads<NB>()), lds, st,
                           static_cast<const W *>(L->Q), L->b, tpart, nt, B, L->D, L->r, s_out, mask_out);
        return 0;
    });
    return hip_status(hipSuccess);
}

template <typename W, int NB, int MODE>
bool prepare_rows(const svdp_layer *L)
{
    const RowsPlan p = plan_rows<W, NB>(L);
    if (p.kind == ROWS_SEQ) return grant_lds<k_rows_seq<W, NB, MODE>>(p.lds);
    if constexpr (std::is_same<W, bf16>::value) {
        if (p.kind == ROWS_MATRIX) return grant_lds<k_gate_up_mfma<NB, MODE>>(p.lds);
    }
    return grant_lds<k_rows<W, NB, MODE>>(p.lds);
}

// Gate, up and down over the list.  With y == nullptr the final sum of the partial results is left out (they
// stay in the workspace): the row work by itself, for timing.
template <typename W, int NB, int MODE>
svdp_status launch_rows(const svdp_layer *L, const void *x, int B, const uint64_t *mask, const int32_t *idx_in,
                        const int32_t *nnz_in, int32_t *idx_out, int32_t *nnz_out, const Workspace &w, float *y,
                        hipStream_t st)
{
    const RowsPlan p = plan_rows<W, NB>(L);
    const int d = L->d, D = L->D;
    const W *Wg = static_cast<const W *>(L->W_gate), *Wu = static_cast<const W *>(L->W_up);
    const W *Wd = static_cast<const W *>(L->W_downT), *xs = static_cast<const W *>(x);
    bool matrix = false;
    if constexpr (std::is_same<W, bf16>::value) {
        matrix = p.kind == ROWS_MATRIX;
        if (matrix) {
            // gate/up kernel, then the down projection over column slices, which leaves DOWN_RG partial outputs
            char *region = reinterpret_cast<char *>(w.ypart);
            float *hbuf = reinterpret_cast<float *>(region + split_h_offset(d, NB));
            int32_t *lst = reinterpret_cast<int32_t *>(region + split_list_offset(d, D, NB));
            hipLaunchKernelGGL((k_gate_up_mfma<NB, MODE>), dim3(ROWS_BLOCKS), dim3(ROWS_THREADS), p.lds, st, Wg, Wu, xs, B,
                               d, D, mask, idx_in, nnz_in, idx_out, nnz_out, w.nnz, p.max_chunk, p.min_chunk, L->flags,
                               hbuf, lst);
            hipLaunchKernelGGL((k_down_slices<NB, MODE == ROWS_DENSE>), dim3(d / DS_SW, DOWN_RG), dim3(DS_THREADS), 0, st,
                               Wd, lst, MODE == ROWS_DENSE ? nullptr : w.nnz, D, D, d, hbuf, DOWN_MIN_CHUNK, w.ypart);
        }
    }
    if (matrix) {
        // launched above
    } else if (p.kind == ROWS_SEQ) {
        hipLaunchKernelGGL((k_rows_seq<W, NB, MODE>), dim3(ROWS_BLOCKS), dim3(ROWS_THREADS), p.lds, st, Wg, Wu, Wd, xs, B,
                           d, D, mask, idx_in, nnz_in, idx_out, nnz_out, w.nnz, p.max_chunk, p.min_chunk, L->flags,
                           w.ypart);
    } else {
        hipLaunchKernelGGL((k_rows<W, NB, MODE>), dim3(ROWS_BLOCKS), dim3(ROWS_THREADS), p.lds, st, Wg, Wu, Wd, xs, B, d,
                           D, mask, idx_in, nnz_in, idx_out, nnz_out, w.nnz, p.max_chunk, p.min_chunk, L->flags, w.ypart);
    }
    if (y != nullptr) {
        const int vpt = d / 4;
        const int blocks = B * ((vpt + RED_COLS - 1) / RED_COLS);
        hipLaunchKernelGGL(k_reduce_y, dim3(blocks), dim3(RED_COLS * RED_SEGS), 0, st, w.ypart,
                           MODE == ROWS_DENSE ? nullptr : w.nnz, D, D, p.split ? DOWN_RG : ROWS_BLOCKS,
                           p.split ? DOWN_MIN_CHUNK : p.min_chunk, NB, B, d, y);
    }
    return hip_status(hipSuccess);
}

template <typename W, int NB>
bool tsum_needed(const svdp_layer *L)
{
    // finish t once instead of in every score block (the vector score kernel splits the partial
    // list over threads through LDS, which costs more than a launch from 4 tokens up)
    return NB >= 4 && L->d > XP_ROWS && !scores_on_matrix<W, NB>(L);
}

template <typename W, int NB>
svdp_status run_predict(const svdp_layer *L, const void *x, int B, float *s, uint64_t *mask, const Workspace &w,
                        hipStream_t st, const GlueArgs *glue)
{
    int nt = 0;
    svdp_status e = launch_xP<W, NB>(L, x, B, w.tpart, &nt, st, glue);
    if (e != SVDP_OK) return e;
    if (tsum_needed<W, NB>(L)) {
        const int count = NB * L->r;
        float *t = w.tpart + (size_t)XP_MAX_BLOCKS * NB * L->r;
        hipLaunchKernelGGL(k_tsum, dim3((count + 255) / 256), dim3(256), 0, st, w.tpart, nt, count, t);
        e = hip_status(hipSuccess);
        if (e != SVDP_OK) return e;
        return launch_scores<W, NB>(L, t, 1, B, s, mask, st);
    }
    return launch_scores<W, NB>(L, w.tpart, nt, B, s, mask, st);
}

// The whole step: every LDS grant first (on failure nothing has been enqueued), then the launches.
svdp_status step_impl(const svdp_layer *L, const void *x, int B, float *y, uint64_t *mask_out, int32_t *idx_out,
                      int32_t *nnz_out, const Workspace &w, hipStream_t st, const GlueArgs *glue)
{
    return dispatch(L->wdtype, nb_of(B), [&](auto wt, auto nb) -> svdp_status {
        using W = typename decltype(wt)::type;
        constexpr int NB = decltype(nb)::value;
        if (!prepare_xP<W, NB>(L, glue != nullptr) || !prepare_scores<W, NB>(L) || !prepare_rows<W, NB, ROWS_MASK>(L))
            return SVDP_ERR_UNSUPPORTED;
        uint64_t *mask = mask_out ? mask_out : w.mask;
        const svdp_status e = run_predict<W, NB>(L, x, B, nullptr, mask, w, st, glue);
        if (e != SVDP_OK) return e;
        // with the glue, x is made by the first kernel (from x_prev = x) and the row kernel reads it from x_out
        const void *xr = glue != nullptr ? glue->x_out : x;
        return launch_rows<W, NB, ROWS_MASK>(L, xr, B, mask, nullptr, nullptr, idx_out, nnz_out, w, y, st);
    });
}

// ---- the scratch buffer of svdp_ffn_step_static: one array per device, in the library's image ----
__device__ __align__(256) unsigned char g_static_scratch[SVDP_STATIC_SCRATCH_BYTES];

std::mutex g_scratch_mutex;
std::atomic<void *> g_scratch_ptr[MAX_DEVICES];

// Address of the current device's copy of the array (looked up once per device).
void *static_scratch()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) {
        (void)hipGetLastError();
        return nullptr;
    }
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p != nullptr) return p;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    p = g_scratch_ptr[dev].load(std::memory_order_relaxed);
    if (p != nullptr) return p;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_scratch)) != hipSuccess || p == nullptr) {
        (void)hipGetLastError();
        return nullptr;
    }
    g_scratch_ptr[dev].store(p, std::memory_order_release);
    return p;
}

// ---- offline build with whitening (Alg. 1): fp64 work buffers and the Jacobi driver ----
struct WhitenWs {
    double *W64, *M, *Mt;       // [D][d], [D][d], [d][D]
    double *Xt;                 // [d][T]
    double *A0, *A1;            // [d][d] symmetric matrix, ping-pong
    double *V0, *V1;            // [d][d] eigenvectors as rows, ping-pong
    double *St;                 // [d][d]  S^T, S = the lower Cholesky factor of X^T X
    double *S;                  // [d][d]  S
    double *lamG;               // [d] eigenvalues by place
    double *invL, *invLt;       // [64][64] scratch; [d/64][64][64] transposed inverses of S's diagonal blocks
    int32_t *fail;              // set by the factorisation if X^T X is not positive definite
    double *Vr;                 // [r][d]
    double *out64;              // [max(D, d)][r]
    double *Uall, *rowsums, *sums;     // [d/64][64][64] strip transforms; norms
    int32_t *sel;               // [r]
    size_t bytes;
};

WhitenWs carve_whiten(void *base, int d, int D, int T, int r)
{
    WhitenWs w;
    char *p = static_cast<char *>(base);
    size_t off = 0;
    auto take = [&](size_t n_doubles) {
        double *q = reinterpret_cast<double *>(p + off);
        off += align_up(n_doubles * 8);
        return q;
    };
    const size_t dd = (size_t)d * d, Dd = (size_t)D * d;
    w.W64 = take(Dd);
    w.M = take(Dd);
    w.Mt = take(Dd);
    w.Xt = take((size_t)d * T);
    w.A0 = take(dd);
    w.A1 = take(dd);
    w.V0 = take(dd);
    w.V1 = take(dd);
    w.St = take(dd);
    w.S = take(dd);
    w.lamG = take(d);
    w.invL = take(64 * 64);
    w.invLt = take((size_t)d * 64);
    w.fail = reinterpret_cast<int32_t *>(take(32));
    w.Vr = take((size_t)r * d);
    w.out64 = take((size_t)(D > d ? D : d) * r);
    w.Uall = take((size_t)d * 64);
    w.rowsums = take((size_t)2 * d);
    w.sums = take(2);
    w.sel = reinterpret_cast<int32_t *>(p + off);
    off += align_up((size_t)r * 4);
    w.bytes = off;
    return w;
}

inline dim3 grid1(size_t n) { return dim3((unsigned)((n + 255) / 256)); }

// C = A B^T, or with Cin: C = Cin - A B^T (C and Cin different memory)
void dgemm_nt(const double *A, int lda, const double *Bm, int ldb, double *C, int ldc, int M, int N, int K, hipStream_t st,
              const double *Cin = nullptr, int ldcin = 0)
{
    if (M <= 0 || N <= 0) return;
    hipLaunchKernelGGL(k_dgemm_nt, dim3((N + DG_BN - 1) / DG_BN, (M + DG_BM - 1) / DG_BM), dim3(256), 0, st, A, lda, Bm, ldb,
                       C, ldc, M, N, K, Cin, ldcin);
}

// L (lower, [n][n], zero above the diagonal) with L L^T = C; T: scratch [n][n]; invLt: [n/64][64][64], the
// transposed inverses of L's diagonal blocks; invL: scratch [64][64]; scale: device double; fail: device int,
// set to 1 if C is not positive definite to working precision (then L is not to be used).
void cholesky_blocked(const double *C, double *L, double *T, int n, double *invL, double *invLt, double *scale, int *fail,
                      hipStream_t st)
{
    const int nb = n / CH_B;
    hipLaunchKernelGGL(k_max_diag, dim3(1), dim3(256), 0, st, C, n, scale);
    for (int k = 0; k < nb; ++k) {
        const size_t row0 = (size_t)k * CH_B * n, diag = row0 + (size_t)k * CH_B;
        // T[k:, k] = C[k:, k] - L[k:, :k] L[k, :k]^T   (K = 0 for the first block column: a copy)
        dgemm_nt(L + row0, n, L + row0, n, T + diag, n, n - k * CH_B, CH_B, k * CH_B, st, C + diag, n);
        hipLaunchKernelGGL(k_chol_diag, dim3(1), dim3(256), 0, st, T, L, n, diag, scale, 1e-13, invL,
                           invLt + (size_t)k * CH_B * CH_B, fail);
        // L[k+1:, k] = T[k+1:, k] Lkk^-T
        dgemm_nt(T + diag + (size_t)CH_B * n, n, invL, CH_B, L + diag + (size_t)CH_B * n, n, n - (k + 1) * CH_B, CH_B, CH_B,
                 st);
    }
    hipLaunchKernelGGL(k_zero_upper_blocks, grid1((size_t)n * n), dim3(256), 0, st, L, n);
}

// Bout [r][n] = Bin [r][n] L^-1 for the lower-triangular L given as Lt = L^T [n][n] and the transposed inverses of
// its diagonal blocks: block back-substitution from the last block column to the first.  tmp: scratch [r][64].
void solve_right_lower(const double *Bin, double *Bout, int r, int n, const double *Lt, const double *invLt, double *tmp,
                       hipStream_t st)
{
    const int nb = n / CH_B;
    for (int i = nb - 1; i >= 0; --i) {
        const int c0 = i * CH_B, rest = n - (i + 1) * CH_B;
        // tmp = Bin[:, i] - Bout[:, i+1:] L[i+1:, i]      (L[k][c0 + a] = Lt[c0 + a][k])
        dgemm_nt(Bout + c0 + CH_B, n, Lt + (size_t)c0 * n + c0 + CH_B, n, tmp, CH_B, r, CH_B, rest, st, Bin + c0, n);
        // Bout[:, i] = tmp Lii^-1
        dgemm_nt(tmp, CH_B, invLt + (size_t)i * CH_B * CH_B, CH_B, Bout + c0, n, r, CH_B, CH_B, st);
    }
}

// Eigen-decomposition of the symmetric matrix in *A (n x n, n % 64 == 0) by block Jacobi sweeps.  On return
// *A / *V point at the buffers holding the (numerically) diagonal matrix and the eigenvectors as rows, lam[i]
// (device) = (*A)[i][i].  Uall: n/64 matrices of 64 x 64.  Synchronises the stream once per sweep (the
// convergence figure is read on the host).
svdp_status jacobi_eigh(double **A, double **Aalt, double **V, double **Valt, int n, double *Uall, double *rowsums,
                        double *sums, double *lam, double tol, int max_sweeps, int *sweeps_out, hipStream_t st)
{
    const size_t lds_solve = (size_t)2 * BJ_S * BJ_LD * 8, lds_two = (size_t)2 * BJ_S * BJ_LD * 8,
                 lds_one = lds_two;
    if (!grant_lds<k_bjacobi_solve>(lds_solve) || !grant_lds<k_bjacobi_apply<true>>(lds_two) ||
        !grant_lds<k_bjacobi_apply<false>>(lds_one))
        return SVDP_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(k_identity, grid1((size_t)n * n), dim3(256), 0, st, *V, n);
    const int strips = n / BJ_S, rounds = n / BJ_B > 2 ? n / BJ_B - 1 : 1;
    const int ct = strips >= 32 ? 4 : 1, cgrid = (strips + ct - 1) / ct;      // column tiles per block
    int sweep = 0;
    for (;; ++sweep) {
        hipLaunchKernelGGL(k_jacobi_norms, dim3(n), dim3(256), 0, st, *A, n, rowsums);
        hipLaunchKernelGGL(k_jacobi_norms_finish, dim3(1), dim3(256), 0, st, rowsums, n, *A, sums, lam);
        double h[2] = {0.0, 0.0};
        if (hipMemcpyAsync(h, sums, sizeof(h), hipMemcpyDeviceToHost, st) != hipSuccess ||
            hipStreamSynchronize(st) != hipSuccess) {
            (void)hipGetLastError();
            return SVDP_ERR_HIP;
        }
        if (!(h[1] == h[1]) || h[0] <= tol * tol * h[1] || sweep >= max_sweeps) break;
        for (int round = 0; round < rounds; ++round) {
            hipLaunchKernelGGL(k_bjacobi_solve, dim3(strips), dim3(BJ_SOLVE_THREADS), lds_solve, st, *A, n, Uall);
            hipLaunchKernelGGL(k_bjacobi_apply<true>, dim3(cgrid, strips), dim3(256), lds_two, st, *A, Uall, n, ct, *Aalt);
            hipLaunchKernelGGL(k_bjacobi_apply<false>, dim3(cgrid, strips), dim3(256), lds_one, st, *V, Uall, n, ct, *Valt);
            std::swap(*A, *Aalt);
            std::swap(*V, *Valt);
        }
    }
    if (sweeps_out != nullptr) *sweeps_out = sweep;
    return hip_status(hipSuccess);
}

template <typename W>
svdp_status whiten_impl(const void *W_gate, const void *X, int d, int D, int T, int r, float *P, float *Q, float *sigma,
                        int32_t *sweeps, const WhitenWs &w, hipStream_t st)
{
    const W *Wg = static_cast<const W *>(W_gate), *Xs = static_cast<const W *>(X);
    const double tol = 1e-11;          // off-diagonal Frobenius norm relative to the matrix's
    const int max_sweeps = 24;
    std::vector<double> lam(d);
    std::vector<int32_t> order(d);

    // second moments C = X^T X  (d x d) and its Cholesky factor S (lower, S S^T = C)
    hipLaunchKernelGGL((k_transpose_to_f64<W>), dim3((d + 31) / 32, (T + 31) / 32), dim3(256), 0, st, Xs, T, d, w.Xt);
    dgemm_nt(w.Xt, T, w.Xt, T, w.A0, d, d, d, T, st);
    if (hipMemsetAsync(w.fail, 0, 4, st) != hipSuccess) {
        (void)hipGetLastError();
        return SVDP_ERR_HIP;
    }
    cholesky_blocked(w.A0, w.S, w.A1, d, w.invL, w.invLt, w.sums, w.fail, st);
    int32_t failed = 0;
    if (hipMemcpyAsync(&failed, w.fail, 4, hipMemcpyDeviceToHost, st) != hipSuccess ||
        hipStreamSynchronize(st) != hipSuccess) {
        (void)hipGetLastError();
        return SVDP_ERR_HIP;
    }
    // S needs C positive definite (more independent tokens than dimensions)
    if (failed != 0) return SVDP_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((k_transpose_to_f64<double>), dim3((d + 31) / 32, (d + 31) / 32), dim3(256), 0, st, w.S, d, d, w.St);

    // M = W_gate S, G = M^T M
    hipLaunchKernelGGL((k_to_f64<W>), grid1((size_t)D * d), dim3(256), 0, st, Wg, (size_t)D * d, w.W64);
    dgemm_nt(w.W64, d, w.St, d, w.M, d, D, d, d, st);
    hipLaunchKernelGGL((k_transpose_to_f64<double>), dim3((d + 31) / 32, (D + 31) / 32), dim3(256), 0, st, w.M, D, d, w.Mt);
    double *A = w.A0, *Aalt = w.A1, *V = w.V0, *Valt = w.V1;
    dgemm_nt(w.Mt, D, w.Mt, D, A, d, d, d, D, st);
    int sw2 = 0;
    svdp_status e = jacobi_eigh(&A, &Aalt, &V, &Valt, d, w.Uall, w.rowsums, w.sums, w.lamG, tol, max_sweeps, &sw2, st);
    if (e != SVDP_OK) return e;
    if (hipMemcpyAsync(lam.data(), w.lamG, (size_t)d * 8, hipMemcpyDeviceToHost, st) != hipSuccess ||
        hipStreamSynchronize(st) != hipSuccess) {
        (void)hipGetLastError();
        return SVDP_ERR_HIP;
    }
    // the r largest eigenvalues (= squared singular values of W S), largest first; ties by place
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return lam[a] > lam[b]; });
    if (hipMemcpyAsync(w.sel, order.data(), (size_t)r * 4, hipMemcpyHostToDevice, st) != hipSuccess) {
        (void)hipGetLastError();
        return SVDP_ERR_HIP;
    }
    // Q = A = M V_r
    hipLaunchKernelGGL(k_gather_rows, grid1((size_t)r * d), dim3(256), 0, st, V, w.sel, r, d, w.Vr);
    dgemm_nt(w.M, d, w.Vr, d, w.out64, r, D, r, d, st);
    hipLaunchKernelGGL(k_f64_to_f32, grid1((size_t)D * r), dim3(256), 0, st, w.out64, (size_t)D * r, Q);
    // B = V_r^T S^-1 (block back-substitution; V_r^T is w.Vr, rows = the chosen eigenvectors), P = B^T
    solve_right_lower(w.Vr, w.out64, r, d, w.St, w.invLt, w.Uall, st);
    hipLaunchKernelGGL((k_transpose_to_f64<double>), dim3((d + 31) / 32, (r + 31) / 32), dim3(256), 0, st, w.out64, r, d, w.M);
    hipLaunchKernelGGL(k_f64_to_f32, grid1((size_t)d * r), dim3(256), 0, st, w.M, (size_t)d * r, P);
    if (hipStreamSynchronize(st) != hipSuccess) {                 // order[] leaves scope: the copy above must be done
        (void)hipGetLastError();
        return SVDP_ERR_HIP;
    }
    if (sigma != nullptr)
        for (int k = 0; k < r; ++k) sigma[k] = (float)std::sqrt(std::max(lam[order[k]], 0.0));
    if (sweeps != nullptr) {
        sweeps[0] = 0;              // the factor of the second moments is a Cholesky factor: no sweeps
        sweeps[1] = sw2;
    }
    return hip_status(hipSuccess);
}

}  // namespace

extern "C" {

size_t svdp_workspace_bytes(const svdp_layer *layer, int32_t max_batch)
{
    if (layer == nullptr || bad_batch(max_batch)) return 0;
    if (check_shape(layer->d, layer->D, layer->r, layer->wdtype) != SVDP_OK) return 0;
    if ((layer->flags & ~ALL_FLAGS) ||
        ((layer->flags & SVDP_FLAG_ENGINE_VECTOR) && (layer->flags & SVDP_FLAG_ENGINE_MATRIX)))
        return 0;
    if (!layer_fits(layer, nb_of(max_batch))) return 0;
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
    return dispatch(layer->wdtype, nb_of(B), [&](auto wt, auto nb) -> svdp_status {
        using W = typename decltype(wt)::type;
        constexpr int NB = decltype(nb)::value;
        if (!prepare_xP<W, NB>(layer, false) || !prepare_scores<W, NB>(layer)) return SVDP_ERR_UNSUPPORTED;
        return run_predict<W, NB>(layer, x, B, s, nullptr, w, static_cast<hipStream_t>(stream), nullptr);
    });
}

svdp_status svdp_compact(const float *s, int32_t B, int32_t D, uint64_t *mask, int32_t *idx, int32_t *nnz,
                         void *ws, size_t ws_bytes, void *stream)
{
    (void)ws;
    (void)ws_bytes;
    if (s == nullptr || mask == nullptr || idx == nullptr || nnz == nullptr || bad_batch(B) || D <= 0) return SVDP_ERR_INVALID_ARG;
    if (D % 64 != 0) return SVDP_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(k_mask_from_scores, dim3((D / 64 + 3) / 4), dim3(256), 0, st, s, B, D, mask);
    const svdp_status e = hip_status(hipSuccess);
    if (e != SVDP_OK) return e;
    hipLaunchKernelGGL(k_compact_scan, dim3(1), dim3(SCAN_THREADS), 0, st, mask, D / 64, idx, nnz);
    return hip_status(hipSuccess);
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
    return dispatch(layer->wdtype, nb_of(B), [&](auto wt, auto nb) -> svdp_status {
        using W = typename decltype(wt)::type;
        constexpr int NB = decltype(nb)::value;
        if (!prepare_rows<W, NB, ROWS_LIST>(layer)) return SVDP_ERR_UNSUPPORTED;
        return launch_rows<W, NB, ROWS_LIST>(layer, x, B, nullptr, idx, nnz, nullptr, nullptr, w, y,
                                             static_cast<hipStream_t>(stream));
    });
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
    return dispatch(layer->wdtype, nb_of(B), [&](auto wt, auto nb) -> svdp_status {
        using W = typename decltype(wt)::type;
        constexpr int NB = decltype(nb)::value;
        if (!prepare_rows<W, NB, ROWS_DENSE>(layer)) return SVDP_ERR_UNSUPPORTED;
        return launch_rows<W, NB, ROWS_DENSE>(layer, x, B, nullptr, nullptr, nullptr, nullptr, nullptr, w, y,
                                              static_cast<hipStream_t>(stream));
    });
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
    return step_impl(layer, x, B, y, mask_out, idx_out, nnz_out, w, static_cast<hipStream_t>(stream), nullptr);
}

svdp_status svdp_ffn_step_static(const svdp_layer *layer, const void *x, int32_t B, float *y, uint64_t *mask_out,
                                 int32_t *idx_out, int32_t *nnz_out, void *stream)
{
    svdp_status st = check_layer(layer, true, true);
    if (st != SVDP_OK) return st;
    if (x == nullptr || y == nullptr || bad_batch(B) || !aligned16(x) || !aligned16(y)) return SVDP_ERR_INVALID_ARG;
    if (!layer_fits(layer, nb_of(B))) return SVDP_ERR_UNSUPPORTED;
    // the size test comes first: a layer or batch beyond the array is refused whatever the device says
    if (carve(nullptr, layer->d, layer->D, layer->r, nb_of(B)).bytes > (size_t)SVDP_STATIC_SCRATCH_BYTES)
        return SVDP_ERR_WORKSPACE;
    void *scratch = static_scratch();
    if (scratch == nullptr) return SVDP_ERR_HIP;
    Workspace w;
    st = check_ws(layer, B, scratch, (size_t)SVDP_STATIC_SCRATCH_BYTES, &w);
    if (st != SVDP_OK) return st;
    return step_impl(layer, x, B, y, mask_out, idx_out, nnz_out, w, static_cast<hipStream_t>(stream), nullptr);
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
    return step_impl(layer, x_prev, B, y, mask_out, idx_out, nnz_out, w, static_cast<hipStream_t>(stream), &glue);
}

svdp_status svdp_active_rows(const svdp_layer *layer, const void *x, int32_t B, const uint64_t *mask, float *y,
                             void *ws, size_t ws_bytes, void *stream)
{
    svdp_status st = check_layer(layer, false, true);
    if (st != SVDP_OK) return st;
    if (x == nullptr || mask == nullptr || bad_batch(B) || !aligned16(x) || (y != nullptr && !aligned16(y)))
        return SVDP_ERR_INVALID_ARG;
    Workspace w;
    st = check_ws(layer, B, ws, ws_bytes, &w);
    if (st != SVDP_OK) return st;
    return dispatch(layer->wdtype, nb_of(B), [&](auto wt, auto nb) -> svdp_status {
        using W = typename decltype(wt)::type;
        constexpr int NB = decltype(nb)::value;
        if (!prepare_rows<W, NB, ROWS_MASK>(layer)) return SVDP_ERR_UNSUPPORTED;
        hipStream_t hs = static_cast<hipStream_t>(stream);
        return launch_rows<W, NB, ROWS_MASK>(layer, x, B, mask, nullptr, nullptr, nullptr, nullptr, w, y, hs);
    });
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
    else
        hipLaunchKernelGGL(k_stack_glue<bf16>, dim3(1), dim3(256), 0, st, static_cast<const bf16 *>(x), y, shift, d,
                           eps, static_cast<bf16 *>(x_next));
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

int64_t svdp_calib_need(double sparsity, int32_t D, int32_t T)
{
    if (D < 1 || T < 1 || std::isnan(sparsity)) return -1;
    const int64_t all = (int64_t)D * (int64_t)T;
    const double target = sparsity * (double)D * (double)T;         // (sparsity * D) * T, in double
    if (!(target > 0.0)) return 0;
    if (target >= (double)all) return all;
    int64_t n = (int64_t)std::ceil(target);
    while (n > 0 && (double)(n - 1) >= target) --n;
    return n < 0 ? 0 : n > all ? all : n;
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
    if (!grant_lds<k_calib_sort>(lds)) return SVDP_ERR_UNSUPPORTED;
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

size_t svdp_whiten_workspace_bytes(int32_t d, int32_t D, int32_t T, int32_t r)
{
    if (d < 64 || d % 64 != 0 || D < 1 || T < d || r < 1 || r > d) return 0;
    return carve_whiten(nullptr, d, D, T, r).bytes;
}

svdp_status svdp_whiten_factors(const void *W_gate, const void *X, int32_t d, int32_t D, int32_t T, int32_t r,
                                int32_t wdtype, float *P, float *Q, float *sigma, int32_t *sweeps, void *ws,
                                size_t ws_bytes, void *stream)
{
    if (W_gate == nullptr || X == nullptr || P == nullptr || Q == nullptr || d < 1 || D < 1 || T < 1 || r < 1)
        return SVDP_ERR_INVALID_ARG;
    if (wdtype != SVDP_F32 && wdtype != SVDP_BF16) return SVDP_ERR_UNSUPPORTED;
    if (d < 64 || d % 64 != 0 || T < d || r > d) return SVDP_ERR_UNSUPPORTED;
    if (ws == nullptr || (reinterpret_cast<uintptr_t>(ws) & (ALIGN - 1))) return SVDP_ERR_WORKSPACE;
    const WhitenWs w = carve_whiten(ws, d, D, T, r);
    if (ws_bytes < w.bytes) return SVDP_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (wdtype == SVDP_F32) return whiten_impl<float>(W_gate, X, d, D, T, r, P, Q, sigma, sweeps, w, st);
    return whiten_impl<bf16>(W_gate, X, d, D, T, r, P, Q, sigma, sweeps, w, st);
}

const char *svdp_version(void) { return "0.5"; }

}  // extern "C"
