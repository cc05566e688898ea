// Host side of the C ABI declared in include/psgd.h: argument checks, launch planning, workspace
// layout, pointer-table upload, and the sequences of batched launches that make up one SSP-Comp
// step, one SVD-Comp step (Algorithm 1) and the reconstruction.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/psgd.h"
#include "psgd_dev.h"

namespace psgd {
hipError_t launch_prod(int nb, int planes, bool colmode, bool form, bool lazy, bool onew, const LayerDev* layers,
                       const int* ids, int n_ids, int max_tiles, int out_role, int epi, int gate, hipStream_t st);
hipError_t launch_form_row(int nb, int planes, bool gbf, bool onew, int lazy, const LayerDev* layers, const int* ids,
                           int n_ids, int max_tiles, int out_role, int epi, int nt_m, const int* xtab, int xstride,
                           int xtiles, hipStream_t st);
bool form_row_supported(int nb, int planes, bool gbf, bool onew, bool lazy);
hipError_t launch_col_prod(int nb, int planes, const LayerDev* layers, const int* ids, int n_ids, int max_tiles,
                           int out_role, int epi, int gate, int nt_s, const int* xtab, int xstride, int xtiles,
                           hipStream_t st);
bool col_prod_supported(int nb, int planes);
hipError_t launch_row_prod(int nb, int planes, const LayerDev* layers, const int* ids, int n_ids, int max_tiles,
                           int out_role, int epi, int gate, int nt_s, const int* xtab, int xstride, int xtiles,
                           hipStream_t st);
bool row_prod_supported(int nb, int planes);
hipError_t launch_outer(int nb, int planes, bool decomp, bool form, bool kept, const LayerDev* layers, const int* ids,
                        int n_ids, int max_tiles, void* const* outs, int out_bf16, hipStream_t st);
hipError_t launch_max_iterations(const LayerDev* layers, const int* ids, int n_ids, int mx, int* out, hipStream_t st);
hipError_t launch_msgd(int nb, int planes, const LayerDev* layers, const int* ids, int n_ids, int max_tiles,
                       float* const* moms, float* const* xs, float mu, float eta, bool kept, hipStream_t st);
hipError_t launch_adam(int nb, int planes, const LayerDev* layers, const int* ids, int n_ids, int max_tiles,
                       float* const* m1s, float* const* m2s, float* const* xs, const float* coef, bool kept,
                       hipStream_t st);
hipError_t launch_finish(bool colmode, int form, const LayerDev* layers, const int* ids, int n_ids, int max_blocks,
                         int cp, int out_role, int epi, int gate, int chol_gate, int a2gate, double tol2, int w,
                         int local_ok, hipStream_t st);
hipError_t launch_thin_gram(const LayerDev* layers, const int* ids, int n_ids, int max_blocks, int role, int cp,
                            int gate, hipStream_t st);
hipError_t launch_pack(const LayerDev* layers, const int* ids, int n_ids, int max_lenP, int role_a, int role_b,
                       int cp, int which, hipStream_t st);
hipError_t launch_chol(const LayerDev* layers, const int* ids, int n_ids, int w, int role, double tol2, int pass,
                       int slot_rows, int gate, int a2gate, int local_ok, int after_finish, hipStream_t st);
hipError_t launch_slot_sum(const LayerDev* layers, const int* ids, int n_ids, int max_len, int role, int slot_rows,
                           int group, int gate, hipStream_t st);
hipError_t launch_apply(const LayerDev* layers, const int* ids, int n_ids, int max_lenP, int w_in, int w_out,
                        int src_role, int dst_role, int mode, int cp, int gate, int a2gate, double tol2,
                        bool small, int which, hipStream_t st);
hipError_t launch_init_block(const LayerDev* layers, const int* ids, int n_ids, int max_len, int w, int dst_role,
                             int src_role, int warm, uint32_t seed, hipStream_t st);
hipError_t launch_jacobi(const LayerDev* layers, const int* ids, int n_ids, int w, int role, float* sigma_out,
                         hipStream_t st);
hipError_t launch_copy(void* dst, const void* src, size_t n_bytes, hipStream_t st);
hipError_t launch_put(void* dst, const void* src_host, size_t bytes, hipStream_t st);
hipError_t launch_clear_status(const LayerDev* layers, const int* ids, int n_ids, hipStream_t st);
enum ApplyModeHost { APPLY_PASS1 = 1, APPLY_PASS2 = 2, APPLY_RITZ = 3 };
}  // namespace psgd

using namespace psgd;

namespace {

constexpr int kMaxWidth = 192;      // widest thin block (packed Cholesky factor and product operands must fit in LDS)
constexpr int kTargetTiles = 1024;  // workgroups per forming-pass launch we try to reach by splitting the reduction
constexpr int kTargetTilesPlain = 512;   // ... per launch of a product that only reads M: half as many, twice as long-lived
                                         // (config 2: pass 2a 20.4 -> 18.6 us, its refresh step 1.00 -> 0.96 ms)
constexpr int kTargetTilesWide = 256;    // ... at thin widths of 64 and more (see choose_split)
constexpr int kMaxSplit = 32;
constexpr int64_t kMaxLd = (int64_t)1 << 23;   // largest leading dimension (elements)

inline int64_t round_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

struct Plan {            // host copy of what a layer needs
    psgd_layer_desc d;
    int transposed;
    int rowsP, colsP;
    int m, n;
};

struct Lists {
    std::vector<int> norm, tr;   // layer ids stored row-major as logical / as the transpose
};

}  // namespace

struct psgd_ctx {
    uint64_t serial = 0;     // unique per context (the built-in workspace remembers whose contents it holds)
    int n_layers = 0;
    int n_workers = 0;
    psgd_options opt{};
    std::vector<Plan> plan;
    Lists lists;
    int rmax = 0;
    int cpc = 0;     // packed width of the compress step: 32 * ceil(rmax / 32)
    int wz = 0;      // block width of the subspace iteration (r + oversampling, multiple of 8)
    int cpz = 0;     // its packed width: wz rounded up to a multiple of 32
    int cpmax = 0;   // max(cpc, cpz)
    int planes = 2;  // bf16 planes per fp32 operand of the MFMA products (2: 3 products, 3: 6 products)
    bool reform_m = false;   // SSP step forms M = mean G + E in every pass instead of storing it over E
    bool lazy = false;       // deferred residual: E_{t+1} = M - P~ Q^T is applied by the next forming pass
    bool lazy_tr = false;    // ... also for the layers stored with rows < cols (column-mode forming pass: width 32 only)
    bool pending = false;    // the E buffers of the row-major layers hold M_t, their residual is still owed
    double kernel_bytes[3] = {0.0, 0.0, 0.0};   // algorithmic bytes of the three streaming kernels of one SSP step
    // batched splits
    int split_row_b = 1, split_col_b = 1;       // products that read M
    int split_row_bf = 1, split_col_bf = 1;     // forming passes
    int split_row_v2 = 1;                       // forming pass on 32 x 256 tiles (form_row_kernel)
    int split_col_v2 = 1;                       // column-mode product on 32 x 256 tiles (col_prod_kernel)
    int grad_kind = 0;                          // 1: every layer has fp32 gradients, 2: every layer bf16, 0: mixed
    bool nt_m = false;                          // the row-major layers' M is too large to be found in a cache again
    // XCD table of the forming pass on 32 x 256 tiles (see form_row_kernel): 16 rows of xstride ints; built when the
    // row-major layers are many enough to be dealt evenly to the 8 XCDs
    std::vector<int> hXtab, hXtabC;             // (forming pass; column-mode product: other tile counts)
    int xstride = 0, xtiles = 0, xtiles_c = 0;
    size_t off_xtab = 0, off_xtab_c = 0;
    // workspace layout (byte offsets)
    // The gradient pointer table and the layer descriptors (which point into it) exist kGSlots times: a caller
    // that rotates between a few sets of gradient buffers finds its table already on the device.
    static constexpr int kGSlots = 4;
    size_t off_layers_s[kGSlots] = {}, off_gtab_s[kGSlots] = {};
    size_t off_iters = 0;            // one int: most iterations any layer's next refresh will run
    size_t off_ids = 0, off_outs = 0, off_moms = 0, off_m2s = 0, off_xs = 0, off_single_part[2] = {0, 0};
    std::vector<size_t> off_layer;   // start of each layer's private region
    size_t ws_bytes = 0;
    // cached tables
    void* bound_ws = nullptr;
    void* outs_ws = nullptr;     // workspace that holds the current table of decompress outputs
    void* msgd_ws = nullptr;     // ... and of the momentum and weight buffers of psgd_decompress_msgd / _adam
    void* m2_ws = nullptr;       // ... and of the second-moment buffers of psgd_decompress_adam
    void* factors_ws = nullptr;  // workspace whose row-major operand copies are the P~, Q of the last compress call
    bool factors_kept = false;   // ... a call with a deferred residual: in the layers that defer they are the kept copies
    bool tables_valid = false;
    std::vector<const void*> hG;                       // the caller's current table
    std::vector<const void*> hGs[kGSlots];             // what each device slot holds (empty: nothing yet)
    int cur_slot = 0, next_victim = 0;
    std::vector<float*> hE, hQ, hP;
    std::vector<void*> hOut;
    std::vector<float*> hMom, hM2, hX;
    std::vector<int> hIds;
    std::vector<LayerDev> hLayers;   // n_layers + 1 (last = scratch descriptor of single-layer calls)
    int last_hip = 0;
    double algo_bytes = 0.0;
    // The per-layer iteration counts of the next refresh are decided on the device.  Their maximum is copied to
    // pinned host memory after every batched refresh (asynchronously, with an event behind it); a later refresh
    // that finds the event complete launches only that many iterations instead of the whole budget.
    // A copy describes the counts as the refresh it was enqueued behind left them: it is used by the very next
    // batched refresh on the same workspace and by no other (refresh_seq), and not at all if something else has
    // changed the counts in between (iters_gen: a single-layer psgd_refresh, another workspace, a reset).  The
    // copies go through a small ring of pinned words, so that a loop that runs ahead of the GPU (tau = 1) still
    // has a free word for every refresh; when none is free the next refresh launches the whole budget.  Whatever
    // the host launches, the device never runs an iteration that was not launched (see gate_open).
    static constexpr int kIterSlots = 4;
    struct IterFetch { int* h = nullptr; hipEvent_t ev = nullptr; bool pending = false; int gen = 0; uint64_t seq = 0; };
    IterFetch fetch[kIterSlots];
    bool fetch_ready = false;        // pinned words and events exist
    bool fetch_failed = false;       // ... could not be created: every refresh launches the whole budget
    int fetch_last = -1;             // slot of the copy enqueued behind the last batched refresh (-1: none)
    uint64_t refresh_seq = 0;        // batched refreshes run so far
    int iters_gen = 0;
    // optional timing of the three streaming kernels with event pairs on the caller's stream
    bool prof_on = false;
    int prof_mask = (1 << PSGD_PROF_TAGS) - 1;   // which of the tagged launches are timed
    std::vector<hipEvent_t> prof_ev;      // pairs (start, stop)
    std::vector<int> prof_tag;            // tag of each pair
    size_t prof_used = 0;                 // pairs recorded so far
};

namespace {

int fail_hip(psgd_ctx* c, hipError_t e) {
    c->last_hip = (int)e;
    return PSGD_E_HIP;
}

#define PSGD_TRY(expr)                                   \
    do {                                                 \
        hipError_t e__ = (expr);                         \
        if (e__ != hipSuccess) return fail_hip(ctx, e__); \
    } while (0)

struct LayerRegion {
    size_t part[2], pack[2][6], lzf[2][3], z[2], gram, tmat, eval, status, end;
};

// byte layout of one layer's private workspace region, relative to its start
LayerRegion layer_region(const psgd_ctx* c, const Plan& p) {
    LayerRegion R{};
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = (size_t)round_up((int64_t)(o + bytes), 256); return at; };
    const int lenP[2] = {p.rowsP, p.colsP};
    int split[2] = {c->split_row_b > c->split_row_bf ? c->split_row_b : c->split_row_bf,
                    c->split_col_b > c->split_col_bf ? c->split_col_b : c->split_col_bf};
    if (c->split_row_v2 > split[0]) split[0] = c->split_row_v2;
    if (c->split_col_v2 > split[1]) split[1] = c->split_col_v2;
    for (int s = 0; s < 2; ++s) R.part[s] = take((size_t)split[s] * lenP[s] * c->wz * sizeof(float));
    for (int s = 0; s < 2; ++s)
        for (int k = 0; k < 2 * c->planes; ++k) R.pack[s][k] = take((size_t)lenP[s] * c->cpmax * sizeof(bf16_t));
    if (c->lazy && (!p.transposed || c->lazy_tr))
        for (int s = 0; s < 2; ++s)
            for (int k = 0; k < c->planes; ++k) R.lzf[s][k] = take((size_t)lenP[s] * c->cpc * sizeof(bf16_t));
    const int len[2] = {(int)p.d.rows, (int)p.d.cols};
    for (int s = 0; s < 2; ++s) R.z[s] = take((size_t)len[s] * c->wz * sizeof(float));
    const size_t w2 = (size_t)(c->wz + 2) * (c->wz + 2);
    const int max_lenP = lenP[0] > lenP[1] ? lenP[0] : lenP[1];
    R.gram = take((size_t)(max_lenP / kGramRows2) * w2 * sizeof(double));
    R.tmat = take(w2 * sizeof(double));
    R.eval = take((size_t)(c->wz + 2) * sizeof(double));
    R.status = take(kStatusWords * sizeof(int));
    R.end = o;
    return R;
}

// PSGD_TARGET_TILES (environment, tuning knob): workgroups a product launch should reach; 0 = not set
int target_tiles_env() {
    static int v = -1;
    if (v < 0) {
        const char* e = std::getenv("PSGD_TARGET_TILES");
        v = e ? std::atoi(e) : 0;
        if (v < 1) v = 0;
    }
    return v;
}

// PSGD_FORM_ROW=0 (environment, measurement knob): forming passes use the 128 x 64 kernel everywhere
bool form_row_env() {
    static int v = -1;
    if (v < 0) {
        const char* e = std::getenv("PSGD_FORM_ROW");
        v = (e && e[0] == '0') ? 0 : 1;
    }
    return v == 1;
}

// Reduction split of a launch with `base_tiles` output blocks.  cp: packed width of the thin operand.  At widths
// of 64 and more one workgroup per compute unit is the target: the partial products that finish_kernel has to add
// up grow with the width, and the wide product kernels do not gain from more workgroups (4096 x 4096: the step at
// r = 64 takes 0.325 ms with 1024 workgroups, 0.302 with 256; at r = 128 0.514 and 0.473; at r = 16 and 32 it is
// the other way round).
int choose_split(int64_t base_tiles, int min_chunks, bool form, int cp) {
    int target = target_tiles_env();
    if (target == 0) target = cp >= 64 ? kTargetTilesWide : (form ? kTargetTiles : kTargetTilesPlain);
    else if (!form && target > kTargetTilesPlain) target = target / 2;
    if (base_tiles >= target) return 1;
    int64_t s = (target + base_tiles - 1) / base_tiles;
    if (s > kMaxSplit) s = kMaxSplit;
    if (s > min_chunks) s = min_chunks;
    if (s < 1) s = 1;
    return (int)s;
}

void build_layer_dev(psgd_ctx* c, char* ws, int l, int slot, LayerDev* out) {
    const Plan& p = c->plan[l];
    const LayerRegion R = layer_region(c, p);
    char* base = ws + c->off_layer[l];
    LayerDev L{};
    L.rows = (int)p.d.rows; L.cols = (int)p.d.cols; L.ld = p.d.ld; L.r = p.d.r; L.wz = c->wz;
    L.gdt = p.d.grad_dtype; L.n_workers = c->n_workers; L.transposed = p.transposed; L.planes = c->planes;
    L.rowsP = p.rowsP; L.colsP = p.colsP;
    L.split_row = c->split_row_b; L.split_col = c->split_col_b;
    L.split_row_f = c->split_row_bf; L.split_col_f = c->split_col_bf;
    L.split_row_v2 = c->split_row_v2;
    L.split_col_v2 = c->split_col_v2;
    L.G = reinterpret_cast<const void* const*>(ws + c->off_gtab_s[slot]) + (size_t)l * c->n_workers;
    L.S = c->hE.empty() ? nullptr : c->hE[l];
    const int side_p = side_of_role(p.transposed, ROLE_P), side_q = side_of_role(p.transposed, ROLE_Q);
    L.thin[ROLE_P] = ThinRef{c->hP.empty() ? nullptr : c->hP[l], p.d.r, p.d.r};
    L.thin[ROLE_Q] = ThinRef{c->hQ.empty() ? nullptr : c->hQ[l], p.d.r, p.d.r};
    L.thin[ROLE_ZP] = ThinRef{reinterpret_cast<float*>(base + R.z[side_p]), c->wz, c->wz};
    L.thin[ROLE_ZQ] = ThinRef{reinterpret_cast<float*>(base + R.z[side_q]), c->wz, c->wz};
    for (int s = 0; s < 2; ++s) {
        L.part[s] = reinterpret_cast<float*>(base + R.part[s]);
        for (int k = 0; k < c->planes; ++k) {
            L.pack[s].n[k] = reinterpret_cast<bf16_t*>(base + R.pack[s][2 * k]);
            L.pack[s].t[k] = reinterpret_cast<bf16_t*>(base + R.pack[s][2 * k + 1]);
            L.lzf[s][k] = (c->lazy && (!p.transposed || c->lazy_tr)) ? reinterpret_cast<bf16_t*>(base + R.lzf[s][k]) : nullptr;
        }
    }
    L.gram = reinterpret_cast<double*>(base + R.gram);
    L.tmat = reinterpret_cast<double*>(base + R.tmat);
    L.eval = reinterpret_cast<double*>(base + R.eval);
    L.status = reinterpret_cast<int*>(base + R.status);
    *out = L;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Refresh the cached host tables from the caller's; returns true when the device copy is stale.
template <typename T, typename U>
bool sync_table(std::vector<T>& cache, U const* user, size_t n) {
    if (!user) return false;
    bool changed = cache.size() != n;
    if (changed) cache.assign(n, nullptr);
    for (size_t i = 0; i < n; ++i)
        if (cache[i] != (T)user[i]) { cache[i] = (T)user[i]; changed = true; }
    return changed;
}

int check_table(const void* const* tab, size_t n) {
    if (!tab) return PSGD_E_INVALID_ARG;
    for (size_t i = 0; i < n; ++i) {
        if (!tab[i]) return PSGD_E_INVALID_ARG;
        if (!aligned16(tab[i])) return PSGD_E_ALIGN;
    }
    return PSGD_OK;
}

// Whether work put on `st` is being recorded into a graph instead of executed.
static bool is_capturing(hipStream_t st) {
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    const bool yes = hipStreamIsCapturing(st, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone;
    (void)hipGetLastError();
    return yes;
}

// Upload what has changed: the layer descriptors and id lists (new workspace, or new E/Q/P
// pointers) and/or the table of gradient pointers.  Stream-ordered, so launches already queued keep
// seeing the old tables.
int upload_tables(psgd_ctx* ctx, void* workspace, hipStream_t st, bool desc_changed, bool g_changed) {
    char* ws = reinterpret_cast<char*>(workspace);
    const bool fresh = !ctx->tables_valid || ctx->bound_ws != workspace;
    const int nl = ctx->n_layers;
    if (fresh || desc_changed || g_changed) {
        // Under stream capture nothing may be uploaded: a copy node would read this context's host arrays again at
        // every replay, and the clearing of a new workspace's status words would become a memset node.  The one
        // thing that is allowed to differ from the last eager call is which of the gradient tables already on the
        // device is used.
        bool slot_known = false;
        for (int k = 0; k < psgd_ctx::kGSlots; ++k) slot_known |= !ctx->hG.empty() && ctx->hGs[k] == ctx->hG;
        const bool upload = fresh || desc_changed || (g_changed && !ctx->hG.empty() && !slot_known);
        if (upload && is_capturing(st)) {
            ctx->tables_valid = false;      // the host copies are ahead of the device now: upload all next time
            return PSGD_E_CAPTURE;
        }
    }
    // (tables go to the device as kernel arguments, launch_put: the host arrays are free again when it returns)
    if (fresh) ctx->iters_gen++;   // the iteration counts live in the workspace: a bound fetched from another one is void
    if (fresh || desc_changed) {
        ctx->hLayers.resize(nl + 1);
        for (int slot = 0; slot < psgd_ctx::kGSlots; ++slot) {
            for (int l = 0; l < nl; ++l) build_layer_dev(ctx, ws, l, slot, &ctx->hLayers[l]);
            ctx->hLayers[nl] = ctx->hLayers[0];
            PSGD_TRY(launch_put(ws + ctx->off_layers_s[slot], ctx->hLayers.data(), (size_t)(nl + 1) * sizeof(LayerDev), st));
        }
    }
    if (fresh) {
        std::vector<int>& ids = ctx->hIds;
        ids.assign(3 * (size_t)nl + 1, 0);
        for (int l = 0; l < nl; ++l) ids[l] = l;
        for (size_t i = 0; i < ctx->lists.norm.size(); ++i) ids[nl + i] = ctx->lists.norm[i];
        for (size_t i = 0; i < ctx->lists.tr.size(); ++i) ids[2 * (size_t)nl + i] = ctx->lists.tr[i];
        ids[3 * (size_t)nl] = nl;   // id of the scratch descriptor
        PSGD_TRY(launch_put(ws + ctx->off_ids, ids.data(), ids.size() * sizeof(int), st));
        if (!ctx->hXtab.empty()) PSGD_TRY(launch_put(ws + ctx->off_xtab, ctx->hXtab.data(), ctx->hXtab.size() * sizeof(int), st));
        if (!ctx->hXtabC.empty()) PSGD_TRY(launch_put(ws + ctx->off_xtab_c, ctx->hXtabC.data(), ctx->hXtabC.size() * sizeof(int), st));
    }
    if (fresh)
        for (auto& v : ctx->hGs) v.clear();
    if ((fresh || g_changed) && !ctx->hG.empty()) {
        // a slot that already holds this table, else the next one in turn
        int slot = -1;
        for (int k = 0; k < psgd_ctx::kGSlots; ++k)
            if (ctx->hGs[k] == ctx->hG) slot = k;
        if (slot < 0) {
            slot = ctx->next_victim;
            ctx->next_victim = (ctx->next_victim + 1) % psgd_ctx::kGSlots;
            ctx->hGs[slot] = ctx->hG;
            PSGD_TRY(launch_put(ws + ctx->off_gtab_s[slot], ctx->hG.data(), ctx->hG.size() * sizeof(void*), st));
        }
        ctx->cur_slot = slot;
    }
    if (fresh) {
        // status words of a new workspace start at zero ("iterations the next refresh needs" = unknown); a fill
        // kernel, not a memset, so that nothing on this path would ever become a memset node of a graph
        PSGD_TRY(launch_clear_status(reinterpret_cast<const LayerDev*>(ws + ctx->off_layers_s[0]),
                                     reinterpret_cast<const int*>(ws + ctx->off_ids), nl, st));
    }
    ctx->bound_ws = workspace;
    ctx->tables_valid = true;
    return PSGD_OK;
}

struct Launcher {
    psgd_ctx* ctx;
    char* ws;
    hipStream_t st;
    const LayerDev* layers;
    const int *ids_all, *ids_norm, *ids_tr;
    int n_all, n_norm, n_tr;
    // geometry maxima over the layers addressed by this launcher
    int max_rows = 0, max_cols = 0, max_rowsP = 0, max_colsP = 0;
    int tiles_row = 0, tiles_col = 0, tiles_outer = 0, blocks_row = 0, blocks_col = 0;
    int tiles_row_f = 0, tiles_col_f = 0;       // forming passes
    int tiles_row_v2 = 0, split_row_v2 = 1;     // the forming pass on 32 x 256 tiles
    int tiles_col_v2 = 0, split_col_v2 = 1;     // the column-mode product on 32 x 256 tiles
    int split_row = 1, split_col = 1, split_row_f = 1, split_col_f = 1;
    hipError_t err = hipSuccess;
    bool prof_mute = false;   // the refresh's products are not part of the per-kernel timing
    bool capturing = false;   // the stream records into a graph: no event records
    int gate = -1;            // iteration gate of the launches inside the subspace iteration (-1: none)
    bool keep_e = false;      // FORM products leave E in place (M is formed again by the later passes)
    bool lazy_form = false;   // the forming pass of the row-major layers also applies their pending residual
    bool lazy_share = false;  // ... and the transposed operand copies of Q_{t-1} are what the step before left: they hold
                              // the kept Q, which the pass then need not read
    bool kept_packs = false;  // compress step with a deferred residual: the row-major operand copies of its P~ and Q go
                              // to the kept copies (fragment order) in the layers that have them
    bool use_form_row = true; // PSGD_FORM_ROW=0 (environment, measurement knob): the older 128 x 64 forming pass
    bool use_xtab = true;     // PSGD_XTAB=0 (environment, measurement knob): plain layer-by-layer launch order
    bool use_xtab_c = true;   // PSGD_XTAB_C=0 (likewise): the same for the column-mode product alone

    void note(hipError_t e) { if (err == hipSuccess && e != hipSuccess) err = e; }
    // event pair around one tagged launch group (only when profiling is on and pairs are left)
    int prof_begin(int tag) {
        if (prof_mute || capturing || !ctx->prof_on || !((ctx->prof_mask >> tag) & 1) || ctx->prof_used >= ctx->prof_ev.size() / 2) return -1;
        const int k = (int)ctx->prof_used++;
        ctx->prof_tag[k] = tag;
        note(hipEventRecord(ctx->prof_ev[2 * k], st));
        return k;
    }
    void prof_end(int k) { if (k >= 0) note(hipEventRecord(ctx->prof_ev[2 * k + 1], st)); }
    int max_len() const { return max_rows > max_cols ? max_rows : max_cols; }
    int max_lenP() const { return max_rowsP > max_colsP ? max_rowsP : max_colsP; }

    // operand copies of caller-supplied thin matrices: the transposed ones for a product, the row-major ones for an
    // outer-product kernel
    enum { PACK_ROWMAJOR = 1, PACK_TRANSPOSED = 2 };
    void pack(int role, int cp, int which, int role_b = -1) {
        note(launch_pack(layers, ids_all, n_all, max_lenP(), role, role_b, cp, which, st));
    }
    // product whose result is P-like (lives on the long side) or Q-like, stored in thin[out_role];
    // chol_gate >= -1: the first CholeskyQR pass on the result follows at once (see prod_orth)
    void prod(bool p_like, bool form, int nb, int out_role, int epi, int chol_gate = -2, int a2gate = -2,
              double tol2 = 0.0, int w = 0, bool small = false) {
        // normal storage: P-like result is L-side -> row mode; transposed storage: column mode
        const int k = prof_begin(p_like ? PSGD_PROF_SWEEP1 : PSGD_PROF_SWEEP2);
        const int ef = epi | (keep_e ? EPI_KEEP_E : 0) | (kept_packs && epi == EPI_PACK ? EPI_KEPT : 0);
        const int tiles_row = form ? tiles_row_f : this->tiles_row, tiles_col = form ? tiles_col_f : this->tiles_col;
        const int split_row = form ? split_row_f : this->split_row, split_col = form ? split_col_f : this->split_col;
        const bool onew = ctx->n_workers == 1;
        // forming pass on row-major layers at compress-step widths: the kernel built on 32 x 256 tiles
        // (never inside the gated part of the subspace iteration: its first product carries gate iteration 0,
        // which is open for every layer)
        const bool v2 = form && p_like && n_norm > 0 && ctx->grad_kind != 0 && use_form_row &&
                        form_row_supported(nb, ctx->planes, ctx->grad_kind == 2, onew, lazy_form);
        // (the XCD table pays where the thin operands are a large part of what a workgroup reads: width 64)
        const int* xtab = (ctx->xstride > 0 && use_xtab && nb >= 2 && ids_norm == ids_all + ctx->n_layers)
                              ? reinterpret_cast<const int*>(ws + ctx->off_xtab) : nullptr;
        // the same product on a matrix that is already formed (the refresh's iteration, further power steps)
        const bool r2 = !form && p_like && n_norm > 0 && use_form_row && row_prod_supported(nb, ctx->planes);
        const bool gram32 = (v2 || r2) && split_row_v2 == 1 && epi == EPI_GRAM && w > 16 && chol_gate >= -1;
        // the second product on row-major layers at those widths likewise
        const bool c2 = !form && !p_like && n_norm > 0 && use_form_row && col_prod_supported(nb, ctx->planes);
        const int* xtab_c = (ctx->xstride > 0 && use_xtab && use_xtab_c && nb >= 2 && ids_norm == ids_all + ctx->n_layers)
                                ? reinterpret_cast<const int*>(ws + ctx->off_xtab_c) : nullptr;
        if (c2) note(launch_col_prod(nb, ctx->planes, layers, ids_norm, n_norm, tiles_col_v2, out_role, ef, gate, ctx->nt_m ? 1 : 0, xtab_c, ctx->xstride, ctx->xtiles_c, st));
        else if (r2) note(launch_row_prod(nb, ctx->planes, layers, ids_norm, n_norm, tiles_row_v2, out_role, gram32 ? ef : (ef & ~EPI_KIND_MASK), gate, ctx->nt_m ? 1 : 0, xtab, ctx->xstride, ctx->xtiles, st));
        else if (v2) note(launch_form_row(nb, ctx->planes, ctx->grad_kind == 2, onew, lazy_form ? (lazy_share ? 2 : 1) : 0, layers, ids_norm, n_norm, tiles_row_v2, out_role, gram32 ? ef : (ef & ~EPI_KIND_MASK), ctx->nt_m ? 1 : 0, xtab, ctx->xstride, ctx->xtiles, st));
        else note(launch_prod(nb, ctx->planes, !p_like, form, form && p_like && lazy_form, onew, layers, ids_norm, n_norm, p_like ? tiles_row : tiles_col, out_role, ef, gate, st));
        note(launch_prod(nb, ctx->planes, p_like, form, form && p_like && lazy_form && ctx->lazy_tr, onew, layers, ids_tr, n_tr, p_like ? tiles_col : tiles_row, out_role, ef, gate, st));
        prof_end(k);
        // split reductions are completed (and the epilogue run) by a second, small launch, whose last
        // workgroup per layer also factorises the Gram matrix; unsplit products need a launch for that
        const bool rv2 = v2 || r2;
        const bool split_n = rv2 ? split_row_v2 > 1 : c2 ? split_col_v2 > 1 : (p_like ? split_row > 1 : split_col > 1), split_t = p_like ? split_col > 1 : split_row > 1;
        if (split_n) note(launch_finish(!p_like, rv2 ? 2 : c2 ? 3 : (form ? 1 : 0), layers, ids_norm, n_norm, p_like ? blocks_row : blocks_col, 32 * nb, out_role, epi | (ef & EPI_KEPT), gate, chol_gate, a2gate, tol2, w, small ? 1 : 0, st));
        if (split_t) note(launch_finish(p_like, form ? 1 : 0, layers, ids_tr, n_tr, p_like ? blocks_col : blocks_row, 32 * nb, out_role, epi | (ef & EPI_KEPT), gate, chol_gate, a2gate, tol2, w, small ? 1 : 0, st));
        // (an unsplit launch of that kernel writes one partial Gram matrix per 32-row block itself where the
        // factorisation is a launch of its own -- widths above 16 --, and leaves them to a small pass over the result,
        // one per 128 rows, where the apply kernel factorises for itself)
        if (rv2 && !split_n && epi == EPI_GRAM && !gram32) note(launch_thin_gram(layers, ids_norm, n_norm, blocks_row, out_role, 32 * nb, gate, st));
        // (after a split product only the layers finish_kernel leaves to it -- wide, many Gram slots -- and none at
        // widths where there are no such layers)
        if (chol_gate >= -1) {
            // (32-row slots: added up in groups of 16 side by side first, the factorisation's one workgroup per layer
            // would otherwise spend most of its time on that sum)
            if (gram32) note(launch_slot_sum(layers, ids_norm, n_norm, max_rows, out_role, 32, 16, gate, st));
            if (!split_n || w > 16) note(launch_chol(layers, ids_norm, n_norm, w, out_role, tol2, 1, gram32 ? 32 : kGramRows1, chol_gate, a2gate, small ? 1 : 0, gram32 ? 16 : (split_n ? 1 : 0), st));
            if (!split_t || w > 16) note(launch_chol(layers, ids_tr, n_tr, w, out_role, tol2, 1, kGramRows1, chol_gate, a2gate, small ? 1 : 0, split_t ? 1 : 0, st));
        }
    }
    // thin[out_role] = product as in prod(), then CholeskyQR2 on it: the first pass always, the second
    // when the first one's pivots ask for it (decided on the device) and `pass2` allows it.  Inside the
    // subspace iteration the second pass is only wanted where exact orthonormality matters: on Z in a
    // layer's last iteration.  cp > 0: also leave the split-bf16 operand copies of the result.
    enum Pass2 { PASS2_NEVER = 0, PASS2_ALWAYS = 1, PASS2_LAST_ITERATION = 2 };
    void prod_orth(bool p_like, bool form, int nb, int out_role, int w, double tol2, int cp, int kind, Pass2 pass2) {
        const int g = gate < 0 ? -1 : gate_with_kind(gate, kind);
        const int a2 = pass2 == PASS2_ALWAYS ? -1 : (pass2 == PASS2_NEVER || gate < 0) ? -2 : gate_with_kind(gate, 2);
        // narrow blocks everywhere: the apply kernel factorises per workgroup and hands over to the second
        // factorisation itself; otherwise the second factorisation is a launch of its own
        const bool small = w <= 16;
        // (inside the iteration only products read the result: no row-major operand copies)
        const int wh = gate >= 0 ? PACK_TRANSPOSED : (PACK_ROWMAJOR | PACK_TRANSPOSED | (kept_packs ? 4 : 0));
        prod(p_like, form, nb, out_role, EPI_GRAM, g, a2, tol2, w, small);
        note(launch_apply(layers, ids_all, n_all, max_lenP(), w, w, out_role, out_role, APPLY_PASS1, cp, g, a2, tol2, small, wh, st));
        if (a2 != -2) {
            const int g2 = a2 == -1 ? g : a2;
            if (!small) note(launch_chol(layers, ids_all, n_all, w, out_role, tol2, 2, kGramRows2, g2, -2, 0, 0, st));
            note(launch_apply(layers, ids_all, n_all, max_lenP(), w, w, out_role, out_role, APPLY_PASS2, cp, g2, a2, tol2, small, wh, st));
        }
    }
    // the same CholeskyQR2 on a thin[out_role] that the caller supplied: its Gram slots come from a pass of their own
    void orth_given(int out_role, int w, double tol2, int cp) {
        const bool small = w <= 16;
        const int blocks = (max_lenP() + 127) / 128;
        note(launch_thin_gram(layers, ids_all, n_all, blocks, out_role, cp, -1, st));
        note(launch_chol(layers, ids_all, n_all, w, out_role, tol2, 1, kGramRows1, -1, -1, small ? 1 : 0, 0, st));
        note(launch_apply(layers, ids_all, n_all, max_lenP(), w, w, out_role, out_role, APPLY_PASS1, cp, -1, -1, tol2, small, 3, st));
        if (!small) note(launch_chol(layers, ids_all, n_all, w, out_role, tol2, 2, kGramRows2, -1, -2, 0, 0, st));
        note(launch_apply(layers, ids_all, n_all, max_lenP(), w, w, out_role, out_role, APPLY_PASS2, cp, -1, -1, tol2, small, 3, st));
    }
    void residual(int nb, bool form = false) {
        const int k = prof_begin(PSGD_PROF_RESIDUAL);
        note(launch_outer(nb, ctx->planes, false, form, false, layers, ids_all, n_all, tiles_outer, nullptr, 0, st));
        prof_end(k);
    }
    // deferred residual: the layers that defer keep their operands; the others (stored with rows < cols, at
    // widths above 32) take their residual at once
    // (the layers that defer need no launch: the step's apply and product kernels have written their kept copies)
    void residual_deferred(int nb) {
        if (ctx->lazy_tr) return;
        const int k = prof_begin(PSGD_PROF_RESIDUAL);
        note(launch_outer(nb, ctx->planes, false, false, false, layers, ids_tr, n_tr, tiles_outer, nullptr, 0, st));
        prof_end(k);
    }
    // E <- M - (kept P~)(kept Q)^T for the layers that defer: what the deferred residual still owes
    void residual_owed(int nb) {
        const int k = prof_begin(PSGD_PROF_RESIDUAL);
        if (ctx->lazy_tr) note(launch_outer(nb, ctx->planes, false, false, true, layers, ids_all, n_all, tiles_outer, nullptr, 0, st));
        else note(launch_outer(nb, ctx->planes, false, false, true, layers, ids_norm, n_norm, tiles_outer, nullptr, 0, st));
        prof_end(k);
    }
};

void geometry(const psgd_ctx* c, int l, int split_row, int split_col, int split_row_f, int split_col_f, Launcher& L) {
    const Plan& p = c->plan[l];
    auto mx = [](int& a, int b) { if (b > a) a = b; };
    mx(L.max_rows, (int)p.d.rows); mx(L.max_cols, (int)p.d.cols);
    mx(L.max_rowsP, p.rowsP); mx(L.max_colsP, p.colsP);
    mx(L.tiles_row, (int)((p.d.rows + 127) / 128) * split_row);
    mx(L.tiles_col, (int)((p.d.cols + 127) / 128) * split_col);
    mx(L.tiles_row_f, (int)((p.d.rows + 127) / 128) * split_row_f);
    mx(L.tiles_col_f, (int)((p.d.cols + 127) / 128) * split_col_f);
    mx(L.blocks_row, (int)((p.d.rows + 127) / 128));
    mx(L.blocks_col, (int)((p.d.cols + 127) / 128));
    L.split_row = split_row; L.split_col = split_col;
    L.split_row_f = split_row_f; L.split_col_f = split_col_f;
    L.split_row_v2 = c->split_row_v2;
    mx(L.tiles_row_v2, (p.rowsP / 32) * c->split_row_v2);
    L.split_col_v2 = c->split_col_v2;
    mx(L.tiles_col_v2, ((p.colsP + 255) / 256) * c->split_col_v2);
    mx(L.tiles_outer, (int)((p.d.rows + 127) / 128) * (int)((p.d.cols + 127) / 128));
}

Launcher batch_launcher(psgd_ctx* ctx, void* workspace, hipStream_t st) {
    Launcher L{};
    L.ctx = ctx; L.ws = reinterpret_cast<char*>(workspace); L.st = st;
    L.capturing = ctx->prof_on && is_capturing(st);
    L.layers = reinterpret_cast<const LayerDev*>(L.ws + ctx->off_layers_s[ctx->cur_slot]);
    const int nl = ctx->n_layers;
    const int* ids = reinterpret_cast<const int*>(L.ws + ctx->off_ids);
    L.ids_all = ids; L.ids_norm = ids + nl; L.ids_tr = ids + 2 * (size_t)nl;
    L.n_all = nl; L.n_norm = (int)ctx->lists.norm.size(); L.n_tr = (int)ctx->lists.tr.size();
    for (int l = 0; l < nl; ++l) geometry(ctx, l, ctx->split_row_b, ctx->split_col_b, ctx->split_row_bf, ctx->split_col_bf, L);
    L.use_form_row = form_row_env();
    { static int v = -1; if (v < 0) { const char* e = std::getenv("PSGD_XTAB"); v = (e && e[0] == '0') ? 0 : 1; } L.use_xtab = v == 1; }
    { static int v = -1; if (v < 0) { const char* e = std::getenv("PSGD_XTAB_C"); v = (e && e[0] == '0') ? 0 : 1; } L.use_xtab_c = v == 1; }
    return L;
}

double tol2_of(const psgd_ctx* c) {
    const double t = c->opt.rank_tol > 0.f ? (double)c->opt.rank_tol : 1e-5;
    return t * t;
}

// Block subspace iteration + Rayleigh-Ritz for the layers of `L`: leaves P~ (Ritz vectors of the r
// largest singular values) in thin[ROLE_P] and Q = M^T P~ in thin[ROLE_Q].
void refresh_sequence(psgd_ctx* ctx, Launcher& L, bool form_first, bool warm, float* sigma_out, int final_cp,
                      int launch_iters = 0, int least_iters = 0) {
    const int wz = ctx->wz, cpz = ctx->cpz, nbz = cpz / 32;
    const int iters = ctx->opt.refresh_iters > 0 ? ctx->opt.refresh_iters : 16;
    const int n_launch = launch_iters > 0 && launch_iters < iters ? launch_iters : iters;
    const double tol2 = tol2_of(ctx);
    L.prof_mute = true;
    L.note(launch_init_block(L.layers, L.ids_all, L.n_all, L.max_len(), wz, ROLE_ZQ, ROLE_Q, warm ? 1 : 0,
                             ctx->opt.seed, L.st));
    L.pack(ROLE_ZQ, cpz, Launcher::PACK_TRANSPOSED);
    for (int it = 0; it < n_launch; ++it) {
        // every layer runs its own number of iterations (decided on the device from the Ritz values of
        // its previous refresh); launches past that number find their gate closed and exit at once
        L.gate = make_gate(it, 0, iters, n_launch);
        // Z = orth(M Y);  Y = M^T Z, orthonormalised except in a layer's last iteration
        // (the second CholeskyQR pass on Z belongs to a layer's last iteration: where the smallest count among the
        // layers is known, the iterations before it need no launch for it)
        const bool may_be_last = least_iters <= 0 || it + 1 >= least_iters;
        L.prod_orth(true, form_first && it == 0, nbz, ROLE_ZP, wz, tol2, cpz, 0,
                    may_be_last ? Launcher::PASS2_LAST_ITERATION : Launcher::PASS2_NEVER);
        L.prod_orth(false, false, nbz, ROLE_ZQ, wz, tol2, cpz, 1, Launcher::PASS2_NEVER);
    }
    L.gate = -1;
    // Rayleigh-Ritz on H = Y^T Y (its partial Gram matrices are the last product's)
    L.note(launch_jacobi(L.layers, L.ids_all, L.n_all, wz, ROLE_ZQ, sigma_out, L.st));
    L.note(launch_apply(L.layers, L.ids_all, L.n_all, L.max_lenP(), wz, ctx->rmax, ROLE_ZP, ROLE_P, APPLY_RITZ,
                        final_cp, -1, -2, 0.0, false, 3, L.st));
    L.note(launch_apply(L.layers, L.ids_all, L.n_all, L.max_lenP(), wz, ctx->rmax, ROLE_ZQ, ROLE_Q, APPLY_RITZ,
                        final_cp, -1, -2, 0.0, false, 3, L.st));
    L.prof_mute = false;
}

}  // namespace

extern "C" {

int psgd_init(psgd_ctx** out, int n_layers, const psgd_layer_desc* layers, int n_workers, const psgd_options* opt) {
    if (!out) return PSGD_E_INVALID_ARG;
    *out = nullptr;
    if (!layers || n_layers < 1 || n_layers > 65535 || n_workers < 1 || n_workers > 4096) return PSGD_E_INVALID_ARG;
    psgd_ctx* c = new (std::nothrow) psgd_ctx();
    if (!c) return PSGD_E_NOMEM;
    {
        static std::atomic<uint64_t> next_serial{1};
        c->serial = next_serial.fetch_add(1);
    }
    c->n_layers = n_layers;
    c->n_workers = n_workers;
    if (opt) c->opt = *opt;
    else { c->opt = psgd_options{}; c->opt.refresh_warm_start = 1; c->opt.refresh_oversample = -1; c->opt.seed = 0x5eed5eedu; }
    int rc = PSGD_OK;
    int rmax = 0;
    c->plan.resize(n_layers);
    for (int l = 0; l < n_layers && rc == PSGD_OK; ++l) {
        psgd_layer_desc d = layers[l];
        if (d.rows < 1 || d.cols < 1 || d.rows > (1 << 24) || d.cols > (1 << 24)) { rc = PSGD_E_SHAPE; break; }
        if (d.r < 1 || d.r > d.rows || d.r > d.cols) { rc = PSGD_E_SHAPE; break; }
        if (d.grad_dtype != PSGD_F32 && d.grad_dtype != PSGD_BF16) { rc = PSGD_E_INVALID_ARG; break; }
        if (d.ld == 0) d.ld = d.cols;
        if (d.ld < d.cols || d.ld % 8 != 0) { rc = PSGD_E_ALIGN; break; }
        // the kernels address a lane's pieces of a 128-row tile with 32-bit byte offsets: 127 * ld * 4 < 2^32
        if (d.ld > kMaxLd) { rc = PSGD_E_SHAPE; break; }
        Plan& p = c->plan[l];
        p.d = d;
        p.transposed = d.rows < d.cols ? 1 : 0;
        p.rowsP = (int)round_up(d.rows, kLenPad);
        p.colsP = (int)round_up(d.cols, kLenPad);
        p.m = (int)(d.rows >= d.cols ? d.rows : d.cols);
        p.n = (int)(d.rows >= d.cols ? d.cols : d.rows);
        (p.transposed ? c->lists.tr : c->lists.norm).push_back(l);
        if (d.r > rmax) rmax = d.r;
    }
    // launch order: the largest layers first (a launch ends with its shortest-lived workgroups)
    auto by_size = [&](int a, int b) {
        return c->plan[a].d.rows * c->plan[a].d.cols > c->plan[b].d.rows * c->plan[b].d.cols;
    };
    if (rc == PSGD_OK) {
        std::stable_sort(c->lists.norm.begin(), c->lists.norm.end(), by_size);
        std::stable_sort(c->lists.tr.begin(), c->lists.tr.end(), by_size);
    }
    if (rc == PSGD_OK) {
        // operand planes: bf16 gradients are compared at 2e-2, two planes (2^-17) are ample; fp32
        // gradients are held to 1e-4 of ||E||, which can be 100x smaller than ||M||: three planes
        bool any_f32 = false;
        for (auto& p : c->plan) any_f32 |= (p.d.grad_dtype == PSGD_F32);
        const int prec = c->opt.precision;
        if (prec != 0 && prec != 2 && prec != 3) rc = PSGD_E_INVALID_ARG;
        c->planes = prec ? prec : (any_f32 ? 3 : 2);
        // M between the passes: stored over E (N*sg + 20 bytes per element over the three kernels) or formed
        // again from G and E in every pass (3*N*sg + 16).  Equal bytes at N*sg = 2 (one bf16 worker), where
        // forming again makes pass 1 read-only -- but the residual then merges three streams and is the slower
        // by more than pass 1 gains (7B-shaped set: 35.4 against 31.6 ms per step), so storing is the default.
        const int pol = c->opt.m_policy;
        if (pol < 0 || pol > 2) rc = PSGD_E_INVALID_ARG;
        if (c->opt.power_iters < 0 || c->opt.power_iters > 64) rc = PSGD_E_INVALID_ARG;
        if (c->opt.refresh_iters < 0 || c->opt.refresh_iters > kMaxRefreshIterations) rc = PSGD_E_INVALID_ARG;
        c->reform_m = pol == 2;
        if (c->opt.lazy_residual != 0 && c->opt.lazy_residual != 1) rc = PSGD_E_INVALID_ARG;
        if (c->opt.q_resident != 0 && c->opt.q_resident != 1) rc = PSGD_E_INVALID_ARG;
        if (c->opt.lazy_residual && c->reform_m) rc = PSGD_E_INVALID_ARG;      // the deferred residual lives in the stored M
        c->lazy = c->opt.lazy_residual == 1;
    }
    if (rc == PSGD_OK) {
        c->rmax = rmax;
        c->cpc = (int)round_up(rmax, 32);
        int over = c->opt.refresh_oversample;
        if (over < 0) over = 8;
        if (c->opt.refresh_oversample < 0) over = rmax / 4 > 8 ? rmax / 4 : 8;
        c->wz = (int)round_up(rmax + over, 8);
        int nmin = c->plan[0].n;
        for (auto& p : c->plan) if (p.n < nmin) nmin = p.n;
        if (c->wz > nmin) c->wz = nmin;                                         // block no wider than the matrix
        c->cpz = (int)round_up(c->wz, 32);
        c->cpmax = c->cpz > c->cpc ? c->cpz : c->cpc;
        if (c->cpmax > kMaxWidth) rc = PSGD_E_SHAPE;
        if (c->lazy && c->cpc > 128) rc = PSGD_E_SHAPE;
        c->lazy_tr = c->lazy && c->cpc == 32;
    }
    if (rc != PSGD_OK) { delete c; return rc; }
    // reduction splits of the batched launches
    int64_t base_row = 0, base_col = 0;
    int min_chunks_row = 1 << 30, min_chunks_col = 1 << 30;
    for (auto& p : c->plan) {
        base_row += (p.d.rows + 127) / 128;
        base_col += (p.d.cols + 127) / 128;
        const int cr = (int)((p.d.cols + 63) / 64), cc = (int)((p.d.rows + 63) / 64);
        if (cr < min_chunks_row) min_chunks_row = cr;
        if (cc < min_chunks_col) min_chunks_col = cc;
    }
    c->split_row_b = choose_split(base_row, min_chunks_row, false, c->cpc);
    c->split_col_b = choose_split(base_col, min_chunks_col, false, c->cpc);
    c->split_row_bf = choose_split(base_row, min_chunks_row, true, c->cpc);
    c->split_col_bf = choose_split(base_col, min_chunks_col, true, c->cpc);
    {
        // the forming pass on 32 x 256 tiles: row-major layers only
        int64_t base = 0, base_c = 0, m_bytes = 0;
        int min_chunks = 1 << 30, min_chunks_c = 1 << 30;
        bool f32 = false, b16 = false;
        for (auto& p : c->plan) {
            (p.d.grad_dtype == PSGD_F32 ? f32 : b16) = true;
            if (p.transposed) continue;
            base += p.rowsP / 32;
            base_c += (p.colsP + 255) / 256;
            m_bytes += p.d.rows * p.d.cols * 4;
            const int ch = (int)((p.d.cols + 255) / 256), chc = (int)((p.d.rows + 31) / 32);
            if (ch < min_chunks) min_chunks = ch;
            if (chc < min_chunks_c) min_chunks_c = chc;
        }
        c->split_row_v2 = base > 0 ? choose_split(base, min_chunks, true, 32) : 1;
        c->split_col_v2 = base_c > 0 ? choose_split(base_c, min_chunks_c, false, 32) : 1;
        c->grad_kind = f32 && b16 ? 0 : (f32 ? 1 : 2);
        // M that the second pass can find in the 256 MB memory-side cache is stored with plain stores
        c->nt_m = m_bytes > ((int64_t)96 << 20);
        if (const char* e = std::getenv("PSGD_NT_M")) c->nt_m = e[0] != '0';     // (measurement knob)
        // XCD table: the row-major layers (positions in the id list `norm`), largest first, each to the XCD with the
        // least work so far
        const int n_norm = (int)c->lists.norm.size();
        if (n_norm >= 32) {
            c->xstride = n_norm + 2;
            // work = rows x cols decides the deal (the same for both kernels), tiles = what a layer launches
            auto build = [&](std::vector<int>& tab, int& xtiles, auto tiles_of) {
                tab.assign((size_t)16 * c->xstride, 0);
                std::vector<int> order(n_norm);
                for (int i = 0; i < n_norm; ++i) order[i] = i;
                auto work_of = [&](int pos) { const Plan& p = c->plan[c->lists.norm[pos]]; return p.d.rows * p.d.cols; };
                std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return work_of(a) > work_of(b); });
                int64_t work[8] = {0, 0, 0, 0, 0, 0, 0, 0};
                int total[8] = {0, 0, 0, 0, 0, 0, 0, 0}, count[8] = {0, 0, 0, 0, 0, 0, 0, 0};
                for (int pos : order) {
                    int x = 0;
                    for (int k = 1; k < 8; ++k) if (work[k] < work[x]) x = k;
                    tab[(size_t)(8 + x) * c->xstride + count[x]] = pos;
                    total[x] += tiles_of(pos);
                    work[x] += work_of(pos);
                    count[x] += 1;
                    tab[(size_t)x * c->xstride + count[x]] = total[x];
                }
                for (int x = 0; x < 8; ++x) {
                    tab[(size_t)x * c->xstride + c->xstride - 1] = count[x];
                    if (total[x] > xtiles) xtiles = total[x];
                }
            };
            build(c->hXtab, c->xtiles, [&](int pos) { return (c->plan[c->lists.norm[pos]].rowsP / 32) * c->split_row_v2; });
            build(c->hXtabC, c->xtiles_c, [&](int pos) { return ((c->plan[c->lists.norm[pos]].colsP + 255) / 256) * c->split_col_v2; });
        }
    }
    // workspace layout
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = (size_t)round_up((int64_t)(o + bytes), 256); return at; };
    for (int k = 0; k < psgd_ctx::kGSlots; ++k) c->off_layers_s[k] = take((size_t)(n_layers + 1) * sizeof(LayerDev));
    c->off_ids = take((3 * (size_t)n_layers + 1) * sizeof(int));
    c->off_iters = take(psgd_ctx::kIterSlots * sizeof(int));
    c->off_xtab = take(c->hXtab.size() * sizeof(int) + 16);
    c->off_xtab_c = take(c->hXtabC.size() * sizeof(int) + 16);
    for (int k = 0; k < psgd_ctx::kGSlots; ++k) c->off_gtab_s[k] = take((size_t)n_layers * n_workers * sizeof(void*));
    c->off_outs = take((size_t)n_layers * sizeof(void*));
    c->off_moms = take((size_t)n_layers * sizeof(void*));
    c->off_xs = take((size_t)n_layers * sizeof(void*));
    c->off_m2s = take((size_t)n_layers * sizeof(void*));
    int max_rowsP = 0, max_colsP = 0;
    for (auto& p : c->plan) { if (p.rowsP > max_rowsP) max_rowsP = p.rowsP; if (p.colsP > max_colsP) max_colsP = p.colsP; }
    c->off_single_part[0] = take((size_t)kMaxSplit * max_rowsP * c->wz * sizeof(float));
    c->off_single_part[1] = take((size_t)kMaxSplit * max_colsP * c->wz * sizeof(float));
    c->off_layer.resize(n_layers);
    double bytes = 0.0;
    for (int l = 0; l < n_layers; ++l) {
        c->off_layer[l] = o;
        o += layer_region(c, c->plan[l]).end;
        const Plan& p = c->plan[l];
        const double sg = p.d.grad_dtype == PSGD_BF16 ? 2.0 : 4.0;
        // two passes separated by the global QR: either M is stored between them (N*sg + 16 bytes
        // per element) or formed twice from the gradients (2*N*sg + 12); the smaller one counts
        const double a = n_workers * sg + 16.0, b = 2.0 * n_workers * sg + 12.0;
        bytes += (double)p.d.rows * (double)p.d.cols * (a < b ? a : b);
        bytes += 4.0 * 4.0 * (double)(p.d.rows + p.d.cols) * p.d.r;
        const double e = (double)p.d.rows * (double)p.d.cols, nsg = n_workers * sg;
        const double thin = 4.0 * (double)(p.d.rows + p.d.cols) * 32.0 * ((p.d.r + 31) / 32);
        const bool deferred = c->lazy && (!p.transposed || c->lazy_tr);
        // (deferred residual: the kept P~ and Q are read as well -- the kept Q not where the pass takes it from the
        // product's own fragments: q_resident, row-major layers)
        const double kept_q = 4.0 * (double)p.d.cols * 32.0 * ((p.d.r + 31) / 32);
        const bool shared_q = deferred && c->opt.q_resident == 1 && !p.transposed;
        c->kernel_bytes[0] += e * (nsg + 4.0 + (c->reform_m ? 0.0 : 4.0)) + thin * (deferred ? 2.0 : 1.0) - (shared_q ? kept_q : 0.0);
        c->kernel_bytes[1] += e * (c->reform_m ? nsg + 4.0 : 4.0) + thin;
        if (!deferred) c->kernel_bytes[2] += e * (c->reform_m ? nsg + 8.0 : 8.0) + thin;
    }
    c->ws_bytes = o;
    c->algo_bytes = bytes;
    // host tables at their final capacity, so that no compute call allocates host memory either
    {
        const size_t nl = (size_t)n_layers, ng = nl * (size_t)n_workers;
        c->hG.reserve(ng);
        for (auto& v : c->hGs) v.reserve(ng);
        c->hE.reserve(nl); c->hQ.reserve(nl); c->hP.reserve(nl);
        c->hOut.reserve(nl); c->hMom.reserve(nl); c->hM2.reserve(nl); c->hX.reserve(nl);
        c->hIds.reserve(3 * nl + 1);
        c->hLayers.reserve(nl + 1);
    }
    *out = c;
    return PSGD_OK;
}

size_t psgd_workspace_bytes(const psgd_ctx* ctx) { return ctx ? ctx->ws_bytes : 0; }

double psgd_algorithmic_bytes(const psgd_ctx* ctx) { return ctx ? ctx->algo_bytes : 0.0; }

double psgd_kernel_bytes(const psgd_ctx* ctx, int tag) {
    return (ctx && tag >= 0 && tag < 3) ? ctx->kernel_bytes[tag] : 0.0;
}

static int bind_common(psgd_ctx* ctx, void* workspace, hipStream_t st, const void* const* G, float* const* E,
                       float* const* Q, float* const* P) {
    if (!ctx || !workspace) return PSGD_E_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return PSGD_E_ALIGN;
    const size_t nl = (size_t)ctx->n_layers;
    int rc;
    if (G && (rc = check_table(G, nl * ctx->n_workers)) != PSGD_OK) return rc;
    if (E && (rc = check_table(reinterpret_cast<const void* const*>(E), nl)) != PSGD_OK) return rc;
    if (Q && (rc = check_table(reinterpret_cast<const void* const*>(Q), nl)) != PSGD_OK) return rc;
    if (P && (rc = check_table(reinterpret_cast<const void* const*>(P), nl)) != PSGD_OK) return rc;
    const bool g_changed = sync_table(ctx->hG, G, nl * ctx->n_workers);
    bool changed = false;
    changed |= sync_table(ctx->hE, E, nl);
    changed |= sync_table(ctx->hQ, Q, nl);
    changed |= sync_table(ctx->hP, P, nl);
    return upload_tables(ctx, workspace, st, changed, g_changed);
}

int psgd_workspace_reset(psgd_ctx* ctx) {
    if (!ctx || ctx->pending) return PSGD_E_INVALID_ARG;
    ctx->tables_valid = false;
    ctx->bound_ws = nullptr;
    ctx->outs_ws = nullptr;
    ctx->msgd_ws = nullptr;
    ctx->m2_ws = nullptr;
    ctx->factors_ws = nullptr;
    ctx->iters_gen++;
    return PSGD_OK;
}

int psgd_compress(psgd_ctx* ctx, void* workspace, void* stream, const void* const* G, float* const* E,
                  float* const* Q, float* const* P) {
    if (!ctx || !G || !E || !Q || !P) return PSGD_E_INVALID_ARG;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (ctx->pending && ctx->bound_ws != workspace) return PSGD_E_INVALID_ARG;   // the kept operands live in the old one
    int rc = bind_common(ctx, workspace, st, G, E, Q, P);
    if (rc != PSGD_OK) return rc;
    // Q_{t-1} as a product operand: packed from the caller's buffers, unless they are promised to be what the last
    // call wrote there, whose operand copies are still in place
    const bool q_in_place = ctx->opt.q_resident == 1 && ctx->factors_ws == workspace;
    ctx->factors_ws = nullptr;
    Launcher L = batch_launcher(ctx, workspace, st);
    const int cp = ctx->cpc, nb = cp / 32;
    if (!q_in_place) L.pack(ROLE_Q, cp, Launcher::PACK_TRANSPOSED);
    // P = M Q_{t-1} (M formed on the way and, unless it is formed again below, stored over E);
    // P~ = QR(P), operand copies of P~;  Q_t = M^T P~, operand copies of Q_t;  K times (Eq. (8)), K = 1 by default
    const bool re = ctx->reform_m;
    const int K = ctx->opt.power_iters > 0 ? ctx->opt.power_iters : 1;
    L.kept_packs = ctx->lazy;
    for (int k = 0; k < K; ++k) {
        L.keep_e = re;
        L.lazy_form = ctx->pending;            // E of the row-major layers is M_{t-1} - (kept P~)(kept Q)^T
        L.lazy_share = q_in_place;
        L.prod_orth(true, k == 0 || re, nb, ROLE_P, ctx->rmax, tol2_of(ctx), cp, 0, Launcher::PASS2_ALWAYS);
        if (k == 0) ctx->pending = false;      // the buffers hold M_t from here on
        L.lazy_form = false;
        L.prod(false, re, nb, ROLE_Q, EPI_PACK);
        L.keep_e = false;
    }
    if (ctx->lazy) {
        L.residual_deferred(nb);                   // owed: E <- M - P~ Q_t^T, applied by the next forming pass
        ctx->pending = L.n_norm > 0 || ctx->lazy_tr;
    } else {
        L.residual(nb, re);                        // E <- M - P~ Q_t^T
    }
    if (L.err != hipSuccess) return fail_hip(ctx, L.err);
    ctx->factors_ws = workspace;                   // the operand copies of P~_t and Q_t are in place
    ctx->factors_kept = ctx->lazy;
    return PSGD_OK;
}

// The built-in workspace of psgd_compress_static: one array per GPU (every device that loads this code object holds its
// own copy at its own address).  In host code the array's name is only a handle for hipGetSymbolAddress; the device
// address it returns, looked up once per device with that device current, is what is passed on.
static __device__ __align__(256) unsigned char g_static_workspace[PSGD_STATIC_WORKSPACE_BYTES];
namespace {
constexpr int kMaxDevices = 64;
struct StaticWorkspace { void* ptr = nullptr; uint64_t owner = 0; };
StaticWorkspace g_static_ws[kMaxDevices];
std::mutex g_static_mutex;
}  // namespace

int psgd_compress_static(psgd_ctx* ctx, void* stream, const void* const* G, float* const* E, float* const* Q,
                         float* const* P) {
    if (!ctx || !G || !E || !Q || !P) return PSGD_E_INVALID_ARG;
    if (ctx->ws_bytes > (size_t)PSGD_STATIC_WORKSPACE_BYTES) return PSGD_E_TOO_LARGE;
    int dev = -1;
    PSGD_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return PSGD_E_INVALID_ARG;
    void* ws = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_static_mutex);
        StaticWorkspace& W = g_static_ws[dev];
        if (!W.ptr) {
            void* p = nullptr;
            PSGD_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_workspace)));
            if (!p) return fail_hip(ctx, hipErrorInvalidSymbol);
            W.ptr = p;
        }
        ws = W.ptr;
        if (W.owner != ctx->serial) {
            // another context's tables, counters and operand copies are in the buffer (or nothing yet)
            if (ctx->pending && ctx->bound_ws == ws) return PSGD_E_INVALID_ARG;      // its kept operands are gone
            if (ctx->bound_ws == ws) { ctx->tables_valid = false; ctx->iters_gen++; }
            if (ctx->outs_ws == ws) ctx->outs_ws = nullptr;
            if (ctx->msgd_ws == ws) ctx->msgd_ws = nullptr;
            if (ctx->m2_ws == ws) ctx->m2_ws = nullptr;
            if (ctx->factors_ws == ws) ctx->factors_ws = nullptr;
            W.owner = ctx->serial;
        }
    }
    return psgd_compress(ctx, ws, stream, G, E, Q, P);
}

// The two halves of psgd_compress between which a data-parallel job averages P over its workers (and after which
// it averages Q): each worker runs them on its own gradient and error buffer.
int psgd_compress_project(psgd_ctx* ctx, void* workspace, void* stream, const void* const* G, float* const* E,
                          float* const* Q, float* const* P) {
    if (!ctx || !G || !E || !Q || !P) return PSGD_E_INVALID_ARG;
    if (ctx->lazy || ctx->reform_m || ctx->opt.power_iters > 1) return PSGD_E_INVALID_ARG;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    int rc = bind_common(ctx, workspace, st, G, E, Q, P);
    if (rc != PSGD_OK) return rc;
    ctx->factors_ws = nullptr;
    Launcher L = batch_launcher(ctx, workspace, st);
    const int cp = ctx->cpc, nb = cp / 32;
    L.pack(ROLE_Q, cp, Launcher::PACK_TRANSPOSED);
    L.prod(true, true, nb, ROLE_P, EPI_NONE);          // M = mean G + E stored over E;  P = M Q_{t-1}, as it is
    if (L.err != hipSuccess) return fail_hip(ctx, L.err);
    return PSGD_OK;
}

int psgd_compress_finish(psgd_ctx* ctx, void* workspace, void* stream, float* const* E, float* const* Q,
                         float* const* P) {
    if (!ctx || !E || !Q || !P) return PSGD_E_INVALID_ARG;
    if (ctx->lazy || ctx->reform_m || ctx->opt.power_iters > 1) return PSGD_E_INVALID_ARG;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    int rc = bind_common(ctx, workspace, st, nullptr, E, Q, P);
    if (rc != PSGD_OK) return rc;
    Launcher L = batch_launcher(ctx, workspace, st);
    const int cp = ctx->cpc, nb = cp / 32;
    L.orth_given(ROLE_P, ctx->rmax, tol2_of(ctx), cp);  // P~ = QR(P), operand copies of P~
    L.prod(false, false, nb, ROLE_Q, EPI_PACK);         // Q = M^T P~ (this worker's M), operand copies
    L.residual(nb, false);                              // E <- M - P~ Q^T
    if (L.err != hipSuccess) return fail_hip(ctx, L.err);
    ctx->factors_ws = workspace;                        // (copies of P~ and of this worker's Q)
    ctx->factors_kept = false;
    return PSGD_OK;
}

int psgd_flush_residual(psgd_ctx* ctx, void* workspace, void* stream, float* const* E) {
    if (!ctx || !E) return PSGD_E_INVALID_ARG;
    if (!ctx->pending) return PSGD_OK;
    if (ctx->bound_ws != workspace) return PSGD_E_INVALID_ARG;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    int rc = bind_common(ctx, workspace, st, nullptr, E, nullptr, nullptr);
    if (rc != PSGD_OK) return rc;
    Launcher L = batch_launcher(ctx, workspace, st);
    L.prof_mute = true;
    L.residual_owed(ctx->cpc / 32);
    ctx->pending = false;
    if (L.err != hipSuccess) return fail_hip(ctx, L.err);
    return PSGD_OK;
}

int psgd_compress_refresh(psgd_ctx* ctx, void* workspace, void* stream, const void* const* G, float* const* E,
                          float* const* Q, float* const* P) {
    if (!ctx || !G || !E || !Q || !P) return PSGD_E_INVALID_ARG;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (ctx->pending && ctx->bound_ws != workspace) return PSGD_E_INVALID_ARG;   // the kept operands live in the old one
    int rc = bind_common(ctx, workspace, st, G, E, Q, P);
    if (rc != PSGD_OK) return rc;
    ctx->factors_ws = nullptr;
    Launcher L = batch_launcher(ctx, workspace, st);
    if (ctx->pending) {
        // the subspace iteration forms M from a materialised E: settle what the deferred residual owes first
        L.prof_mute = true;
        L.residual_owed(ctx->cpc / 32);
        L.prof_mute = false;
        ctx->pending = false;
    }
    // how many iterations to launch: the bound fetched behind the last refresh, if that copy has arrived and nothing
    // else has changed the counts since.  (None of this bookkeeping under stream capture: a captured refresh
    // launches the whole budget and fetches nothing.)
    const bool capturing = is_capturing(st);
    int bound = 0, least = 0;
    if (!capturing && ctx->fetch_last >= 0) {
        psgd_ctx::IterFetch& F = ctx->fetch[ctx->fetch_last];
        if (F.pending && hipEventQuery(F.ev) == hipSuccess) {
            F.pending = false;
            if (F.gen == ctx->iters_gen && F.seq == ctx->refresh_seq) {
                bound = F.h[0] & 0xffff;
                least = bound > 0 ? (F.h[0] >> 16) : 0;
            }
        }
        (void)hipGetLastError();      // (hipErrorNotReady of the query is not an error)
    }
    const int iters_max = ctx->opt.refresh_iters > 0 ? ctx->opt.refresh_iters : 16;
    refresh_sequence(ctx, L, true, ctx->opt.refresh_warm_start != 0, nullptr, ctx->cpc, bound, least);
    L.residual(ctx->cpc / 32);
    ctx->refresh_seq++;
    ctx->fetch_last = -1;
    if (capturing) ctx->iters_gen++;
    // fetch the bound for the next one (pinned words and events are created on first use; without them every
    // refresh simply launches the whole budget)
    if (!capturing && !ctx->fetch_ready && !ctx->fetch_failed) {
        void* hp = nullptr;
        bool ok = hipHostMalloc(&hp, psgd_ctx::kIterSlots * sizeof(int), hipHostMallocDefault) == hipSuccess;
        for (int k = 0; ok && k < psgd_ctx::kIterSlots; ++k) {
            ctx->fetch[k].h = static_cast<int*>(hp) + k;
            ok = hipEventCreateWithFlags(&ctx->fetch[k].ev, hipEventDisableTiming) == hipSuccess;
            if (!ok) ctx->fetch[k].ev = nullptr;
        }
        if (!ok) {
            for (auto& F : ctx->fetch) { if (F.ev) (void)hipEventDestroy(F.ev); F.ev = nullptr; F.h = nullptr; }
            if (hp) (void)hipHostFree(hp);
            ctx->fetch_failed = true;
        }
        ctx->fetch_ready = ok;
        (void)hipGetLastError();
    }
    if (!capturing && ctx->fetch_ready) {
        int slot = -1;
        for (int k = 0; k < psgd_ctx::kIterSlots && slot < 0; ++k) {
            psgd_ctx::IterFetch& F = ctx->fetch[k];
            if (F.pending && hipEventQuery(F.ev) == hipSuccess) F.pending = false;
            if (!F.pending) slot = k;
        }
        (void)hipGetLastError();
        if (slot >= 0) {
            psgd_ctx::IterFetch& F = ctx->fetch[slot];
            int* d_it = reinterpret_cast<int*>(L.ws + ctx->off_iters) + slot;
            L.note(launch_max_iterations(L.layers, L.ids_all, L.n_all, iters_max, d_it, st));
            L.note(hipMemcpyAsync(F.h, d_it, sizeof(int), hipMemcpyDeviceToHost, st));
            L.note(hipEventRecord(F.ev, st));
            if (L.err == hipSuccess) {
                F.pending = true; F.gen = ctx->iters_gen; F.seq = ctx->refresh_seq;
                ctx->fetch_last = slot;
            }
        }
    }
    if (L.err != hipSuccess) return fail_hip(ctx, L.err);
    ctx->factors_ws = workspace;
    ctx->factors_kept = false;
    return PSGD_OK;
}

int psgd_refresh(psgd_ctx* ctx, void* workspace, void* stream, int layer, const float* M, float* P, float* Q,
                 float* sigma) {
    if (!ctx || !workspace || !M || !P || !Q) return PSGD_E_INVALID_ARG;
    if (layer < 0 || layer >= ctx->n_layers) return PSGD_E_INVALID_ARG;
    if (!aligned16(M) || !aligned16(P) || !aligned16(Q)) return PSGD_E_ALIGN;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    int rc = bind_common(ctx, workspace, st, nullptr, nullptr, nullptr, nullptr);
    if (rc != PSGD_OK) return rc;
    char* ws = reinterpret_cast<char*>(workspace);
    if (is_capturing(st)) return PSGD_E_CAPTURE;       // (every call uploads a descriptor from the host)
    ctx->factors_ws = nullptr;                         // (it rewrites operand copies of this layer)
    const Plan& p = ctx->plan[layer];
    // scratch descriptor: this layer's private regions, the caller's M/P/Q, splits sized for one layer
    LayerDev D;
    build_layer_dev(ctx, ws, layer, ctx->cur_slot, &D);
    D.S = const_cast<float*>(M);
    D.thin[ROLE_P].ptr = P;
    D.thin[ROLE_Q].ptr = Q;
    D.split_row = choose_split((p.d.rows + 127) / 128, (int)((p.d.cols + 63) / 64), false, ctx->cpz);
    D.split_col = choose_split((p.d.cols + 127) / 128, (int)((p.d.rows + 63) / 64), false, ctx->cpz);
    D.split_row_f = D.split_row; D.split_col_f = D.split_col;      // (no forming pass in this call)
    D.part[0] = reinterpret_cast<float*>(ws + ctx->off_single_part[0]);
    D.part[1] = reinterpret_cast<float*>(ws + ctx->off_single_part[1]);
    ctx->hLayers[ctx->n_layers] = D;
    PSGD_TRY(launch_put(ws + ctx->off_layers_s[ctx->cur_slot] + (size_t)ctx->n_layers * sizeof(LayerDev), &D, sizeof(LayerDev), st));
    // this call rewrites the layer's iteration count: what the host knows about the next batched refresh is void
    ctx->iters_gen++;
    Launcher L{};
    L.ctx = ctx; L.ws = ws; L.st = st;
    L.layers = reinterpret_cast<const LayerDev*>(ws + ctx->off_layers_s[ctx->cur_slot]);
    const int* ids = reinterpret_cast<const int*>(ws + ctx->off_ids) + 3 * (size_t)ctx->n_layers;
    L.ids_all = ids; L.n_all = 1;
    L.ids_norm = ids; L.n_norm = p.transposed ? 0 : 1;
    L.ids_tr = ids; L.n_tr = p.transposed ? 1 : 0;
    geometry(ctx, layer, D.split_row, D.split_col, D.split_row_f, D.split_col_f, L);
    refresh_sequence(ctx, L, false, false, sigma, 0);
    if (L.err != hipSuccess) return fail_hip(ctx, L.err);
    return PSGD_OK;
}

// Factors of a decompress-type call: the caller's P and Q (packed by the call), or, with both tables null, the
// operand copies the last compress-type call left in this workspace.  *packed: whether the copies are in place.
static int bind_factors(psgd_ctx* ctx, void* workspace, hipStream_t st, const float* const* P, const float* const* Q,
                        bool* packed) {
    *packed = !P && !Q;
    if (*packed) {
        if (!workspace || ctx->factors_ws != workspace) return PSGD_E_INVALID_ARG;
        return bind_common(ctx, workspace, st, nullptr, nullptr, nullptr, nullptr);
    }
    if (!P || !Q) return PSGD_E_INVALID_ARG;
    ctx->factors_ws = nullptr;          // the copies will be the caller's P and Q
    return bind_common(ctx, workspace, st, nullptr, nullptr, const_cast<float* const*>(Q), const_cast<float* const*>(P));
}

int psgd_decompress(psgd_ctx* ctx, void* workspace, void* stream, const float* const* P, const float* const* Q,
                    void* const* out, int out_dtype) {
    if (!ctx || !out) return PSGD_E_INVALID_ARG;
    if (out_dtype != PSGD_F32 && out_dtype != PSGD_BF16) return PSGD_E_INVALID_ARG;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    int rc = check_table(reinterpret_cast<const void* const*>(out), (size_t)ctx->n_layers);
    if (rc != PSGD_OK) return rc;
    bool packed = false;
    rc = bind_factors(ctx, workspace, st, P, Q, &packed);
    if (rc != PSGD_OK) return rc;
    char* ws = reinterpret_cast<char*>(workspace);
    if (sync_table(ctx->hOut, out, (size_t)ctx->n_layers) || ctx->outs_ws != workspace) {
        if (is_capturing(st)) { ctx->outs_ws = nullptr; return PSGD_E_CAPTURE; }
        PSGD_TRY(launch_put(ws + ctx->off_outs, ctx->hOut.data(), ctx->hOut.size() * sizeof(void*), st));
    }
    ctx->outs_ws = workspace;
    Launcher L = batch_launcher(ctx, workspace, st);
    const int cp = ctx->cpc, nb = cp / 32;
    if (!packed) L.pack(ROLE_P, cp, Launcher::PACK_ROWMAJOR, ROLE_Q);
    // (factors of a compress call with a deferred residual: the layers that defer hold them as their kept copies)
    const bool kept = packed && ctx->factors_kept;
    const int n_kept = !kept ? 0 : ctx->lazy_tr ? L.n_all : L.n_norm;
    const int* ids_kept = ctx->lazy_tr ? L.ids_all : L.ids_norm;
    void* const* outs = reinterpret_cast<void* const*>(ws + ctx->off_outs);
    const int obf = out_dtype == PSGD_BF16 ? 1 : 0;
    if (n_kept > 0) L.note(launch_outer(nb, ctx->planes, true, false, true, L.layers, ids_kept, n_kept, L.tiles_outer, outs, obf, st));
    if (!kept) L.note(launch_outer(nb, ctx->planes, true, false, false, L.layers, L.ids_all, L.n_all, L.tiles_outer, outs, obf, st));
    else if (!ctx->lazy_tr) L.note(launch_outer(nb, ctx->planes, true, false, false, L.layers, L.ids_tr, L.n_tr, L.tiles_outer, outs, obf, st));
    if (L.err != hipSuccess) return fail_hip(ctx, L.err);
    return PSGD_OK;
}

int psgd_decompress_msgd(psgd_ctx* ctx, void* workspace, void* stream, const float* const* P, const float* const* Q,
                         float* const* mom, float* const* X, float mu, float eta) {
    if (!ctx || !mom || !X) return PSGD_E_INVALID_ARG;
    if (!(mu >= 0.f && mu < 1.f) || !(eta == eta)) return PSGD_E_INVALID_ARG;      // Algorithm 2: 0 <= mu < 1
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const size_t nl = (size_t)ctx->n_layers;
    int rc = check_table(reinterpret_cast<const void* const*>(mom), nl);
    if (rc == PSGD_OK) rc = check_table(reinterpret_cast<const void* const*>(X), nl);
    if (rc != PSGD_OK) return rc;
    bool packed = false;
    rc = bind_factors(ctx, workspace, st, P, Q, &packed);
    if (rc != PSGD_OK) return rc;
    char* ws = reinterpret_cast<char*>(workspace);
    const bool changed = sync_table(ctx->hMom, mom, nl) | sync_table(ctx->hX, X, nl);
    if (changed || ctx->msgd_ws != workspace) {
        if (is_capturing(st)) { ctx->msgd_ws = nullptr; return PSGD_E_CAPTURE; }
        PSGD_TRY(launch_put(ws + ctx->off_moms, ctx->hMom.data(), nl * sizeof(void*), st));
        PSGD_TRY(launch_put(ws + ctx->off_xs, ctx->hX.data(), nl * sizeof(void*), st));
    }
    ctx->msgd_ws = workspace;
    Launcher L = batch_launcher(ctx, workspace, st);
    const int cp = ctx->cpc, nb = cp / 32;
    if (!packed) L.pack(ROLE_P, cp, Launcher::PACK_ROWMAJOR, ROLE_Q);
    const bool kept = packed && ctx->factors_kept;      // (see psgd_decompress)
    const int n_kept = !kept ? 0 : ctx->lazy_tr ? L.n_all : L.n_norm;
    const int* ids_kept = ctx->lazy_tr ? L.ids_all : L.ids_norm;
    float* const* dm = reinterpret_cast<float* const*>(ws + ctx->off_moms);
    float* const* dx = reinterpret_cast<float* const*>(ws + ctx->off_xs);
    if (n_kept > 0) L.note(launch_msgd(nb, ctx->planes, L.layers, ids_kept, n_kept, L.tiles_outer, dm, dx, mu, eta, true, st));
    if (!kept) L.note(launch_msgd(nb, ctx->planes, L.layers, L.ids_all, L.n_all, L.tiles_outer, dm, dx, mu, eta, false, st));
    else if (!ctx->lazy_tr) L.note(launch_msgd(nb, ctx->planes, L.layers, L.ids_tr, L.n_tr, L.tiles_outer, dm, dx, mu, eta, false, st));
    if (L.err != hipSuccess) return fail_hip(ctx, L.err);
    return PSGD_OK;
}

int psgd_decompress_adam(psgd_ctx* ctx, void* workspace, void* stream, const float* const* P, const float* const* Q,
                         float* const* m1, float* const* m2, float* const* X, int step, float eta, float beta1,
                         float beta2, float eps, float weight_decay) {
    if (!ctx || !m1 || !m2 || !X) return PSGD_E_INVALID_ARG;
    if (step < 1 || !(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f) || !(eps >= 0.f) ||
        !(eta == eta) || !(weight_decay == weight_decay))
        return PSGD_E_INVALID_ARG;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const size_t nl = (size_t)ctx->n_layers;
    int rc = check_table(reinterpret_cast<const void* const*>(m1), nl);
    if (rc == PSGD_OK) rc = check_table(reinterpret_cast<const void* const*>(m2), nl);
    if (rc == PSGD_OK) rc = check_table(reinterpret_cast<const void* const*>(X), nl);
    if (rc != PSGD_OK) return rc;
    bool packed = false;
    rc = bind_factors(ctx, workspace, st, P, Q, &packed);
    if (rc != PSGD_OK) return rc;
    char* ws = reinterpret_cast<char*>(workspace);
    const bool changed = sync_table(ctx->hMom, m1, nl) | sync_table(ctx->hX, X, nl);
    if (changed || ctx->msgd_ws != workspace) {
        if (is_capturing(st)) { ctx->msgd_ws = nullptr; return PSGD_E_CAPTURE; }
        PSGD_TRY(launch_put(ws + ctx->off_moms, ctx->hMom.data(), nl * sizeof(void*), st));
        PSGD_TRY(launch_put(ws + ctx->off_xs, ctx->hX.data(), nl * sizeof(void*), st));
    }
    ctx->msgd_ws = workspace;
    if (sync_table(ctx->hM2, m2, nl) || ctx->m2_ws != workspace) {
        if (is_capturing(st)) { ctx->m2_ws = nullptr; return PSGD_E_CAPTURE; }
        PSGD_TRY(launch_put(ws + ctx->off_m2s, ctx->hM2.data(), nl * sizeof(void*), st));
    }
    ctx->m2_ws = workspace;
    // bias corrections in double: 1 - beta^t loses nothing for beta close to 1 and small t
    const double bc1 = 1.0 - std::pow((double)beta1, (double)step), bc2 = 1.0 - std::pow((double)beta2, (double)step);
    const float coef[8] = {beta1, beta2, (float)(1.0 - (double)beta1), (float)(1.0 - (double)beta2),
                           (float)((double)eta / bc1), (float)(1.0 / std::sqrt(bc2)), eps,
                           (float)((double)eta * (double)weight_decay)};
    Launcher L = batch_launcher(ctx, workspace, st);
    const int cp = ctx->cpc, nb = cp / 32;
    if (!packed) L.pack(ROLE_P, cp, Launcher::PACK_ROWMAJOR, ROLE_Q);
    const bool kept = packed && ctx->factors_kept;      // (see psgd_decompress)
    const int n_kept = !kept ? 0 : ctx->lazy_tr ? L.n_all : L.n_norm;
    const int* ids_kept = ctx->lazy_tr ? L.ids_all : L.ids_norm;
    float* const* d1 = reinterpret_cast<float* const*>(ws + ctx->off_moms);
    float* const* d2 = reinterpret_cast<float* const*>(ws + ctx->off_m2s);
    float* const* dx = reinterpret_cast<float* const*>(ws + ctx->off_xs);
    if (n_kept > 0) L.note(launch_adam(nb, ctx->planes, L.layers, ids_kept, n_kept, L.tiles_outer, d1, d2, dx, coef, true, st));
    if (!kept) L.note(launch_adam(nb, ctx->planes, L.layers, L.ids_all, L.n_all, L.tiles_outer, d1, d2, dx, coef, false, st));
    else if (!ctx->lazy_tr) L.note(launch_adam(nb, ctx->planes, L.layers, L.ids_tr, L.n_tr, L.tiles_outer, d1, d2, dx, coef, false, st));
    if (L.err != hipSuccess) return fail_hip(ctx, L.err);
    return PSGD_OK;
}

int psgd_status(psgd_ctx* ctx, void* workspace, void* stream, int layer, psgd_layer_status* out) {
    if (!ctx || !workspace || !out || layer < 0 || layer >= ctx->n_layers) return PSGD_E_INVALID_ARG;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    PSGD_TRY(hipStreamSynchronize(st));
    char* ws = reinterpret_cast<char*>(workspace);
    const LayerRegion R = layer_region(ctx, ctx->plan[layer]);
    int raw[kStatusWords] = {};
    PSGD_TRY(hipMemcpy(raw, ws + ctx->off_layer[layer] + R.status, sizeof(raw), hipMemcpyDeviceToHost));
    out->rank_deficient = raw[0];
    out->refresh_iters_next = raw[4];
    out->refresh_iters_no_gap = raw[25] < 2 ? 2 : raw[25];
    std::memcpy(&out->sigma_max, &raw[2], sizeof(float));
    std::memcpy(&out->sigma_r, &raw[3], sizeof(float));
    return PSGD_OK;
}

int psgd_copy_bytes(void* stream, void* dst, const void* src, size_t n_bytes) {
    if (!dst || !src || (n_bytes & 15u) || !aligned16(dst) || !aligned16(src)) return PSGD_E_INVALID_ARG;
    hipError_t e = launch_copy(dst, src, n_bytes, reinterpret_cast<hipStream_t>(stream));
    return e == hipSuccess ? PSGD_OK : PSGD_E_HIP;
}

int psgd_last_hip_error(const psgd_ctx* ctx) { return ctx ? ctx->last_hip : 0; }

const char* psgd_strerror(int code) {
    switch (code) {
        case PSGD_OK: return "ok";
        case PSGD_E_INVALID_ARG: return "invalid argument";
        case PSGD_E_SHAPE: return "unsupported shape or rank";
        case PSGD_E_ALIGN: return "leading dimension or pointer alignment";
        case PSGD_E_HIP: return "HIP runtime error";
        case PSGD_E_NOMEM: return "out of host memory";
        case PSGD_E_CAPTURE: return "stream capture: pointer tables not on the device yet (make the same call eagerly once first)";
        case PSGD_E_TOO_LARGE: return "the context needs more workspace than the library's built-in buffer holds";
        default: return "unknown error";
    }
}

int psgd_profile_enable(psgd_ctx* ctx, int max_records) {
    if (!ctx || max_records < 0 || max_records > (1 << 20)) return PSGD_E_INVALID_ARG;
    for (hipEvent_t e : ctx->prof_ev) (void)hipEventDestroy(e);
    ctx->prof_ev.clear();
    ctx->prof_tag.assign((size_t)max_records, 0);
    ctx->prof_used = 0;
    ctx->prof_on = max_records > 0;
    for (int i = 0; i < 2 * max_records; ++i) {
        hipEvent_t e;
        PSGD_TRY(hipEventCreate(&e));
        ctx->prof_ev.push_back(e);
    }
    return PSGD_OK;
}

int psgd_profile_select(psgd_ctx* ctx, int tag_mask) {
    if (!ctx || tag_mask < 0 || tag_mask >= (1 << PSGD_PROF_TAGS)) return PSGD_E_INVALID_ARG;
    ctx->prof_mask = tag_mask;
    return PSGD_OK;
}

int psgd_profile_read(psgd_ctx* ctx, double* total_ms, int* count, int n_tags) {
    if (!ctx || !total_ms || !count || n_tags < 1) return PSGD_E_INVALID_ARG;
    for (int t = 0; t < n_tags; ++t) { total_ms[t] = 0.0; count[t] = 0; }
    for (size_t k = 0; k < ctx->prof_used; ++k) {
        PSGD_TRY(hipEventSynchronize(ctx->prof_ev[2 * k + 1]));
        float ms = 0.f;
        PSGD_TRY(hipEventElapsedTime(&ms, ctx->prof_ev[2 * k], ctx->prof_ev[2 * k + 1]));
        const int t = ctx->prof_tag[k];
        if (t >= 0 && t < n_tags) { total_ms[t] += ms; count[t] += 1; }
    }
    ctx->prof_used = 0;
    return PSGD_OK;
}

void psgd_destroy(psgd_ctx* ctx) {
    if (!ctx) return;
    for (auto& F : ctx->fetch) {
        if (F.pending) (void)hipEventSynchronize(F.ev);
        if (F.ev) (void)hipEventDestroy(F.ev);
    }
    if (ctx->fetch[0].h) (void)hipHostFree(ctx->fetch[0].h);
    for (hipEvent_t e : ctx->prof_ev) (void)hipEventDestroy(e);
    delete ctx;
}

}  // extern "C"
