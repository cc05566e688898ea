// The forming pass on layers stored with rows >= cols, at compress-step widths (r <= 64):
//
//   M = (1/N) sum_i G^(i) + E      (Eq. (7a) averaged over the workers; stored in place of E)
//   P = M Q_{t-1}                  (Algorithm 1, SSP-Comp; also the first product of the refresh's iteration)
//
// and, with LAZY, the residual the previous step still owes on the way in (Algorithm 2, error update):
//   E = M_{t-1} - P~_{t-1} Q_{t-1}^T,  rounded to fp32 as a residual pass would have stored it.
//
// Geometry.  What bounds this pass is HBM, and what HBM gives depends on the run length per row: measured on this
// machine, an in-place "bf16 + fp32 -> fp32" walk reaches 4.8 TB/s with 64 columns per row and step, 5.6 with 256,
// and 6.2 with 256 and non-temporal stores.  A workgroup therefore owns 32 rows and walks them 256 columns at a time;
// every load and store instruction of a wavefront covers 1 KB of one row (512 bytes of a bf16 gradient).
// The four waves split the 256 columns of a step between them as the reduction range of the product (64 each) and
// add their partial results at the end.  M goes through LDS once (split into bf16 planes, in the layout of the MFMA A
// operand); the thin operand comes pre-split in MFMA fragment order (PackRef::t) and is loaded straight into
// registers, 1 KB per fragment, no LDS and no barrier of its own.  With two planes the A tile is double-buffered
// in LDS and a step has one barrier.
#include <type_traits>

#include "psgd_dev.h"

namespace psgd {

constexpr int FR = 32;          // rows of S per workgroup
constexpr int FK = 256;         // columns of S per step
constexpr int FLD = FK + 8;     // LDS row stride of an A plane (bf16 elements): rows 4 banks apart
constexpr int FDW = FK + 4;     // LDS row stride of the correction tile (fp32, LAZY)

template <int PL> __device__ inline bool form_keep_term(int ka, int kb) { return PL == 2 ? (ka + kb <= 1) : (ka + kb <= 2); }

__device__ inline floatx4 widen4(uintx2 v) {
    return floatx4{__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xffff0000u), __uint_as_float(v.y << 16),
                   __uint_as_float(v.y & 0xffff0000u)};
}
__device__ inline floatx4 widen4(floatx4 v) { return v; }

template <int NB, int PL, bool LAZY> constexpr int form_abuf() { return (PL == 2 && !LAZY) ? 2 : 1; }
template <int NB, int PL, bool LAZY> constexpr size_t form_lds_bytes() {
    const size_t a = (size_t)form_abuf<NB, PL, LAZY>() * PL * FR * FLD * sizeof(bf16_t);
    const size_t d = LAZY ? (size_t)FR * FDW * sizeof(float) : 0;
    const size_t red = (size_t)4 * FR * (32 * NB + 1) * sizeof(float);
    return a + d > red ? a + d : red;
}

// GBF: the gradients are bf16 (else fp32); ONEW: one worker (no loop over further gradient buffers);
// LAZY: the residual of the previous compress step is applied on the way in.
template <int NB, int PL, bool GBF, bool ONEW, bool LAZY>
__global__ __launch_bounds__(kThreads, 2) void form_row_kernel(const LayerDev* __restrict__ layers,
                                                                const int* __restrict__ ids, int out_role,
                                                                int epi_flags, int nt_m) {
    using GV = typename std::conditional<GBF, uintx2, floatx4>::type;
    using GT = typename std::conditional<GBF, bf16_t, float>::type;
    constexpr int cp = 32 * NB;
    constexpr int ABUF = form_abuf<NB, PL, LAZY>();
    constexpr int APL = FR * FLD;
    const LayerDev& L = layers[ids[blockIdx.y]];
    const bool store_m = !(epi_flags & EPI_KEEP_E);
    const int n_ob = L.rowsP / FR;                       // (row blocks past the end write the zeros of the padding)
    const int n_split = L.split_row_v2;
    const int tile = blockIdx.x;
    if (tile >= n_ob * n_split) return;
    const int sp = tile % n_split, ob = tile / n_split;
    const int row0 = ob * FR;
    const int n_chunks = (L.cols + FK - 1) / FK;
    const int cps = (n_chunks + n_split - 1) / n_split;
    const int ch0 = sp * cps;
    const int n_loc = row0 < L.rows ? max(min(n_chunks, ch0 + cps) - ch0, 0) : 0;

    extern __shared__ __align__(16) unsigned char smem[];
    bf16_t* a_pl = reinterpret_cast<bf16_t*>(smem);                              // ABUF x PL planes of [FR][FLD]
    float* d_lds = reinterpret_cast<float*>(a_pl + ABUF * PL * APL);             // [FR][FDW] (LAZY)

    const int t = threadIdx.x;
    const int lane = t & 63, wv = t >> 6;
    const int li = lane & 31, lg = lane >> 5;
    const float inv_n = ONEW ? 1.0f : 1.0f / (float)L.n_workers;
    const int nw = ONEW ? 1 : L.n_workers;
    const int64_t ld = L.ld;
    const int colsP = L.colsP;
    PSGD_GLOBAL float* S = as_global(L.S);
    // this thread's pieces of a tile: piece u at row row0 + 4 u + wv, columns ch * FK + 4 lane .. + 3
    const int64_t lane_off = (int64_t)(row0 + wv) * ld + 4 * lane;
    const int64_t ustep = 4 * ld;
    auto grad_ptr = [&](int w) { return reinterpret_cast<const PSGD_GLOBAL GT*>(as_global(as_global(L.G)[w])); };
    auto tile_full = [&](int ch) { return row0 + FR <= L.rows && ch * FK + FK <= L.cols; };
    auto piece_ok = [&](int ch, int u) { return row0 + 4 * u + wv < L.rows && ch * FK + 4 * lane < L.cols; };
    auto load_g = [&](int w, int ch, GV (&x)[8]) {
        const PSGD_GLOBAL GT* gp = grad_ptr(w) + lane_off + (int64_t)ch * FK;
        if (tile_full(ch)) {
#pragma unroll
            for (int u = 0; u < 8; ++u) x[u] = ld_stream<NT_G>(reinterpret_cast<const PSGD_GLOBAL GV*>(gp + u * ustep));
        } else {
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                x[u] = GV{};
                if (piece_ok(ch, u)) x[u] = ld_stream<NT_G>(reinterpret_cast<const PSGD_GLOBAL GV*>(gp + u * ustep));
            }
        }
    };
    auto load_e = [&](int ch, floatx4 (&x)[8]) {
        const PSGD_GLOBAL float* ep = S + lane_off + (int64_t)ch * FK;
        if (tile_full(ch)) {
#pragma unroll
            for (int u = 0; u < 8; ++u) x[u] = ld_stream<NT_E_IN>(reinterpret_cast<const PSGD_GLOBAL floatx4*>(ep + u * ustep));
        } else {
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                x[u] = floatx4{0.f, 0.f, 0.f, 0.f};
                if (piece_ok(ch, u)) x[u] = ld_stream<NT_E_IN>(reinterpret_cast<const PSGD_GLOBAL floatx4*>(ep + u * ustep));
            }
        }
    };
    // Each row block starts its walk at a step of its own and wraps around (consecutive blocks go to different XCDs,
    // the blocks of one XCD start near each other, every layer adds a phase): blocks walking in step would all be on
    // the same few memory channels, and this order keeps the thin operand chunks of the blocks that share an L2 close.
    const int rot = n_loc > 0 ? ((ob & 7) * (n_loc >> 3) + 2 * (ob >> 3) + (int)blockIdx.y) % n_loc : 0;
    auto chunk_at = [&](int it) { const int c = it + rot; return ch0 + (c >= n_loc ? c - n_loc : c); };

    // thin operand: this wave's fragments for its 64 columns of the step, four k-steps of 16
    const PackRef XK = L.pack[SIDE_W];
    bf16x8 bfrag[4][NB][PL];
    auto load_b = [&](int ch) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const int kg = ch * (FK / 16) + 4 * wv + ks;
            const bool ok = 16 * kg < colsP;                  // (uniform; past the padded length M is zero anyway)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int k = 0; k < PL; ++k) {
                    bfrag[ks][nb][k] = bf16x8{};
                    if (ok) bfrag[ks][nb][k] = *reinterpret_cast<const PSGD_GLOBAL bf16x8*>(
                                as_global(XK.t[k]) + (((int64_t)kg * NB + nb) * 64 + lane) * 8);
                }
        }
    };
    // LAZY: the rows of the kept P~ copy this workgroup owns stay in registers (A operand of the correction, all
    // k-steps); the kept Q rows of a step's columns are the B operand, loaded per step like the thin operand above.
    // Wave v forms the correction for columns 64 v .. 64 v + 63 of the step.
    bf16x8 pres[LAZY ? 2 * NB : 1][PL];
    if (LAZY) {
#pragma unroll
        for (int ks = 0; ks < 2 * NB; ++ks)
#pragma unroll
            for (int k = 0; k < PL; ++k)
                pres[ks][k] = *reinterpret_cast<const PSGD_GLOBAL bf16x8*>(
                    as_global(L.lz[SIDE_L][k]) + (int64_t)(row0 + li) * cp + 16 * ks + 8 * lg);
    }
    auto correction = [&](int ch) {
        // d_lds[row][col] = sum_k P~[row0 + row][k] Q[ch * FK + col][k] for this wave's 64 columns
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            floatx16 d;
#pragma unroll
            for (int v = 0; v < 16; ++v) d[v] = 0.f;
            const int col = ch * FK + 64 * wv + 32 * q + li;
            const bool ok = col < colsP;
#pragma unroll
            for (int ks = 0; ks < 2 * NB; ++ks) {
                bf16x8 qv[PL];
#pragma unroll
                for (int k = 0; k < PL; ++k) {
                    qv[k] = bf16x8{};
                    if (ok) qv[k] = *reinterpret_cast<const PSGD_GLOBAL bf16x8*>(
                                as_global(L.lz[SIDE_W][k]) + (int64_t)col * cp + 16 * ks + 8 * lg);
                }
#pragma unroll
                for (int sum = 2 * (PL - 1); sum >= 0; --sum)
#pragma unroll
                    for (int ka = 0; ka < PL; ++ka) {
                        const int kb = sum - ka;
                        if (kb >= 0 && kb < PL && form_keep_term<PL>(ka, kb))
                            d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pres[ks][ka], qv[kb], d, 0, 0, 0);
                    }
            }
#pragma unroll
            for (int v = 0; v < 16; ++v)
                d_lds[(8 * (v >> 2) + 4 * lg + (v & 3)) * FDW + 64 * wv + 32 * q + li] = d[v];
        }
    };

    floatx16 acc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[nb][v] = 0.f;

    floatx4 e[8];
    GV g[8];
    if (n_loc > 0) {
        load_e(chunk_at(0), e);
        load_g(0, chunk_at(0), g);
        load_b(chunk_at(0));
        if (LAZY) {
            correction(chunk_at(0));
            __syncthreads();                 // (later steps: the barrier that ends the step before)
        }
    }
    for (int it = 0; it < n_loc; ++it) {
        const int ch = chunk_at(it);
        bf16_t* a_cur = a_pl + (ABUF == 2 ? (it & 1) * PL * APL : 0);
        // ---- M = mean G + E in registers
        floatx4 m[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) m[u] = widen4(g[u]);
        if (!ONEW) {
            if (NB == 1 && GBF) {
                // two workers' loads in flight where the registers allow it
                GV xa[8], xb[8];
                int w = 1;
                if (w < nw) load_g(w, ch, xa);
                for (; w + 1 < nw; w += 2) {
                    load_g(w + 1, ch, xb);
#pragma unroll
                    for (int u = 0; u < 8; ++u) m[u] += widen4(xa[u]);
                    if (w + 2 < nw) load_g(w + 2, ch, xa);
#pragma unroll
                    for (int u = 0; u < 8; ++u) m[u] += widen4(xb[u]);
                }
                if (w < nw) {
#pragma unroll
                    for (int u = 0; u < 8; ++u) m[u] += widen4(xa[u]);
                }
            } else {
                for (int w = 1; w < nw; ++w) {
                    GV x[8];
                    load_g(w, ch, x);
#pragma unroll
                    for (int u = 0; u < 8; ++u) m[u] += widen4(x[u]);
                }
            }
        }
        if (LAZY) {
            // E = M_{t-1} - (rank-r product), rounded to fp32 here as the residual pass would have stored it
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const floatx4 d = *reinterpret_cast<const floatx4*>(d_lds + (4 * u + wv) * FDW + 4 * lane);
                e[u] -= d;
            }
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) m[u] = m[u] * inv_n + e[u];
        const bool full = tile_full(ch);
        if (!full) {
            // pieces outside the matrix were loaded as zero; cut the column tail (the padding up to ld is not data)
            const int c = ch * FK + 4 * lane;
            const bool k1 = c + 1 < L.cols, k2 = c + 2 < L.cols, k3 = c + 3 < L.cols;
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                m[u].y = k1 ? m[u].y : 0.f;
                m[u].z = k2 ? m[u].z : 0.f;
                m[u].w = k3 ? m[u].w : 0.f;
            }
        }
        // ---- M back in place of E
        if (store_m) {
            PSGD_GLOBAL float* mp = S + lane_off + (int64_t)ch * FK;
            if (full) {
                if (nt_m) {
#pragma unroll
                    for (int u = 0; u < 8; ++u) __builtin_nontemporal_store(m[u], reinterpret_cast<PSGD_GLOBAL floatx4*>(mp + u * ustep));
                } else {
#pragma unroll
                    for (int u = 0; u < 8; ++u) *reinterpret_cast<PSGD_GLOBAL floatx4*>(mp + u * ustep) = m[u];
                }
            } else {
                const int c = ch * FK + 4 * lane;
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    if (!piece_ok(ch, u)) continue;
                    PSGD_GLOBAL float* p = mp + u * ustep;
                    if (c + 3 < L.cols) {
                        *reinterpret_cast<PSGD_GLOBAL floatx4*>(p) = m[u];
                    } else {
                        p[0] = m[u].x;
                        if (c + 1 < L.cols) p[1] = m[u].y;
                        if (c + 2 < L.cols) p[2] = m[u].z;
                    }
                }
            }
        }
        // ---- split into planes -> LDS, [row][k] with k contiguous
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            bf16x4 o[PL];
            bf16_t q[PL];
            split_planes<PL>(m[u].x, q);
#pragma unroll
            for (int k = 0; k < PL; ++k) o[k][0] = q[k];
            split_planes<PL>(m[u].y, q);
#pragma unroll
            for (int k = 0; k < PL; ++k) o[k][1] = q[k];
            split_planes<PL>(m[u].z, q);
#pragma unroll
            for (int k = 0; k < PL; ++k) o[k][2] = q[k];
            split_planes<PL>(m[u].w, q);
#pragma unroll
            for (int k = 0; k < PL; ++k) o[k][3] = q[k];
#pragma unroll
            for (int k = 0; k < PL; ++k) *reinterpret_cast<bf16x4*>(a_cur + k * APL + (4 * u + wv) * FLD + 4 * lane) = o[k];
        }
        __syncthreads();
        // ---- the next step's tile goes out now and is in flight during the MFMA phase
        if (it + 1 < n_loc) {
            load_e(chunk_at(it + 1), e);
            load_g(0, chunk_at(it + 1), g);
        }
        // ---- MFMA: 32 rows x cp columns, this wave's 64 of the step's 256 reduction indices
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            bf16x8 av[PL];
#pragma unroll
            for (int k = 0; k < PL; ++k)
                av[k] = *reinterpret_cast<const bf16x8*>(a_cur + k * APL + li * FLD + 64 * wv + 16 * ks + 8 * lg);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int sum = 2 * (PL - 1); sum >= 0; --sum)      // smallest products first
#pragma unroll
                    for (int ka = 0; ka < PL; ++ka) {
                        const int kb = sum - ka;
                        if (kb >= 0 && kb < PL && form_keep_term<PL>(ka, kb))
                            acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[ka], bfrag[ks][nb][kb], acc[nb], 0, 0, 0);
                    }
        }
        // ---- the next step's thin operand fragments (their registers are free now), and its correction
        if (it + 1 < n_loc) {
            load_b(chunk_at(it + 1));
            if (LAZY) correction(chunk_at(it + 1));       // (d_lds was last read before this step's barrier)
        }
        if (ABUF == 1) __syncthreads();
    }
    // ---- add the four waves' partial results
    __syncthreads();
    float* red = reinterpret_cast<float*>(smem);          // [4][FR][cp + 1]
    constexpr int RW = cp + 1;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int v = 0; v < 16; ++v)
            red[(wv * FR + 8 * (v >> 2) + 4 * lg + (v & 3)) * RW + 32 * nb + li] = acc[nb][v];
    __syncthreads();
    const ThinRef T = L.thin[out_role];
    auto total = [&](int row, int col) {
        const float* r = red + row * RW + col;
        return (r[0] + r[FR * RW]) + (r[2 * FR * RW] + r[3 * FR * RW]);
    };
    if (n_split > 1) {
        // one of n_split partial sums: [split][column][row]; finish_kernel adds them up in split order
        PSGD_GLOBAL float* dst = as_global(L.part[SIDE_L]) + (int64_t)sp * L.rowsP * T.width + row0;
        for (int i = t; i < FR * T.width; i += kThreads) {
            const int row = i & (FR - 1), col = i / FR;
            dst[(int64_t)col * L.rowsP + row] = total(row, col);
        }
    } else {
        for (int i = t; i < FR * T.width; i += kThreads) {
            const int row = i / T.width, col = i - row * T.width;
            if (row0 + row < L.rows) as_global(T.ptr)[(int64_t)(row0 + row) * T.ld + col] = total(row, col);
        }
    }
}

template <int NB, int PL>
static hipError_t launch_form_nb(bool gbf, bool onew, bool lazy, const LayerDev* layers, const int* ids, int n_ids,
                                 int max_tiles, int out_role, int epi, int nt_m, hipStream_t st) {
    dim3 grid(max_tiles, n_ids), block(kThreads);
#define PSGD_FORM(GBF, ONEW, LAZY)                                                                             \
    do {                                                                                                       \
        auto kfn = form_row_kernel<NB, PL, GBF, ONEW, LAZY>;                                                   \
        const size_t lds = form_lds_bytes<NB, PL, LAZY>();                                                     \
        if (lds > 48 * 1024) {                                                                                 \
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kfn),                             \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);          \
            if (e != hipSuccess) return e;                                                                     \
        }                                                                                                      \
        hipLaunchKernelGGL(kfn, grid, block, lds, st, layers, ids, out_role, epi, nt_m);                       \
    } while (0)
    if (lazy) {
        if (gbf) { if (onew) PSGD_FORM(true, true, true); else PSGD_FORM(true, false, true); }
        else     { if (onew) PSGD_FORM(false, true, true); else PSGD_FORM(false, false, true); }
    } else {
        if (gbf) { if (onew) PSGD_FORM(true, true, false); else PSGD_FORM(true, false, false); }
        else     { if (onew) PSGD_FORM(false, true, false); else PSGD_FORM(false, false, false); }
    }
#undef PSGD_FORM
    return hipGetLastError();
}

// Variants this kernel is built for: the thin operand fragments of a whole step live in registers next to the tile,
// which the wider and the several-fp32-worker variants cannot afford without spilling.
bool form_row_supported(int nb, int planes, bool gbf, bool onew, bool lazy) {
    if (nb < 1 || nb > 2) return false;
    const bool f32_multi = !gbf && !onew;
    if (nb == 1) return !(planes == 3 && lazy && f32_multi);
    if (planes == 2) return !f32_multi;
    return !lazy && !f32_multi;
}

// nb = width / 32 of the thin operand (1 or 2); gbf: every layer of the launch has bf16 gradients (else every layer
// fp32); onew: one worker; lazy: apply the owed residual on the way in; nt_m: store M with the non-temporal hint
// (matrices too large to be found in a cache by the second pass).  max_tiles: max over the layers of
// (padded rows / 32) * split_row_v2.
hipError_t launch_form_row(int nb, int planes, bool gbf, bool onew, bool lazy, const LayerDev* layers, const int* ids,
                           int n_ids, int max_tiles, int out_role, int epi, int nt_m, hipStream_t st) {
    if (n_ids <= 0 || max_tiles <= 0) return hipSuccess;
    if (nb == 1) return planes == 2 ? launch_form_nb<1, 2>(gbf, onew, lazy, layers, ids, n_ids, max_tiles, out_role, epi, nt_m, st)
                                    : launch_form_nb<1, 3>(gbf, onew, lazy, layers, ids, n_ids, max_tiles, out_role, epi, nt_m, st);
    if (nb == 2) return planes == 2 ? launch_form_nb<2, 2>(gbf, onew, lazy, layers, ids, n_ids, max_tiles, out_role, epi, nt_m, st)
                                    : launch_form_nb<2, 3>(gbf, onew, lazy, layers, ids, n_ids, max_tiles, out_role, epi, nt_m, st);
    return hipErrorInvalidValue;
}

}  // namespace psgd
