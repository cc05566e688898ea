// Tall-skinny products of the power iteration on MFMA (gfx950), one streaming pass over S each.
//
//   row mode    Y_L = S   X_W      (rows x w) = (rows x cols)(cols x w)     e.g. P = M Q      (Algorithm 1)
//   column mode Y_W = S^T X_L      (cols x w) = (cols x rows)(rows x w)     e.g. Q = M^T P~   (Algorithm 1)
//
// With FORM the pass also forms M = (1/N) sum_i G^(i) + E (Eq. (7a) averaged over the workers)
// from the gradient buffers and the error buffer, uses it for the product and (unless the launch
// carries EPI_KEEP_E) stores it in place of E, so that the second pass and the residual read 4 bytes
// per element instead of N*sizeof(G)+4.
//
// Arithmetic: M and X are split into two or three bf16 planes each (x = p0 + p1 (+ p2), each plane the
// rounded remainder of the ones before: 16 or 24 mantissa bits) and the product is accumulated in
// fp32 from the plane products with plane-index sum <= 1 (three products) or <= 2 (six), smallest
// first, with v_mfma_f32_32x32x16_bf16.
// The S tile goes global -> registers (coalesced 16-byte loads, summed over workers) -> LDS in the
// k-contiguous layout the MFMA A operand wants; the thin operand arrives pre-split and transposed.
#include <type_traits>

#include "thin_dev.h"

namespace psgd {

constexpr int BK = 64;          // reduction chunk
constexpr int BT = 128;         // output rows per workgroup (4 waves x 32)
constexpr int LDSW = BK + 8;    // LDS row stride in bf16 elements (144 bytes)

template <int NT = 0>
__device__ inline float4 ld_f32x4(const PSGD_GLOBAL float* p) {
    const floatx4 v = ld_stream<NT>(reinterpret_cast<const PSGD_GLOBAL floatx4*>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}

template <int NT = 0>
__device__ inline float4 ld_bf16x4(const PSGD_GLOBAL bf16_t* p) {
    const uintx2 v = ld_stream<NT>(reinterpret_cast<const PSGD_GLOBAL uintx2*>(p));
    float4 o;
    o.x = __uint_as_float(v.x << 16);
    o.y = __uint_as_float(v.x & 0xffff0000u);
    o.z = __uint_as_float(v.y << 16);
    o.w = __uint_as_float(v.y & 0xffff0000u);
    return o;
}

// A thread's share of one S tile: eight 4-element pieces, piece u at (row0 + u*row_step, col).  The
// address of piece u is (uniform part: tile origin + u * ustep) + (this thread's offset inside the tile),
// so that the eight addresses cost one 32-bit register.  Tiles that lie inside the matrix (`full`, uniform)
// take unpredicated loads; ragged ones load under a per-piece predicate and mask the column tail afterwards
// (the padding up to ld and rows past the end are not data).
struct TileAddr {
    int64_t origin;     // element offset of the tile's first element
    int64_t ustep;      // elements between a thread's consecutive pieces (row_step * ld)
    unsigned lane;      // element offset of this thread's piece 0 from the origin (< 2^30)
    int row0, row_step, col;
    bool full;
    bool quad;          // pieces at rows row0 + {0,1,2,3, 16,17,18,19} (rows of two 16 x 16 MFMA accumulator
                        // blocks) instead of row0 + u * row_step
};

// multiple of ustep that leads to piece u
__device__ inline int piece_mul(const TileAddr& a, int u) { return a.quad ? (u & 3) + 16 * (u >> 2) : u; }
// row of piece u relative to row0
__device__ inline int piece_row(const TileAddr& a, int u) { return a.quad ? (u & 3) + 16 * (u >> 2) : u * a.row_step; }

__device__ inline TileAddr tile_addr(const LayerDev& L, int tile_row0, int tile_col0, int tile_rows, int tile_cols,
                                     int lane_row, int row_step, int lane_col) {
    TileAddr a;
    a.origin = (int64_t)tile_row0 * L.ld + tile_col0;
    a.ustep = (int64_t)row_step * L.ld;
    a.lane = (unsigned)lane_row * (unsigned)L.ld + (unsigned)lane_col;
    a.row0 = tile_row0 + lane_row;
    a.row_step = row_step;
    a.col = tile_col0 + lane_col;
    a.full = tile_row0 + tile_rows <= L.rows && tile_col0 + tile_cols <= L.cols;
    a.quad = false;
    return a;
}

// the layout of the pass that also applies the pending rank-r correction: piece u of a thread sits at row
// lane_row + (u & 3) + 16 * (u >> 2); ustep then holds one row
__device__ inline TileAddr tile_addr_quad(const LayerDev& L, int tile_row0, int tile_col0, int tile_rows, int tile_cols,
                                          int lane_row, int lane_col) {
    TileAddr a = tile_addr(L, tile_row0, tile_col0, tile_rows, tile_cols, lane_row, 1, lane_col);
    a.quad = true;
    return a;
}

__device__ inline bool piece_ok(const LayerDev& L, const TileAddr& a, int u) {
    return a.col < L.cols && a.row0 + piece_row(a, u) < L.rows;
}

// eight pieces of a row-major matrix of T (float or bf16) with the layer's leading dimension, widened to fp32
template <int NT, class T>
__device__ inline void load8(const LayerDev& L, const PSGD_GLOBAL T* base, const TileAddr& a, float4 (&x)[8]) {
    const PSGD_GLOBAL char* b = reinterpret_cast<const PSGD_GLOBAL char*>(base + a.origin);
    const unsigned lb = a.lane * (unsigned)sizeof(T);
    const int64_t sb = a.ustep * (int64_t)sizeof(T);
    if (a.full) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const PSGD_GLOBAL T* p = reinterpret_cast<const PSGD_GLOBAL T*>(b + piece_mul(a, u) * sb + lb);
            if constexpr (sizeof(T) == 4) x[u] = ld_f32x4<NT>(p); else x[u] = ld_bf16x4<NT>(p);
        }
    } else {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            x[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (piece_ok(L, a, u)) {
                const PSGD_GLOBAL T* p = reinterpret_cast<const PSGD_GLOBAL T*>(b + piece_mul(a, u) * sb + lb);
                if constexpr (sizeof(T) == 4) x[u] = ld_f32x4<NT>(p); else x[u] = ld_bf16x4<NT>(p);
            }
        }
    }
}

__device__ inline void load_g8(const LayerDev& L, int w, const TileAddr& a, float4 (&x)[8]) {
    const PSGD_GLOBAL void* gw = as_global(as_global(L.G)[w]);
    if (L.gdt == 0) load8<NT_G>(L, reinterpret_cast<const PSGD_GLOBAL float*>(gw), a, x);
    else load8<NT_G>(L, reinterpret_cast<const PSGD_GLOBAL bf16_t*>(gw), a, x);
}

__device__ inline void add8(float4 (&m)[8], const float4 (&x)[8]) {
#pragma unroll
    for (int u = 0; u < 8; ++u) { m[u].x += x[u].x; m[u].y += x[u].y; m[u].z += x[u].z; m[u].w += x[u].w; }
}

// First half of a tile load, issued before the MFMA phase of the previous chunk so that the loads
// are in flight while the matrix cores work: the S tile itself (!FORM), or worker 0's gradient and E.
template <bool FORM>
__device__ inline void tile_prefetch(const LayerDev& L, const TileAddr& a, float4 (&p0)[8], float4 (&p1)[8]) {
    if (FORM) {
        load_g8(L, 0, a, p0);
        load8<NT_E_IN>(L, as_global(L.S), a, p1);
    } else {
        load8<NT_S_PROD>(L, as_global(L.S), a, p0);
    }
}

// Second half: the remaining workers, the mean, + E, the mask.  The sum over the workers runs in worker order.
// ONEW: compiled for a single worker (no loop over further gradient buffers, and no registers kept for them)
template <bool FORM, bool PIPE, bool ONEW = false>
__device__ inline void tile_finish(const LayerDev& L, const TileAddr& a, float inv_n, const float4 (&p0)[8],
                                   const float4 (&p1)[8], float4 (&m)[8]) {
#pragma unroll
    for (int u = 0; u < 8; ++u) m[u] = p0[u];
    if (FORM) {
        const int nw = ONEW ? 1 : L.n_workers;
        if (ONEW) {
        } else if (PIPE) {
            // two workers' loads in flight: the next worker is requested before the current one is added
            // (where the registers allow it: narrow output blocks)
            float4 xa[8], xb[8];
            int w = 1;
            if (w < nw) load_g8(L, w, a, xa);
            for (; w + 1 < nw; w += 2) {
                load_g8(L, w + 1, a, xb);
                add8(m, xa);
                if (w + 2 < nw) load_g8(L, w + 2, a, xa);
                add8(m, xb);
            }
            if (w < nw) add8(m, xa);
        } else {
            for (int w = 1; w < nw; ++w) {
                float4 x[8];
                load_g8(L, w, a, x);
                add8(m, x);
            }
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            m[u].x = m[u].x * inv_n + p1[u].x; m[u].y = m[u].y * inv_n + p1[u].y;
            m[u].z = m[u].z * inv_n + p1[u].z; m[u].w = m[u].w * inv_n + p1[u].w;
        }
    }
    if (!a.full) {
        // pieces outside the matrix were loaded as zero (and 0 * inv_n + 0 = 0); cut the column tail
        const bool k1 = a.col + 1 < L.cols, k2 = a.col + 2 < L.cols, k3 = a.col + 3 < L.cols;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            m[u].y = k1 ? m[u].y : 0.f;
            m[u].z = k2 ? m[u].z : 0.f;
            m[u].w = k3 ? m[u].w : 0.f;
        }
    }
}

// M back in place of E, same addressing as the loads
__device__ inline void store_m8(const LayerDev& L, const TileAddr& a, const float4 (&m)[8]) {
    PSGD_GLOBAL char* b = reinterpret_cast<PSGD_GLOBAL char*>(as_global(L.S) + a.origin);
    const unsigned lb = a.lane * 4u;
    const int64_t sb = a.ustep * 4;
    if (a.full) {
#pragma unroll
        for (int u = 0; u < 8; ++u)
            st_stream<NT_M_OUT>(reinterpret_cast<PSGD_GLOBAL floatx4*>(b + piece_mul(a, u) * sb + lb), floatx4{m[u].x, m[u].y, m[u].z, m[u].w});
    } else {
        const bool k1 = a.col + 1 < L.cols, k2 = a.col + 2 < L.cols, k3 = a.col + 3 < L.cols;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            if (!piece_ok(L, a, u)) continue;
            PSGD_GLOBAL float* p = reinterpret_cast<PSGD_GLOBAL float*>(b + piece_mul(a, u) * sb + lb);
            if (k3) {
                st_stream<NT_M_OUT>(reinterpret_cast<PSGD_GLOBAL floatx4*>(p), floatx4{m[u].x, m[u].y, m[u].z, m[u].w});
            } else {
                p[0] = m[u].x;
                if (k1) p[1] = m[u].y;
                if (k2) p[2] = m[u].z;
            }
        }
    }
}

// Epilogue on a complete 128 x cp output tile held in LDS as fp32 [BT][tw]: store the rows of the
// thin result, then either the partial Gram matrix of these rows (fp64, upper triangle, slot = block
// index) or the split-bf16 operand copies of the rows.  Called by all threads of the workgroup.
__device__ inline void tile_epilogue(const LayerDev& L, const ThinRef& T, int out_side, int ob, int out_len,
                                     int out_lenP, int cp, int epi, const float* otile, int tw, bool kept = false) {
    const int t = threadIdx.x;
    const int w = T.width;
    for (int e = t; e < BT * w; e += kThreads) {
        const int row = e / w, col = e % w;
        if (ob * BT + row < out_len) as_global(T.ptr)[(int64_t)(ob * BT + row) * T.ld + col] = otile[row * tw + col];
    }
    if (epi == EPI_GRAM) {
        gram_tile_f64(otile, tw, BT, w, L.gram + (int64_t)ob * ((w * (w + 1)) / 2));
    } else if (epi == EPI_PACK) {
        write_packs(L.pack[out_side], L.planes, otile, tw, cp, ob * BT, BT, out_lenP, 3, kept ? L.lzf[out_side] : nullptr);
    }
}

// MFMA products kept per pair of split operands: with two planes hi*hi + lo*hi + hi*lo, with three
// planes also mid*mid and the two products with the third plane (everything down to 2^-24).
// Column mode writes the A tile with 16-byte LDS stores whose lanes are 4 tile rows apart; with the
// plain padded layout every other lane would hit the same banks.  The 16-byte chunk index within a
// row is therefore XOR-ed with bits 3..5 of the row index (same function on the read side).
template <bool COLMODE> __device__ inline int a_chunk(int row, int chunk) { return COLMODE ? (chunk ^ ((row >> 3) & 7)) : chunk; }

template <int PL> __device__ inline bool keep_term(int ka, int kb) { return PL == 2 ? (ka + kb <= 1) : (ka + kb <= 2); }

// Two workgroups share a compute unit when their operand buffers fit its 160 KB of LDS twice; the wide
// variants run alone and may use the whole register file.
constexpr int prod_min_blocks(int nb, int pl) { return 2 * pl * (BT + 32 * nb) * LDSW * 2 <= 160 * 1024 ? 2 : 1; }

// LAZY (FORM): the buffer S holds M_{t-1} and the residual of the previous step is still owed,
// E_t = M_{t-1} - P~_{t-1} Q_{t-1}^T (Algorithm 2, error update).  The pass applies it on the way: the rank-r
// product for the tile comes from the kept operand copies of the two thin matrices -- the one on the side the
// workgroup owns (its 128 rows in row mode, 128 columns in column mode) in registers for the whole pass, the
// chunk's 64 rows of the other one staged in LDS -- on v_mfma_f32_16x16x32_bf16, whose accumulator layout
// -- lane (j, g) holds rows 4g..4g+3 of column j -- with block q bound to matrix columns 4j + q gives every
// lane 4 consecutive columns of 8 rows: the layout the tile is loaded in.  Column mode: width 32 only (the
// resident operand is four blocks wide there, twice the registers of row mode).
template <int NB, int PL> constexpr int prod_lds_elems(bool lazy) {
    return PL * (BT + 32 * NB) * LDSW + (lazy ? PL * BK * (32 * NB + 8) : 0);
}

template <int NB, int PL, bool COLMODE, bool FORM, bool LAZY = false, bool ONEW = false>
__global__ __launch_bounds__(kThreads, (prod_lds_elems<NB, PL>(LAZY) * 4 <= 160 * 1024 ? 2 : 1)) void prod_kernel(const LayerDev* __restrict__ layers,
                                                        const int* __restrict__ ids, int cp, int out_role,
                                                        int epi_flags, int gate) {
    const LayerDev& L = layers[ids[blockIdx.y]];
    if (!gate_open(L, gate)) return;
    const int epi = epi_flags & EPI_KIND_MASK;
    const bool store_m = FORM && !(epi_flags & EPI_KEEP_E);
    const int out_side = COLMODE ? SIDE_W : SIDE_L;
    const int src_side = COLMODE ? SIDE_L : SIDE_W;
    const int out_len = COLMODE ? L.cols : L.rows;
    const int red_len = COLMODE ? L.rows : L.cols;
    const int n_ob = (out_len + BT - 1) / BT;
    const int n_split = FORM ? (COLMODE ? L.split_col_f : L.split_row_f) : (COLMODE ? L.split_col : L.split_row);
    const int tile = blockIdx.x;
    if (tile >= n_ob * n_split) return;
    int ob, sp;
    if (COLMODE) { ob = tile % n_ob; sp = tile / n_ob; }
    else         { sp = tile % n_split; ob = tile / n_split; }
    const int n_chunks = (red_len + BK - 1) / BK;
    const int cps = (n_chunks + n_split - 1) / n_split;
    const int ch0 = sp * cps;
    const int ch1 = min(n_chunks, ch0 + cps);

    extern __shared__ __align__(16) unsigned char smem[];
    bf16_t* a_pl = reinterpret_cast<bf16_t*>(smem);          // PL planes of [BT][LDSW]
    bf16_t* b_pl = a_pl + PL * BT * LDSW;                    // PL planes of [32 NB][LDSW]
    constexpr int APL = BT * LDSW, BPL = NB * 32 * LDSW;

    const int t = threadIdx.x;
    const int lane = t & 63, wv = t >> 6;
    const int li = lane & 31, lg = lane >> 5;
    const int lj = lane & 15, lq = lane >> 4;     // lane coordinates of the 16 x 16 MFMA blocks (LAZY)
    static_assert(!ONEW || FORM, "the single-worker variants are forming passes");
    const float inv_n = ONEW ? 1.0f : 1.0f / (float)L.n_workers;
    const PackRef XK = L.pack[src_side];
    static_assert(!LAZY || (FORM && (!COLMODE || NB == 1)), "the pending correction is applied by a forming pass");
    constexpr int CPW = 32 * NB + 8;                         // LDS row stride of the correction's column operand
    constexpr int CPL = BK * CPW;                            // one plane of it
    bf16_t* c_pl = b_pl + PL * NB * 32 * LDSW;               // PL planes of [BK][CPW] (LAZY only)

    floatx16 acc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[nb][v] = 0.f;

    // thread's position in the S tile: row mode 16 x 16 threads over (row, 4 columns), 8 rows 16 apart;
    // column mode 8 x 32 threads over (8 consecutive rows, 4 columns)
    // (LAZY: wave v owns rows 32v..32v+31 as two 16-row accumulator blocks, lane (j, g) rows 4g..4g+3 of each)
    // (LAZY, column mode: wave v owns rows 32 (v & 1) .. +31 of the chunk and columns 64 (v >> 1) .. +63)
    const int c4 = LAZY ? (COLMODE ? 16 * (wv >> 1) + lj : lj) : COLMODE ? (t & 31) : (t & 15);
    const int r0 = LAZY ? (COLMODE ? 32 * (wv & 1) + 4 * lq : 32 * wv + 4 * lq)
                        : COLMODE ? (t >> 5) : (t >> 4);       // row group in column mode
    auto addr_of = [&](int ch) {
        const int k0 = ch * BK;
        if (LAZY) return COLMODE ? tile_addr_quad(L, k0, ob * BT, BK, BT, r0, 4 * c4)
                                 : tile_addr_quad(L, ob * BT, k0, BT, BK, r0, 4 * c4);
        return COLMODE ? tile_addr(L, k0, ob * BT, BK, BT, 8 * r0, 1, 4 * c4)
                       : tile_addr(L, ob * BT, k0, BT, BK, r0, 16, 4 * c4);
    };
    // LAZY: this wave's part of the kept operand copy on the side the workgroup owns stays in registers for the
    // whole pass (row mode: 2 blocks of 16 rows; column mode: 4 blocks of 16 columns, block q = columns 4j + q);
    // the chunk's 64 rows of the other kept copy are requested one chunk ahead and staged in LDS -- in row mode
    // matrix column c at LDS row (c & 3) * 16 + (c >> 2), so that the 16 lanes of an MFMA block read 16
    // consecutive LDS rows; in column mode matrix row by matrix row
    constexpr int NRES = COLMODE ? 4 : 2;
    bf16x8 ap[LAZY ? NRES : 1][LAZY ? NB : 1][PL];
    uintx4 cq[LAZY ? NB : 1][PL];
    auto corr_prefetch = [&](int ch) {
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int v = t + i * kThreads;          // 0 .. 64 * 4 NB - 1
            const int c = v / (4 * NB), part = v % (4 * NB);
            const int64_t goff = frag_piece(ch * BK + c, part, cp) * 8;      // (the kept copies are in fragment order)
#pragma unroll
            for (int k = 0; k < PL; ++k)
                cq[i][k] = *reinterpret_cast<const PSGD_GLOBAL uintx4*>(as_global(L.lzf[src_side][k]) + goff);
        }
    };
    auto load_ap = [&]() {
#pragma unroll
        for (int h = 0; h < NRES; ++h)
#pragma unroll
            for (int ks = 0; ks < NB; ++ks)
#pragma unroll
                for (int k = 0; k < PL; ++k) {
                    const int own = COLMODE ? 64 * (wv >> 1) + 4 * lj + h : 32 * wv + 16 * h + lj;   // row / column of the tile
                    ap[h][ks][k] = *reinterpret_cast<const PSGD_GLOBAL bf16x8*>(
                        as_global(L.lzf[out_side][k]) + frag_piece(ob * BT + own, 4 * ks + lq, cp) * 8);
                }
    };
    if (LAZY) load_ap();
    // Row mode: workgroups that run at the same time own different row blocks and would all be at the same
    // column offset within their rows, i.e. on the same few memory channels (the row stride is a large power of
    // two); each row block therefore starts its walk at a chunk of its own and wraps around.  Column mode needs
    // nothing of the kind: there the workgroups running together cover whole rows.
    const int n_loc = ch1 - ch0;
    // Which chunk: consecutive row blocks go to different XCDs (8 of them), so the blocks that share an L2 are
    // ob = 8 j + x for fixed x.  XCD x starts an eighth of the walk further on than XCD x - 1, within an XCD block
    // j starts 2 j chunks after block 0, and every layer adds a phase of its own: the workgroups in flight are
    // spread over the channels, while the blocks of one layer on one XCD read nearby chunks of the thin operands
    // at any time and find in the L2 what a neighbour fetched a little earlier.  (With every block on an unrelated
    // walk the operands of the ~16 layers in flight do not fit the L2 and come from memory again and again: the
    // deferred residual's operand alone costs 1.4 ms of a 13.7 ms pass.  What this order takes off it, 0.3 ms or
    // so, is within the run-to-run spread of the pass.)
    const int rot = (COLMODE || n_loc <= 0) ? 0
                    : ((ob & 7) * (n_loc >> 3) + 2 * (ob >> 3) + (int)blockIdx.y) % n_loc;
    auto chunk_at = [&](int it) { const int c = it + rot; return ch0 + (c >= n_loc ? c - n_loc : c); };
    // thin operand chunk: pre-split, in MFMA fragment order (PackRef::t: a 64-row chunk is one run of 64 cp elements);
    // requested one chunk ahead, before the tile's own loads
    // (the wait counter is in issue order: waiting for the chunk then leaves the tile's loads in flight)
    // (only where the registers allow it: the forming passes for several workers are at their limit above width 32
    // and request it after the tile has been consumed instead)
    constexpr bool BPRE = !FORM || ONEW || NB == 1;
    uintx4 bq[NB][PL];
    auto b_prefetch = [&](int ch) {
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int v = t + i * kThreads;        // 0 .. 32*NB*8-1: 16-byte piece of the chunk
            const int64_t goff = ((int64_t)ch * (BK / 16) * NB * 64 + v) * 8;
#pragma unroll
            for (int k = 0; k < PL; ++k)
                bq[i][k] = *reinterpret_cast<const PSGD_GLOBAL uintx4*>(as_global(XK.t[k]) + goff);
        }
    };
    floatx4 d[LAZY ? 2 : 1][4];
    auto corr_to_lds = [&]() {
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int v = t + i * kThreads;
            const int c = v / (4 * NB), part = v % (4 * NB);
#pragma unroll
            for (int k = 0; k < PL; ++k)
                *reinterpret_cast<uintx4*>(c_pl + k * CPL + (COLMODE ? c : (c & 3) * 16 + (c >> 2)) * CPW + 8 * part) = cq[i][k];
        }
    };
    // the rank-r product for the chunk whose kept rows are in LDS, in the tile's register layout
    auto corr_mfma = [&]() {
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int q = 0; q < 4; ++q) d[h][q] = floatx4{0.f, 0.f, 0.f, 0.f};
        if constexpr (!COLMODE) {
            // A operand = the resident rows (block h), B operand = the staged chunk (block q)
#pragma unroll
            for (int ks = 0; ks < NB; ++ks)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    bf16x8 bv[PL];
#pragma unroll
                    for (int k = 0; k < PL; ++k)
                        bv[k] = *reinterpret_cast<const bf16x8*>(c_pl + k * CPL + (16 * q + lj) * CPW + 32 * ks + 8 * lq);
#pragma unroll
                    for (int h = 0; h < 2; ++h)
#pragma unroll
                        for (int sum = 2 * (PL - 1); sum >= 0; --sum)
#pragma unroll
                            for (int ka = 0; ka < PL; ++ka) {
                                const int kb = sum - ka;
                                if (kb >= 0 && kb < PL && keep_term<PL>(ka, kb))
                                    d[h][q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ap[h][ks][ka], bv[kb], d[h][q], 0, 0, 0);
                            }
                }
        } else {
            // A operand = the staged chunk rows (block h of this wave's 32), B operand = the resident columns (block q)
#pragma unroll
            for (int ks = 0; ks < NB; ++ks)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    bf16x8 av[PL];
#pragma unroll
                    for (int k = 0; k < PL; ++k)
                        av[k] = *reinterpret_cast<const bf16x8*>(c_pl + k * CPL + (32 * (wv & 1) + 16 * h + lj) * CPW + 32 * ks + 8 * lq);
#pragma unroll
                    for (int q = 0; q < 4; ++q)
#pragma unroll
                        for (int sum = 2 * (PL - 1); sum >= 0; --sum)
#pragma unroll
                            for (int ka = 0; ka < PL; ++ka) {
                                const int kb = sum - ka;
                                if (kb >= 0 && kb < PL && keep_term<PL>(ka, kb))
                                    d[h][q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[ka], ap[q][ks][kb], d[h][q], 0, 0, 0);
                            }
                }
        }
    };
    float4 p0[8], p1[8];
    if (n_loc > 0) {
        if (LAZY) {
            // the first chunk's product has no MFMA phase before it to hide in
            corr_prefetch(chunk_at(0));
            corr_to_lds();
            __syncthreads();
            corr_mfma();
            __syncthreads();
            if (n_loc > 1) corr_prefetch(chunk_at(1));
        }
        if (BPRE) b_prefetch(chunk_at(0));
        tile_prefetch<FORM>(L, addr_of(chunk_at(0)), p0, p1);
    }
    for (int it = 0; it < n_loc; ++it) {
        const int ch = chunk_at(it);
        // ---- thin operand chunk -> LDS [cp][LDSW] (its buffer is free: the last MFMA phase ended in a barrier)
        auto b_to_lds = [&]() {
#pragma unroll
            for (int i = 0; i < NB; ++i) {
                // piece v = (k16, nb, lane): column 32 nb + (lane & 31), rows 16 k16 + 8 (lane >> 5) .. + 7 of the chunk
                const int v = t + i * kThreads;
                const int k16 = v / (64 * NB), rem = v - k16 * (64 * NB);
                const int c = 32 * (rem >> 6) + (rem & 31), part = 2 * k16 + ((rem >> 5) & 1);
#pragma unroll
                for (int k = 0; k < PL; ++k)
                    *reinterpret_cast<uintx4*>(b_pl + k * BPL + c * LDSW + 8 * part) = bq[i][k];
            }
        };
        if (BPRE) b_to_lds();
        // ---- LAZY: E = M_{t-1} - (rank-r product of the previous step), rounded to fp32 here as the residual kernel
        // would have stored it; the product for this tile was formed during the previous MFMA phase.  The next
        // chunk's rows of the kept operand go to LDS now (their buffer was last read before the last barrier).
        if (LAZY) {
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    float4& e = p1[4 * h + v];
                    e.x -= d[h][0][v]; e.y -= d[h][1][v]; e.z -= d[h][2][v]; e.w -= d[h][3][v];
                }
            if (it + 1 < n_loc) corr_to_lds();
        }
        // ---- S tile: (prefetched) global -> registers -> (store M) -> split -> LDS
        {
            const TileAddr a = addr_of(ch);
            float4 m[8];
            tile_finish<FORM, (NB <= 2 && !LAZY), ONEW>(L, a, inv_n, p0, p1, m);
            if (store_m) store_m8(L, a, m);
            if (!COLMODE) {
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int row = LAZY ? r0 + (u & 3) + 16 * (u >> 2) : r0 + 16 * u;
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
                    for (int k = 0; k < PL; ++k) *reinterpret_cast<bf16x4*>(a_pl + k * APL + row * LDSW + 4 * c4) = o[k];
                }
            } else if constexpr (LAZY) {
                // piece u = 4h + v: rows 16h + v (+ this lane's 32 (wv & 1) + 4 lq), i.e. 4 consecutive k per column
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    bf16x4 o[4][PL];
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        bf16_t q[PL];
                        split_planes<PL>(m[4 * h + v].x, q);
#pragma unroll
                        for (int k = 0; k < PL; ++k) o[0][k][v] = q[k];
                        split_planes<PL>(m[4 * h + v].y, q);
#pragma unroll
                        for (int k = 0; k < PL; ++k) o[1][k][v] = q[k];
                        split_planes<PL>(m[4 * h + v].z, q);
#pragma unroll
                        for (int k = 0; k < PL; ++k) o[2][k][v] = q[k];
                        split_planes<PL>(m[4 * h + v].w, q);
#pragma unroll
                        for (int k = 0; k < PL; ++k) o[3][k][v] = q[k];
                    }
                    const int kk = r0 + 16 * h;                 // first of the 4 rows, a multiple of 4
#pragma unroll
                    for (int q = 0; q < 4; ++q)
#pragma unroll
                        for (int k = 0; k < PL; ++k)
                            *reinterpret_cast<bf16x4*>(a_pl + k * APL + (4 * c4 + q) * LDSW + 8 * a_chunk<true>(4 * c4 + q, kk >> 3) + (kk & 4)) = o[q][k];
                }
            } else {
                const int rg = r0;
                bf16x8 o[4][PL];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    bf16_t q[PL];
                    split_planes<PL>(m[u].x, q);
#pragma unroll
                    for (int k = 0; k < PL; ++k) o[0][k][u] = q[k];
                    split_planes<PL>(m[u].y, q);
#pragma unroll
                    for (int k = 0; k < PL; ++k) o[1][k][u] = q[k];
                    split_planes<PL>(m[u].z, q);
#pragma unroll
                    for (int k = 0; k < PL; ++k) o[2][k][u] = q[k];
                    split_planes<PL>(m[u].w, q);
#pragma unroll
                    for (int k = 0; k < PL; ++k) o[3][k][u] = q[k];
                }
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int k = 0; k < PL; ++k)
                        *reinterpret_cast<bf16x8*>(a_pl + k * APL + (4 * c4 + q) * LDSW + 8 * a_chunk<true>(4 * c4 + q, rg)) = o[q][k];
            }
                }
        if (!BPRE) { b_prefetch(ch); b_to_lds(); }
        __syncthreads();
        // ---- next tile's first loads go out now and stay in flight during the MFMA phase
        if (it + 1 < n_loc) {
            if (BPRE) b_prefetch(chunk_at(it + 1));
            if (LAZY && it + 2 < n_loc) corr_prefetch(chunk_at(it + 2));
            tile_prefetch<FORM>(L, addr_of(chunk_at(it + 1)), p0, p1);
        }
        // ---- MFMA: 32 output rows per wave, NB blocks of 32 columns, 4 k-steps of 16
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            const int aoff = (32 * wv + li) * LDSW + 8 * a_chunk<COLMODE>(32 * wv + li, 2 * ks + lg);
            bf16x8 av[PL];
#pragma unroll
            for (int k = 0; k < PL; ++k) av[k] = *reinterpret_cast<const bf16x8*>(a_pl + k * APL + aoff);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const int boff = (32 * nb + li) * LDSW + 16 * ks + 8 * lg;
                bf16x8 bv[PL];
#pragma unroll
                for (int k = 0; k < PL; ++k) bv[k] = *reinterpret_cast<const bf16x8*>(b_pl + k * BPL + boff);
                // smallest products first
#pragma unroll
                for (int sum = 2 * (PL - 1); sum >= 0; --sum)
#pragma unroll
                    for (int ka = 0; ka < PL; ++ka) {
                        const int kb = sum - ka;
                        if (kb >= 0 && kb < PL && keep_term<PL>(ka, kb))
                            acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[ka], bv[kb], acc[nb], 0, 0, 0);
                    }
            }
        }
        // ---- LAZY: the next chunk's rank-r product, in the same MFMA phase (its rows went to LDS before the barrier)
        if (LAZY && it + 1 < n_loc) corr_mfma();
        __syncthreads();
    }
    const int out_lenP = side_lenP(L, out_side);
    const ThinRef T = L.thin[out_role];
    if (n_split > 1) {
        // This workgroup holds one of n_split partial sums: store it and leave; finish_kernel adds
        // them up in split order.  Layout [split][column][row]: only the T.width real columns are
        // stored, and a lane's four consecutive accumulator rows go out as one 16-byte store.
        const int64_t plane = (int64_t)out_lenP * T.width;
        PSGD_GLOBAL float* __restrict__ dst = as_global(L.part[out_side]) + sp * plane + (int64_t)ob * BT + 32 * wv + 4 * lg;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const int col = 32 * nb + li;
            if (col < T.width) {
#pragma unroll
                for (int vq = 0; vq < 4; ++vq)
                    *reinterpret_cast<PSGD_GLOBAL floatx4*>(dst + (int64_t)col * out_lenP + 8 * vq) =
                        floatx4{acc[nb][4 * vq], acc[nb][4 * vq + 1], acc[nb][4 * vq + 2], acc[nb][4 * vq + 3]};
            }
        }
        return;
    }
    // ---- single split: the tile is complete; stage it in LDS (the operand buffers are dead: all
    // MFMA reads are behind a barrier) and run the epilogue here
    float* otile = reinterpret_cast<float*>(smem);    // [BT][cp + 1]
    const int tw = cp + 1;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = 32 * wv + 8 * (v >> 2) + 4 * lg + (v & 3);
            otile[row * tw + 32 * nb + li] = acc[nb][v];
        }
    __syncthreads();
    tile_epilogue(L, T, out_side, ob, out_len, out_lenP, cp, epi, otile, tw, (epi_flags & EPI_KEPT) != 0);
}

// Sum of the partial products of a split launch + the same epilogue.  One workgroup per 128-row
// output block; the partials are added in split order, so the result is deterministic.
// chol_gate >= -1: the last workgroup to finish a layer goes on to factorise the sum of the partial Gram
// matrices (first CholeskyQR pass) if that gate is open, unless the layer is one where the apply kernel
// does that for itself or one that is left to the chol_kernel launch that follows (see there); -2: no
// factorisation follows.
static_assert(BT == kGramRows1, "one partial Gram matrix per output block of a product");
__global__ __launch_bounds__(kThreads) void finish_kernel(const LayerDev* __restrict__ layers,
                                                          const int* __restrict__ ids, int colmode, int cp,
                                                          int out_role, int epi_flags, int gate, int chol_gate,
                                                          int a2gate, double tol2, int local_ok, int form) {
    __shared__ int s_last;
    const LayerDev& L = layers[ids[blockIdx.y]];
    if (!gate_open(L, gate)) return;
    const int epi = epi_flags & EPI_KIND_MASK;
    const int out_side = colmode ? SIDE_W : SIDE_L;
    const int out_len = colmode ? L.cols : L.rows;
    // form (whose partial sums): 0 = a product of prod_kernel that reads M, 1 = a forming pass of prod_kernel,
    // 2 = a row-mode pass on 32 x 256 tiles (form_row_kernel, row_prod_kernel), 3 = col_prod_kernel
    const int n_split = form == 2 ? L.split_row_v2 : form == 3 ? L.split_col_v2
                        : form ? (colmode ? L.split_col_f : L.split_row_f) : (colmode ? L.split_col : L.split_row);
    const int ob = blockIdx.x;
    if (n_split <= 1 || ob * BT >= out_len) return;
    const int out_lenP = side_lenP(L, out_side);
    const ThinRef T = L.thin[out_role];
    extern __shared__ __align__(16) unsigned char smem[];
    float* otile = reinterpret_cast<float*>(smem);    // [BT][cp + 1]
    const int tw = cp + 1;
    const int t = threadIdx.x;
    for (int e = t; e < BT * cp; e += kThreads) otile[(e / cp) * tw + e % cp] = 0.f;
    __syncthreads();
    const int64_t plane = (int64_t)out_lenP * T.width;
    const PSGD_GLOBAL float* __restrict__ src = as_global(L.part[out_side]) + (int64_t)ob * BT;
    // U items per thread at a time (two where a thread has several: 16 loads of 16 bytes in flight at a split of 8;
    // four spill), eight splits per batch.  Every sum runs in split order.
    auto reduce_items = [&](auto u_tag, int first, int last) {
        constexpr int U = decltype(u_tag)::value;
        for (int item0 = first + t; item0 < last; item0 += U * kThreads) {
            const PSGD_GLOBAL float* sc[U];
            float4 sum[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int item = item0 + u * kThreads < last ? item0 + u * kThreads : item0;     // (clamped: a valid address)
                sc[u] = src + (int64_t)(item / (BT / 4)) * out_lenP + 4 * (item % (BT / 4));
                sum[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            }
            int s2 = 0;
            for (; s2 + 8 <= n_split; s2 += 8) {
                float4 x[U][8];
#pragma unroll
                for (int u = 0; u < U; ++u)
#pragma unroll
                    for (int d = 0; d < 8; ++d) x[u][d] = ld_f32x4(sc[u] + (s2 + d) * plane);
#pragma unroll
                for (int u = 0; u < U; ++u)
#pragma unroll
                    for (int d = 0; d < 8; ++d) { sum[u].x += x[u][d].x; sum[u].y += x[u][d].y; sum[u].z += x[u][d].z; sum[u].w += x[u][d].w; }
            }
            for (; s2 < n_split; ++s2) {
                float4 x[U];
#pragma unroll
                for (int u = 0; u < U; ++u) x[u] = ld_f32x4(sc[u] + s2 * plane);
#pragma unroll
                for (int u = 0; u < U; ++u) { sum[u].x += x[u].x; sum[u].y += x[u].y; sum[u].z += x[u].z; sum[u].w += x[u].w; }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int item = item0 + u * kThreads;
                if (item >= last) continue;
                const int col = item / (BT / 4), r4 = 4 * (item % (BT / 4));
                otile[(r4 + 0) * tw + col] = sum[u].x;
                otile[(r4 + 1) * tw + col] = sum[u].y;
                otile[(r4 + 2) * tw + col] = sum[u].z;
                otile[(r4 + 3) * tw + col] = sum[u].w;
            }
        }
    };
    {
        const int n_items = T.width * (BT / 4);
        if (n_items >= 2 * kThreads) reduce_items(std::integral_constant<int, 2>{}, 0, n_items);
        else reduce_items(std::integral_constant<int, 1>{}, 0, n_items);
    }
    __syncthreads();
    tile_epilogue(L, T, out_side, ob, out_len, out_lenP, cp, epi, otile, tw, (epi_flags & EPI_KEPT) != 0);
    if (epi == EPI_GRAM && chol_gate >= -1 && !local_chol(L, out_role, local_ok) && gate_open(L, chol_gate)) {
        const int n_wg = (out_len + BT - 1) / BT;      // = number of Gram slots (BT == kGramRows1)
        if (grouped_slot_sum(T.width, n_wg)) {
            // wide block, many slots: add the slots up in groups here, side by side; a launch of chol_kernel with
            // twice the threads does the rest
            const int grp = ob / kSlotGroup;
            const int in_grp = min(kSlotGroup, n_wg - grp * kSlotGroup);
            if (last_to_arrive(&L.status[8 + grp], in_grp, &s_last)) sum_slot_group(L.gram, T.width, n_wg, grp);
        } else if (last_to_arrive(&L.status[6], n_wg, &s_last)) {
            chol_body(L, out_role, tol2, 1, kGramRows1, allow2_of(L, a2gate), smem, L.tmat);
        }
    }
}

// Partial Gram matrices of a thin matrix that did not come out of one of these products (the averaged P of a
// data-parallel step, handed back by the caller): one workgroup per 128 rows fills the slot a product's epilogue
// would have filled.
__global__ __launch_bounds__(kThreads) void thin_gram_kernel(const LayerDev* __restrict__ layers,
                                                             const int* __restrict__ ids, int role, int cp,
                                                             int gate) {
    const LayerDev& L = layers[ids[blockIdx.y]];
    if (!gate_open(L, gate)) return;
    const int len = side_len(L, side_of_role(L.transposed, role));
    const int ob = blockIdx.x;
    if (ob * BT >= len) return;
    const ThinRef T = L.thin[role];
    const int w = T.width;
    extern __shared__ __align__(16) unsigned char smem[];
    float* otile = reinterpret_cast<float*>(smem);    // [BT][cp + 1]
    const int tw = cp + 1;
    const int t = threadIdx.x;
    for (int e = t; e < BT * cp; e += kThreads) otile[(e / cp) * tw + e % cp] = 0.f;
    __syncthreads();
    for (int e = t; e < BT * w; e += kThreads) {
        const int row = e / w, col = e % w;
        if (ob * BT + row < len) otile[row * tw + col] = as_global(T.ptr)[(int64_t)(ob * BT + row) * T.ld + col];
    }
    __syncthreads();
    gram_tile_f64(otile, tw, BT, w, L.gram + (int64_t)ob * ((w * (w + 1)) / 2));
}

// gate: iteration gate of the refresh (-1: none)
hipError_t launch_thin_gram(const LayerDev* layers, const int* ids, int n_ids, int max_blocks, int role, int cp,
                            int gate, hipStream_t st) {
    if (n_ids <= 0 || max_blocks <= 0) return hipSuccess;
    dim3 grid(max_blocks, n_ids), block(kThreads);
    const size_t lds = (size_t)BT * (cp + 1) * sizeof(float);
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(thin_gram_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(thin_gram_kernel, grid, block, lds, st, layers, ids, role, cp, gate);
    return hipGetLastError();
}

hipError_t launch_finish(bool colmode, int form, const LayerDev* layers, const int* ids, int n_ids, int max_blocks,
                         int cp, int out_role, int epi, int gate, int chol_gate, int a2gate, double tol2, int w,
                         int local_ok, hipStream_t st) {
    if (n_ids <= 0 || max_blocks <= 0) return hipSuccess;
    dim3 grid(max_blocks, n_ids), block(kThreads);
    size_t lds = (size_t)BT * (cp + 1) * sizeof(float);
    if (chol_gate >= -1 && chol_lds_bytes_upto(w) > lds) lds = chol_lds_bytes_upto(w);
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(finish_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(finish_kernel, grid, block, lds, st, layers, ids, colmode ? 1 : 0, cp, out_role, epi, gate,
                       chol_gate, a2gate, tol2, local_ok, form);
    return hipGetLastError();
}

size_t prod_lds_bytes(int nb, int planes, bool lazy = false) {
    const size_t operands = (size_t)planes * (BT * LDSW + nb * 32 * LDSW + (lazy ? BK * (32 * nb + 8) : 0)) * sizeof(bf16_t);
    const size_t tile = (size_t)BT * (32 * nb + 1) * sizeof(float);
    return operands > tile ? operands : tile;
}

template <int NB, int PL>
static hipError_t launch_nb(bool colmode, bool form, bool lazy, bool onew, const LayerDev* layers, const int* ids,
                            int n_ids, int max_tiles, int out_role, int epi, int gate, hipStream_t st) {
    if (n_ids <= 0 || max_tiles <= 0) return hipSuccess;
    dim3 grid(max_tiles, n_ids), block(kThreads);
    const size_t lds = prod_lds_bytes(NB, PL, lazy);
    const int cp = 32 * NB;
#define PSGD_LAUNCH(...)                                                                               \
    do {                                                                                               \
        auto kfn = prod_kernel<NB, PL, __VA_ARGS__>;                                                   \
        if (lds > 48 * 1024) {                                                                         \
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kfn),                     \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);  \
            if (e != hipSuccess) return e;                                                             \
        }                                                                                              \
        hipLaunchKernelGGL(kfn, grid, block, lds, st, layers, ids, cp, out_role, epi, gate);           \
    } while (0)
    if (lazy) {
        // the forming pass that also applies the pending residual: compress-step widths only, column mode at width 32
        if (!form) return hipErrorInvalidValue;
        if constexpr (NB == 1) {
            if (colmode) { if (onew) PSGD_LAUNCH(true, true, true, true); else PSGD_LAUNCH(true, true, true); }
            else         { if (onew) PSGD_LAUNCH(false, true, true, true); else PSGD_LAUNCH(false, true, true); }
        } else if constexpr (NB <= 4) {
            if (colmode) return hipErrorInvalidValue;
            if (onew) PSGD_LAUNCH(false, true, true, true); else PSGD_LAUNCH(false, true, true);
        } else {
            return hipErrorInvalidValue;
        }
    } else if (form && onew) { if (colmode) PSGD_LAUNCH(true, true, false, true); else PSGD_LAUNCH(false, true, false, true); }
    else if (colmode) { if (form) PSGD_LAUNCH(true, true); else PSGD_LAUNCH(true, false); }
    else              { if (form) PSGD_LAUNCH(false, true); else PSGD_LAUNCH(false, false); }
#undef PSGD_LAUNCH
    return hipGetLastError();
}

// nb = width / 32 of the thin operand (1..6); planes = 2 or 3 bf16 planes per operand.
// lazy: the forming pass also applies the pending rank-r correction (row mode, form, nb <= 4).
// onew: every layer of the launch has one worker (forming passes only; ignored otherwise).
hipError_t launch_prod(int nb, int planes, bool colmode, bool form, bool lazy, bool onew, const LayerDev* layers,
                       const int* ids, int n_ids, int max_tiles, int out_role, int epi, int gate, hipStream_t st) {
#define PSGD_CASE(N)                                                                                          \
    case N:                                                                                                   \
        return planes == 2 ? launch_nb<N, 2>(colmode, form, lazy, onew, layers, ids, n_ids, max_tiles, out_role, epi, gate, st) \
                           : launch_nb<N, 3>(colmode, form, lazy, onew, layers, ids, n_ids, max_tiles, out_role, epi, gate, st);
    switch (nb) {
        PSGD_CASE(1) PSGD_CASE(2) PSGD_CASE(3) PSGD_CASE(4) PSGD_CASE(5) PSGD_CASE(6)
        default: return hipErrorInvalidValue;
    }
#undef PSGD_CASE
}

}  // namespace psgd
