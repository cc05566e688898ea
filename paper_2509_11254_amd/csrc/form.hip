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

template <int NB, int PL, int LAZY> constexpr int form_abuf() { return (PL == 2 && !LAZY) ? 2 : 1; }
template <int NB, int PL, int LAZY> constexpr size_t form_lds_bytes() {
    const size_t a = (size_t)form_abuf<NB, PL, LAZY>() * PL * FR * FLD * sizeof(bf16_t);
    const size_t d = LAZY ? (size_t)FR * FDW * sizeof(float) + (size_t)2 * NB * PL * 64 * 8 * sizeof(bf16_t) : 0;
    const size_t red = (size_t)4 * FR * (32 * NB + 1) * sizeof(float);
    return a + d > red ? a + d : red;
}

// The end of a row-mode product on 32-row blocks: the four waves' partial results (each over its quarter of every
// step's reduction range) are added through LDS, and the block's 32 x cp result goes out -- as one of n_split partial
// sums for finish_kernel, or as rows of the result, then with the block's partial Gram matrix if the launch asks for
// it (one slot per 32 rows).
template <int NB>
__device__ inline void row_epilogue(unsigned char* smem, const floatx16 (&acc)[NB], const LayerDev& L, int out_role,
                                    int epi_flags, int sp, int ob, int n_split) {
    constexpr int cp = 32 * NB;
    const int t = threadIdx.x;
    const int lane = t & 63, wv = __builtin_amdgcn_readfirstlane(t >> 6);
    const int li = lane & 31, lg = lane >> 5;
    const int row0 = ob * FR;
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
        // the rows of the result; the totals also replace the first wave's slice in LDS (every entry is read and
        // written by one thread), from where this row block's partial Gram matrix is formed if the launch asks for
        // it: one slot per 32 rows here (epi_flags carries EPI_GRAM only where the factorisation that follows sums
        // 32-row slots)
        const bool gram = (epi_flags & EPI_KIND_MASK) == EPI_GRAM;
        for (int i = t; i < FR * cp; i += kThreads) {
            const int row = i / cp, col = i - row * cp;
            const float v = total(row, col);
            if (gram) red[row * RW + col] = v;
            if (col < T.width && row0 + row < L.rows) as_global(T.ptr)[(int64_t)(row0 + row) * T.ld + col] = v;
        }
        if (gram) {
            __syncthreads();
            gram_tile_f64(red, RW, FR, T.width, L.gram + (int64_t)ob * ((T.width * (T.width + 1)) / 2));
        }
    }
}

// GBF: the gradients are bf16 (else fp32); ONEW: one worker (no loop over further gradient buffers);
// LAZY: the residual of the previous compress step is applied on the way in (1), and with 2 the kept Q is not read
// at all: the caller vouches that the transposed operand copies of Q_{t-1}, which the product reads anyway, hold the
// same numbers, and the correction's operand is made from those fragments in registers (see correction_shared).
template <int NB, int PL, bool GBF, bool ONEW, int LAZY>
__global__ __launch_bounds__(kThreads, 2) void form_row_kernel(const LayerDev* __restrict__ layers,
                                                                const int* __restrict__ ids, int out_role,
                                                                int epi_flags, int nt_m,
                                                                const int* __restrict__ xtab, int xstride) {
    using GV = typename std::conditional<GBF, uintx2, floatx4>::type;
    using GT = typename std::conditional<GBF, bf16_t, float>::type;
    constexpr int cp = 32 * NB;
    constexpr int ABUF = form_abuf<NB, PL, LAZY>();
    constexpr int APL = FR * FLD;
    // Which layer and tile.  Plain launches: blockIdx.y = layer, blockIdx.x = tile.  With an XCD table (many layers):
    // consecutive workgroup ids go to consecutive XCDs, and XCD x works through the layers dealt to it one after the
    // other -- xtab row x holds the prefix sums of their tile counts, row 8 + x their positions in `ids` -- so that
    // the workgroups that share an L2 at any time read the thin operands of one or two layers, which fit it.
    int layer_pos = blockIdx.y, tile = blockIdx.x;
    if (xtab) {
        const int x = blockIdx.x & 7, s = blockIdx.x >> 3;
        const int* pre = xtab + x * xstride;
        const int n_mine = pre[xstride - 1];               // layers of this XCD (last word of the row)
        if (n_mine == 0 || s >= pre[n_mine]) return;
        int j = 0;
        while (s >= pre[j + 1]) ++j;
        layer_pos = xtab[(8 + x) * xstride + j];
        tile = s - pre[j];
    }
    const LayerDev& L = layers[ids[layer_pos]];
    // (what the loop needs of the layer is read here, once: the loop stores M, and the compiler reads a value again
    // after every store that might have changed it -- a round trip to the scalar cache in front of the loads of the next tile)
    const int rows = L.rows, cols = L.cols;
    const bool store_m = !(epi_flags & EPI_KEEP_E);
    const int n_ob = L.rowsP / FR;                       // (row blocks past the end write the zeros of the padding)
    const int n_split = L.split_row_v2;
    if (tile >= n_ob * n_split) return;
    const int sp = tile % n_split, ob = tile / n_split;
    const int row0 = ob * FR;
    const int n_chunks = (cols + FK - 1) / FK;
    const int cps = (n_chunks + n_split - 1) / n_split;
    const int ch0 = sp * cps;
    const int n_loc = row0 < rows ? max(min(n_chunks, ch0 + cps) - ch0, 0) : 0;

    extern __shared__ __align__(16) unsigned char smem[];
    bf16_t* a_pl = reinterpret_cast<bf16_t*>(smem);                              // ABUF x PL planes of [FR][FLD]
    float* d_lds = reinterpret_cast<float*>(a_pl + ABUF * PL * APL);             // [FR][FDW] (LAZY)
    bf16_t* p_lds = reinterpret_cast<bf16_t*>(d_lds + FR * FDW);                 // [2 NB][PL][64][8] (LAZY)

    const int t = threadIdx.x;
    // (the wave index as a scalar: addresses are then a uniform base in scalar registers plus one 32-bit lane offset)
    const int lane = t & 63, wv = __builtin_amdgcn_readfirstlane(t >> 6);
    const int li = lane & 31, lg = lane >> 5;
    const float inv_n = ONEW ? 1.0f : 1.0f / (float)L.n_workers;
    const int nw = ONEW ? 1 : L.n_workers;
    const int64_t ld = L.ld;
    const int colsP = L.colsP;
    PSGD_GLOBAL float* S = as_global(L.S);
    // this thread's pieces of a tile: piece u at row row0 + 4 u + wv, columns ch * FK + 4 lane .. + 3
    const int64_t wave_off = (int64_t)(row0 + wv) * ld;       // (uniform)
    const int64_t ustep = 4 * ld;
    const unsigned lane_e = 16u * (unsigned)lane, lane_g = (unsigned)sizeof(GV) * (unsigned)lane, lane_f = 16u * (unsigned)lane;
    const auto gtab = as_global(L.G);
    const PSGD_GLOBAL GT* const g_first = reinterpret_cast<const PSGD_GLOBAL GT*>(as_global(gtab[0]));
    auto grad_ptr = [&](int w) { return w == 0 ? g_first : reinterpret_cast<const PSGD_GLOBAL GT*>(as_global(gtab[w])); };
    auto tile_full = [&](int ch) { return row0 + FR <= rows && ch * FK + FK <= cols; };
    auto piece_ok = [&](int ch, int u) { return row0 + 4 * u + wv < rows && ch * FK + 4 * lane < cols; };
    auto load_g = [&](int w, int ch, GV (&x)[8]) {
        const PSGD_GLOBAL GT* gp = grad_ptr(w) + wave_off + (int64_t)ch * FK;
        auto at = [&](int u) { return reinterpret_cast<const PSGD_GLOBAL GV*>(reinterpret_cast<const PSGD_GLOBAL char*>(gp + u * ustep) + lane_g); };
        if (tile_full(ch)) {
#pragma unroll
            for (int u = 0; u < 8; ++u) x[u] = ld_stream<NT_G>(at(u));
        } else {
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                x[u] = GV{};
                if (piece_ok(ch, u)) x[u] = ld_stream<NT_G>(at(u));
            }
        }
    };
    auto load_e = [&](int ch, floatx4 (&x)[8]) {
        const PSGD_GLOBAL float* ep = S + wave_off + (int64_t)ch * FK;
        auto at = [&](int u) { return reinterpret_cast<const PSGD_GLOBAL floatx4*>(reinterpret_cast<const PSGD_GLOBAL char*>(ep + u * ustep) + lane_e); };
        if (tile_full(ch)) {
#pragma unroll
            for (int u = 0; u < 8; ++u) x[u] = ld_stream<NT_E_IN>(at(u));
        } else {
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                x[u] = floatx4{0.f, 0.f, 0.f, 0.f};
                if (piece_ok(ch, u)) x[u] = ld_stream<NT_E_IN>(at(u));
            }
        }
    };
    // Each row block starts its walk at a step of its own and wraps around: blocks walking in step would all be on
    // the same few memory channels (4.9 against 5.6 TB/s for the bare access pattern).  Plain launches: consecutive
    // blocks go to different XCDs, XCD x starts an eighth of the walk after XCD x - 1, block j of an XCD two steps
    // after block 0, every layer adds a phase.  With the XCD table the blocks of an XCD are consecutive blocks of one
    // layer, which are spread over the whole walk.  (Keeping the blocks of an XCD within two steps of each other
    // instead helps the L2 hit rate of the thin operands and hurts the channel spread by more: 12.6 against 11.05 ms
    // on the 7B-shaped set without the table.)
    int rot = 0;
    if (n_loc > 0) rot = xtab ? (ob + layer_pos) % n_loc : ((ob & 7) * (n_loc >> 3) + 2 * (ob >> 3) + layer_pos) % n_loc;
    auto chunk_at = [&](int it) { const int c = it + rot; return ch0 + (c >= n_loc ? c - n_loc : c); };

    // thin operand: this wave's fragments for its 64 columns of the step, four k-steps of 16
    const PackRef XK = L.pack[SIDE_W];
    bf16x8 bfrag[4][NB][PL];
    auto load_b_ks = [&](int ch, int ks, bf16x8 (&bfrag)[4][NB][PL]) {
        {
            // (past the padded length the fragment of the last k-step is read instead: M is zero there, and the
            // operand copies hold finite numbers)
            const int kg = min(ch * (FK / 16) + 4 * wv + ks, colsP / 16 - 1);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int k = 0; k < PL; ++k)
                    bfrag[ks][nb][k] = *reinterpret_cast<const PSGD_GLOBAL bf16x8*>(
                        reinterpret_cast<const PSGD_GLOBAL char*>(as_global(XK.t[k]) + ((int64_t)kg * NB + nb) * 512) + lane_f);
        }
    };
    auto load_b = [&](int ch, bf16x8 (&bfrag)[4][NB][PL]) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) load_b_ks(ch, ks, bfrag);
    };
    // LAZY: the correction d_lds[row][col] = sum_k P~[row0 + row][k] Q[ch * FK + col][k] of a step; wave v forms it
    // for columns 64 v .. 64 v + 63.  The workgroup's 32 rows of the kept P~ copy (A operand, all k-steps) sit in
    // LDS in fragment order; the kept Q rows of the step's columns (B operand) are requested one step ahead, before
    // the next tile's own loads (the wait counter is in issue order: fragments requested after the tile could only be
    // used once the tile had arrived).
    constexpr bool SHARE = LAZY == 2;
    bf16x8 qv[LAZY == 1 ? 2 : 1][LAZY == 1 ? 2 * NB : 1][PL];
    const PSGD_GLOBAL bf16_t* kept_w[PL];
#pragma unroll
    for (int k = 0; k < PL; ++k) kept_w[k] = LAZY == 1 ? as_global(L.lzf[SIDE_W][k]) : nullptr;
    auto load_q = [&](int ch, int q) {
        {
            // 32-column block of the kept Q copy; past the padded length the last block, whose product lands on
            // columns that are outside the matrix and masked
            const int cblk = min(ch * (FK / 32) + 2 * wv + q, colsP / 32 - 1);
#pragma unroll
            for (int ks = 0; ks < 2 * NB; ++ks)
#pragma unroll
                for (int k = 0; k < PL; ++k)
                    qv[q][ks][k] = *reinterpret_cast<const PSGD_GLOBAL bf16x8*>(
                        reinterpret_cast<const PSGD_GLOBAL char*>(kept_w[k] + ((int64_t)cblk * (2 * NB) + ks) * 512) + lane_f);
        }
    };
    auto correction = [&](int q) {
        {
            floatx16 d;
#pragma unroll
            for (int v = 0; v < 16; ++v) d[v] = 0.f;
#pragma unroll
            for (int ks = 0; ks < 2 * NB; ++ks) {
                bf16x8 pv[PL];
#pragma unroll
                for (int k = 0; k < PL; ++k) pv[k] = *reinterpret_cast<const bf16x8*>(p_lds + ((ks * PL + k) * 64 + lane) * 8);
#pragma unroll
                for (int sum = 2 * (PL - 1); sum >= 0; --sum)
#pragma unroll
                    for (int ka = 0; ka < PL; ++ka) {
                        const int kb = sum - ka;
                        if (kb >= 0 && kb < PL && form_keep_term<PL>(ka, kb))
                            d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pv[ka], qv[q][ks][kb], d, 0, 0, 0);
                    }
            }
#pragma unroll
            for (int v = 0; v < 16; ++v)
                d_lds[(8 * (v >> 2) + 4 * lg + (v & 3)) * FDW + 64 * wv + 32 * q + li] = d[v];
        }
    };

    // LAZY == 2.  The product's fragments f[ks][nb][k] hold Q[16 ks + 8 lg + j][32 nb + li] (of the wave's 64 columns):
    // 8 columns of one rank index per lane, where the correction wants 8 rank indices of one column.  The matrix cores
    // turn one into the other: with the fragment as A operand (32 rank indices x 16 columns) and a 0/1 selection matrix
    // as B, two MFMAs leave the 32 x 32 block Q^T[rank][column] in accumulator layout -- lane li + 32 lg: column li,
    // rank indices 8 g + 4 lg + j -- exactly (x * 1 + 0 in fp32 of bf16 numbers).  Its registers 8 s .. 8 s + 7, cut
    // back to bf16, are a B operand for k-step s of that block with the rank indices in the order 8 (i >> 2) + 4 lg +
    // (i & 3), i = 0..7; the kept P~ sits in LDS in the same order (see the fill).  This saves the second stream of Q
    // fragments from L2 (as many bytes as the first, and 1.3 times the tile's from memory).
    bf16x8 sel0, sel1;
    if (SHARE) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            sel0[j] = (bf16_t)((8 * lg + j == li) ? 1.0f : 0.0f);
            sel1[j] = (bf16_t)((8 * lg + j + 16 == li) ? 1.0f : 0.0f);
        }
    }
    auto correction_shared = [&](const bf16x8 (&f)[4][NB][PL]) {
        if constexpr (SHARE) {
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            floatx16 d;
#pragma unroll
            for (int v = 0; v < 16; ++v) d[v] = 0.f;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int kb = PL - 1; kb >= 0; --kb) {          // (smaller plane first)
                    floatx16 tr;
#pragma unroll
                    for (int v = 0; v < 16; ++v) tr[v] = 0.f;
                    tr = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[2 * q][nb][kb], sel0, tr, 0, 0, 0);
                    tr = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[2 * q + 1][nb][kb], sel1, tr, 0, 0, 0);
#pragma unroll
                    for (int s2 = 0; s2 < 2; ++s2) {
                        uintx4 pk;
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            pk[i] = __builtin_amdgcn_perm(__float_as_uint(tr[8 * s2 + 2 * i + 1]),
                                                          __float_as_uint(tr[8 * s2 + 2 * i]), 0x07060302u);
                        bf16x8 qf;
                        __builtin_memcpy(&qf, &pk, 16);
                        const int ks = 2 * nb + s2;
#pragma unroll
                        for (int ka = PL - 1; ka >= 0; --ka)
                            if (form_keep_term<PL>(ka, kb)) {
                                const bf16x8 pv = *reinterpret_cast<const bf16x8*>(p_lds + ((ks * PL + ka) * 64 + lane) * 8);
                                d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pv, qf, d, 0, 0, 0);
                            }
                    }
                }
#pragma unroll
            for (int v = 0; v < 16; ++v)
                d_lds[(8 * (v >> 2) + 4 * lg + (v & 3)) * FDW + 64 * wv + 32 * q + li] = d[v];
            __builtin_amdgcn_sched_barrier(0);      // (one block at a time: interleaved they do not fit the registers)
        }
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
        load_b(chunk_at(0), bfrag);
        if (LAZY) {
            for (int i = t; i < 2 * NB * PL * 64; i += kThreads) {
                const int ks = i / (PL * 64), k = (i / 64) % PL, ln = i & 63;
                const uintx4 pc = *reinterpret_cast<const PSGD_GLOBAL uintx4*>(
                    as_global(L.lzf[SIDE_L][k]) + (((int64_t)ob * (2 * NB) + ks) * 64 + ln) * 8);
                if (SHARE) {
                    // rank indices 16 ks + 8 lg' + 4 h + 0..3 of row ln & 31 (lg' = ln >> 5) go to lane group h, places
                    // 4 lg' .. 4 lg' + 3: the order in which correction_shared gets the other operand
                    bf16_t* dst = p_lds + (i - ln) * 8 + (ln & 31) * 8 + 4 * (ln >> 5);
                    *reinterpret_cast<uintx2*>(dst) = uintx2{pc.x, pc.y};
                    *reinterpret_cast<uintx2*>(dst + 32 * 8) = uintx2{pc.z, pc.w};
                } else {
                    *reinterpret_cast<uintx4*>(p_lds + i * 8) = pc;
                }
            }
            if (LAZY == 1) {
                load_q(chunk_at(0), 0);
                load_q(chunk_at(0), 1);
            }
            __syncthreads();
            if (SHARE) {
                correction_shared(bfrag);
            } else {
                correction(0);
                correction(1);
            }
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
        // ---- the plain pass requests the next step's tile as soon as the registers of this one are free (10.8 -> 10.65 ms
        // on the 7B-shaped set); the others after the barrier below
        constexpr bool EARLY = LAZY == 0 && NB * PL <= 4;  // (where the registers allow it; with LAZY == 2 it gains nothing)
        if (EARLY && it + 1 < n_loc) {
            load_e(chunk_at(it + 1), e);
            load_g(0, chunk_at(it + 1), g);
        }
        const bool full = tile_full(ch);
        if (!full) {
            // pieces outside the matrix were loaded as zero; cut the column tail (the padding up to ld is not data)
            const int c = ch * FK + 4 * lane;
            const bool k0 = c < cols, k1 = c + 1 < cols, k2 = c + 2 < cols, k3 = c + 3 < cols;
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                m[u].x = k0 ? m[u].x : 0.f;           // (LAZY: the correction is not zero there)
                m[u].y = k1 ? m[u].y : 0.f;
                m[u].z = k2 ? m[u].z : 0.f;
                m[u].w = k3 ? m[u].w : 0.f;
            }
        }
        // ---- M back in place of E
        if (store_m) {
            PSGD_GLOBAL float* mp = S + wave_off + (int64_t)ch * FK;
            auto at = [&](int u) { return reinterpret_cast<PSGD_GLOBAL float*>(reinterpret_cast<PSGD_GLOBAL char*>(mp + u * ustep) + lane_e); };
            if (full) {
                if (nt_m) {
#pragma unroll
                    for (int u = 0; u < 8; ++u) __builtin_nontemporal_store(m[u], reinterpret_cast<PSGD_GLOBAL floatx4*>(at(u)));
                } else {
#pragma unroll
                    for (int u = 0; u < 8; ++u) *reinterpret_cast<PSGD_GLOBAL floatx4*>(at(u)) = m[u];
                }
            } else {
                const int c = ch * FK + 4 * lane;
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    if (!piece_ok(ch, u)) continue;
                    PSGD_GLOBAL float* p = at(u);
                    if (c + 3 < cols) {
                        *reinterpret_cast<PSGD_GLOBAL floatx4*>(p) = m[u];
                    } else {
                        p[0] = m[u].x;
                        if (c + 1 < cols) p[1] = m[u].y;
                        if (c + 2 < cols) p[2] = m[u].z;
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
        // ---- the next step's tile goes out now and is in flight during the MFMA phase.  (LAZY: half of the kept Q
        // fragments of the next step go out first, the other half and the tile after this step's product: the
        // registers do not hold the tile, both sets of fragments and the accumulators at once.)
        if (it + 1 < n_loc) {
            if (LAZY == 1) {
                load_q(chunk_at(it + 1), 0);
            } else if (!EARLY) {
                load_e(chunk_at(it + 1), e);
                load_g(0, chunk_at(it + 1), g);
            }
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
            // (LAZY == 2: the fragments of this k-step are used up; the next step's go into their registers now, so
            // that they are on their way during the rest of the product and there for the correction below)
            if (SHARE && it + 1 < n_loc) load_b_ks(chunk_at(it + 1), ks, bfrag);
        }
        // ---- the next step's thin operand fragments (their registers are free now); LAZY: its tile and its
        // correction first (d_lds was last read before this step's barrier)
        if (it + 1 < n_loc) {
            if (SHARE) {
                correction_shared(bfrag);
            } else {
                if (LAZY) {
                    load_q(chunk_at(it + 1), 1);      // (before the tile: the wait counter is in issue order)
                    load_e(chunk_at(it + 1), e);
                    load_g(0, chunk_at(it + 1), g);
                    correction(0);
                    correction(1);
                }
                load_b(chunk_at(it + 1), bfrag);
            }
        }
        if (ABUF == 1) __syncthreads();
    }
    row_epilogue<NB>(smem, acc, L, out_role, epi_flags, sp, ob, n_split);
}

// ---------------------------------------------------------------------------------------------------------------
// The same product without the forming:  thin[out_role] = S X  for a matrix that is already in S (Z = M Y of the
// refresh's iteration).  Reads S only; same geometry as form_row_kernel, two tiles in flight as in col_prod_kernel
// below (see there for the issue order).
// ---------------------------------------------------------------------------------------------------------------
template <int NB, int PL> constexpr int rowprod_abuf() { return PL == 2 ? 2 : 1; }
template <int NB, int PL> constexpr size_t rowprod_lds_bytes() {
    const size_t a = (size_t)rowprod_abuf<NB, PL>() * PL * FR * FLD * sizeof(bf16_t);
    const size_t red = (size_t)4 * FR * (32 * NB + 1) * sizeof(float);
    return a > red ? a : red;
}

template <int NB, int PL>
__global__ __launch_bounds__(kThreads, 2) void row_prod_kernel(const LayerDev* __restrict__ layers,
                                                                const int* __restrict__ ids, int out_role,
                                                                int epi_flags, int gate, int nt_s,
                                                                const int* __restrict__ xtab, int xstride) {
    constexpr int ABUF = rowprod_abuf<NB, PL>();
    constexpr int APL = FR * FLD;
    int layer_pos = blockIdx.y, tile = blockIdx.x;
    if (xtab) {
        const int x = blockIdx.x & 7, s = blockIdx.x >> 3;
        const int* pre = xtab + x * xstride;
        const int n_mine = pre[xstride - 1];
        if (n_mine == 0 || s >= pre[n_mine]) return;
        int j = 0;
        while (s >= pre[j + 1]) ++j;
        layer_pos = xtab[(8 + x) * xstride + j];
        tile = s - pre[j];
    }
    const LayerDev& L = layers[ids[layer_pos]];
    if (!gate_open(L, gate)) return;
    const int n_ob = L.rowsP / FR;
    const int n_split = L.split_row_v2;
    if (tile >= n_ob * n_split) return;
    const int sp = tile % n_split, ob = tile / n_split;
    const int row0 = ob * FR;
    const int n_chunks = (L.cols + FK - 1) / FK;
    const int cps = (n_chunks + n_split - 1) / n_split;
    const int ch0 = sp * cps;
    const int n_loc = row0 < L.rows ? max(min(n_chunks, ch0 + cps) - ch0, 0) : 0;

    extern __shared__ __align__(16) unsigned char smem[];
    bf16_t* a_pl = reinterpret_cast<bf16_t*>(smem);                              // ABUF x PL planes of [FR][FLD]
    const int t = threadIdx.x;
    const int lane = t & 63, wv = __builtin_amdgcn_readfirstlane(t >> 6);
    const int li = lane & 31, lg = lane >> 5;
    const int64_t ld = L.ld;
    const int colsP = L.colsP;
    const PSGD_GLOBAL float* S = as_global(L.S);
    const int64_t wave_off = (int64_t)(row0 + wv) * ld;
    const int64_t ustep = 4 * ld;
    const unsigned lane_e = 16u * (unsigned)lane, lane_f = 16u * (unsigned)lane;
    // this thread's pieces of a tile: piece u at row row0 + 4 u + wv, columns ch * FK + 4 lane .. + 3
    auto tile_full = [&](int ch) { return row0 + FR <= L.rows && ch * FK + FK <= L.cols; };
    auto load_tile = [&](int ch, floatx4 (&x)[8]) {
        const PSGD_GLOBAL float* ep = S + wave_off + (int64_t)ch * FK;
        auto at = [&](int u) { return reinterpret_cast<const PSGD_GLOBAL floatx4*>(reinterpret_cast<const PSGD_GLOBAL char*>(ep + u * ustep) + lane_e); };
        if (tile_full(ch)) {
            if (nt_s) {
#pragma unroll
                for (int u = 0; u < 8; ++u) x[u] = __builtin_nontemporal_load(at(u));
            } else {
#pragma unroll
                for (int u = 0; u < 8; ++u) x[u] = *at(u);
            }
        } else {
            const int c = ch * FK + 4 * lane;
            const bool k0 = c < L.cols, k1 = c + 1 < L.cols, k2 = c + 2 < L.cols, k3 = c + 3 < L.cols;
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                x[u] = floatx4{0.f, 0.f, 0.f, 0.f};
                if (k0 && row0 + 4 * u + wv < L.rows) {
                    const floatx4 v = *at(u);                       // (the padding up to ld may be read, not used)
                    x[u] = floatx4{v.x, k1 ? v.y : 0.f, k2 ? v.z : 0.f, k3 ? v.w : 0.f};
                }
            }
        }
    };
    int rot = 0;
    if (n_loc > 0) rot = xtab ? (ob + layer_pos) % n_loc : ((ob & 7) * (n_loc >> 3) + 2 * (ob >> 3) + layer_pos) % n_loc;
    auto chunk_at = [&](int it) { const int c = it + rot; return ch0 + (c >= n_loc ? c - n_loc : c); };
    const PackRef XK = L.pack[SIDE_W];
    bf16x8 bfrag[4][NB][PL];
    auto load_b = [&](int ch) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const int kg = min(ch * (FK / 16) + 4 * wv + ks, colsP / 16 - 1);     // (past the end M is zero)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int k = 0; k < PL; ++k)
                    bfrag[ks][nb][k] = *reinterpret_cast<const PSGD_GLOBAL bf16x8*>(
                        reinterpret_cast<const PSGD_GLOBAL char*>(as_global(XK.t[k]) + ((int64_t)kg * NB + nb) * 512) + lane_f);
        }
    };
    floatx16 acc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[nb][v] = 0.f;
    // (two tiles in flight where the registers hold them beside the fragments, else one)
    constexpr int AHEAD = (PL == 2 || NB == 1) ? 2 : 1;
    floatx4 xa[8], xb[AHEAD == 2 ? 8 : 1];
    if (n_loc > 0) {
        load_tile(chunk_at(0), xa);
        load_b(chunk_at(0));
        if constexpr (AHEAD == 2) { if (n_loc > 1) load_tile(chunk_at(1), xb); }
    }
    auto step = [&](int it, floatx4 (&x)[8]) {
        bf16_t* a_cur = a_pl + (ABUF == 2 ? (it & 1) * PL * APL : 0);
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            bf16x4 o[PL];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                bf16_t pq[PL];
                split_planes<PL>(x[u][q], pq);
#pragma unroll
                for (int k = 0; k < PL; ++k) o[k][q] = pq[k];
            }
#pragma unroll
            for (int k = 0; k < PL; ++k) *reinterpret_cast<bf16x4*>(a_cur + k * APL + (4 * u + wv) * FLD + 4 * lane) = o[k];
        }
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            bf16x8 av[PL];
#pragma unroll
            for (int k = 0; k < PL; ++k)
                av[k] = *reinterpret_cast<const bf16x8*>(a_cur + k * APL + li * FLD + 64 * wv + 16 * ks + 8 * lg);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int sum = 2 * (PL - 1); sum >= 0; --sum)
#pragma unroll
                    for (int ka = 0; ka < PL; ++ka) {
                        const int kb = sum - ka;
                        if (kb >= 0 && kb < PL && form_keep_term<PL>(ka, kb))
                            acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[ka], bfrag[ks][nb][kb], acc[nb], 0, 0, 0);
                    }
        }
        if (it + 1 < n_loc) load_b(chunk_at(it + 1));
        if (it + AHEAD < n_loc) load_tile(chunk_at(it + AHEAD), x);
        if (ABUF == 1) __syncthreads();
    };
    if constexpr (AHEAD == 2) {
        for (int it = 0; it < n_loc; it += 2) {
            step(it, xa);
            if (it + 1 < n_loc) step(it + 1, xb);
        }
    } else {
        for (int it = 0; it < n_loc; ++it) step(it, xa);
    }
    row_epilogue<NB>(smem, acc, L, out_role, epi_flags, sp, ob, n_split);
}

// ---------------------------------------------------------------------------------------------------------------
// The second product on the same tiles:  Q = M^T P~  (Algorithm 1; also Y = M^T Z of the refresh's iteration) for
// layers stored with rows >= cols, at widths up to 64.  Reads S only (4 bytes per element).
//
// A workgroup owns 256 columns of S -- 256 rows of the result -- and walks down the rows 32 at a time; a load
// instruction of a wavefront covers 1 KB of one row.  A thread holds 8 consecutive rows of 4 columns, so the tile goes to
// LDS transposed with 16-byte writes ([column][32 rows], the 16-byte chunk index XOR-ed with bits of the column so
// that neither the writes nor the MFMA reads collide on banks).  Wave v owns result rows 64 v .. 64 v + 63; all four
// waves use the same fragments of the thin operand, which come straight from memory in MFMA order (PackRef::t).
// ---------------------------------------------------------------------------------------------------------------
constexpr int CW = 256;         // columns of S per workgroup
constexpr int CKR = 32;         // rows of S per step
constexpr int CLD = CKR + 8;    // LDS row stride of the transposed tile (bf16 elements, 80 bytes)

template <int NB, int PL> constexpr size_t colprod_lds_bytes() {
    const size_t a = (size_t)PL * CW * CLD * sizeof(bf16_t);
    const size_t o = (size_t)128 * (32 * NB + 1) * sizeof(float);
    return a > o ? a : o;
}

template <int NB, int PL>
__global__ __launch_bounds__(kThreads, ((PL == 2 && NB == 1) ? 3 : 2)) void col_prod_kernel(const LayerDev* __restrict__ layers,
                                                                const int* __restrict__ ids, int out_role,
                                                                int epi_flags, int gate, int nt_s,
                                                                const int* __restrict__ xtab, int xstride) {
    constexpr int cp = 32 * NB;
    constexpr int APL = CW * CLD;
    // (layer and tile: plain, or through an XCD table as in form_row_kernel -- all workgroups of a layer on one XCD
    // fetch its thin operand into one L2 instead of eight)
    int layer_pos = blockIdx.y, tile = blockIdx.x;
    if (xtab) {
        const int x = blockIdx.x & 7, s = blockIdx.x >> 3;
        const int* pre = xtab + x * xstride;
        const int n_mine = pre[xstride - 1];
        if (n_mine == 0 || s >= pre[n_mine]) return;
        int j = 0;
        while (s >= pre[j + 1]) ++j;
        layer_pos = xtab[(8 + x) * xstride + j];
        tile = s - pre[j];
    }
    const LayerDev& L = layers[ids[layer_pos]];
    if (!gate_open(L, gate)) return;
    const int epi = epi_flags & EPI_KIND_MASK;
    const int n_cb = (L.colsP + CW - 1) / CW;
    const int n_split = L.split_col_v2;
    if (tile >= n_cb * n_split) return;
    const int ob = tile % n_cb, sp = tile / n_cb;
    const int col0 = ob * CW;
    const int n_chunks = (L.rows + CKR - 1) / CKR;
    const int cps = (n_chunks + n_split - 1) / n_split;
    const int ch0 = sp * cps;
    const int n_loc = col0 < L.cols ? max(min(n_chunks, ch0 + cps) - ch0, 0) : 0;

    extern __shared__ __align__(16) unsigned char smem[];
    bf16_t* a_pl = reinterpret_cast<bf16_t*>(smem);          // PL planes of [CW][CLD]
    const int t = threadIdx.x;
    const int lane = t & 63, wv = __builtin_amdgcn_readfirstlane(t >> 6);
    const int li = lane & 31, lg = lane >> 5;
    const int64_t ld = L.ld;
    const int rowsP = L.rowsP;
    const PSGD_GLOBAL float* S = as_global(L.S);
    // this thread's pieces of a tile: piece u at row ch * 32 + 8 wv + u, columns col0 + 4 lane .. + 3.
    // Every step issues the same loads whatever the tile: where a piece lies outside the matrix the address is moved to a
    // place inside it (last row; the lane's first column) and the value is dropped afterwards.  The hardware's wait counter
    // counts loads in issue order, and the compiler can only leave the younger tile in flight while the older one
    // is consumed if the number of loads between them is the same on every path: with loads under conditions it
    // waited for all of them (vmcnt(0) before the LDS writes; vmcnt(16) now).  It also costs 54 registers less.  The
    // pass did not get faster by it (4.85 ms on the 7B-shaped set either way): with everything but the loads compiled
    // out it still takes 4.65 ms, where the same walk as a bare kernel takes 3.75 on the same buffers.
    const int c_lane = col0 + 4 * lane;
    const bool k0 = c_lane < L.cols, k1 = c_lane + 1 < L.cols, k2 = c_lane + 2 < L.cols, k3 = c_lane + 3 < L.cols;
    const unsigned lane_e = k0 ? 16u * (unsigned)lane : 0u;
    const int last_row = L.rows - 1;
    auto tile_full = [&](int ch) { return ch * CKR + CKR <= L.rows && col0 + CW <= L.cols; };
    auto load_tile = [&](int ch, floatx4 (&x)[8]) {
        const int r0 = min(ch * CKR + 8 * wv, last_row), lim = last_row - r0;           // (uniform)
        const PSGD_GLOBAL float* sp0 = S + (int64_t)r0 * ld + col0;
        auto at = [&](int u) { return reinterpret_cast<const PSGD_GLOBAL floatx4*>(reinterpret_cast<const PSGD_GLOBAL char*>(sp0 + (int64_t)min(u, lim) * ld) + lane_e); };
        if (nt_s) {
#pragma unroll
            for (int u = 0; u < 8; ++u) x[u] = __builtin_nontemporal_load(at(u));
        } else {
#pragma unroll
            for (int u = 0; u < 8; ++u) x[u] = *at(u);
        }
    };
    // (what load_tile fetched for places outside the matrix, or for a step past the end of the walk, becomes zero)
    auto mask_tile = [&](int ch, bool live, floatx4 (&x)[8]) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const bool row_ok = live && ch * CKR + 8 * wv + u < L.rows;
            x[u] = floatx4{row_ok && k0 ? x[u].x : 0.f, row_ok && k1 ? x[u].y : 0.f, row_ok && k2 ? x[u].z : 0.f,
                           row_ok && k3 ? x[u].w : 0.f};
        }
    };
    const PackRef XK = L.pack[SIDE_L];
    const unsigned lane_f = 16u * (unsigned)lane;
    auto load_b = [&](int ch, bf16x8 (&bf)[2][NB][PL]) {
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const int kg = min(ch * (CKR / 16) + ks, rowsP / 16 - 1);     // (past the end M is zero)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int k = 0; k < PL; ++k)
                    bf[ks][nb][k] = *reinterpret_cast<const PSGD_GLOBAL bf16x8*>(
                        reinterpret_cast<const PSGD_GLOBAL char*>(as_global(XK.t[k]) + ((int64_t)kg * NB + nb) * 512) + lane_f);
        }
    };
    floatx16 acc[2][NB];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[rb][nb][v] = 0.f;
    // Two tiles in flight: step `it` consumes one tile buffer while the tile of step it + 1 (requested a step ago) is
    // on its way in the other, and requests the tile of step it + 2 into the buffer it has just emptied -- after its
    // MFMA phase and after the fragments of step it + 1 (the wait counter is in issue order: what the next MFMA phase
    // waits for must be older than the tile that is to stay in flight through it).
    floatx4 xa[8], xb[8];
    bf16x8 bfrag[2][NB][PL];
    auto chunk_at = [&](int it) { return ch0 + min(it, n_loc - 1); };      // (steps past the end: the last tile again, dropped)
    if (n_loc > 0) {
        load_tile(chunk_at(0), xa);
        load_b(chunk_at(0), bfrag);
        load_tile(chunk_at(1), xb);
    }
    const int wsw = (lane >> 2) & 3;                  // write side: bits 4, 5 of this thread's columns 4 lane + q
    auto step = [&](int it, floatx4 (&x)[8]) {
        if (it >= n_loc || !tile_full(ch0 + it)) mask_tile(ch0 + it, it < n_loc, x);
        // ---- tile -> planes -> LDS, transposed: column 4 lane + q gets this thread's 8 rows as one 16-byte write
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            bf16x8 o[PL];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                bf16_t pq[PL];
                split_planes<PL>(x[u][q], pq);
#pragma unroll
                for (int k = 0; k < PL; ++k) o[k][u] = pq[k];
            }
#pragma unroll
            for (int k = 0; k < PL; ++k)
                *reinterpret_cast<bf16x8*>(a_pl + k * APL + (4 * lane + q) * CLD + 8 * (wv ^ wsw)) = o[k];
        }
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int rb = 0; rb < 2; ++rb) {
                const int cl = 64 * wv + 32 * rb + li;
                bf16x8 av[PL];
#pragma unroll
                for (int k = 0; k < PL; ++k)
                    av[k] = *reinterpret_cast<const bf16x8*>(a_pl + k * APL + cl * CLD + 8 * ((2 * ks + lg) ^ ((cl >> 4) & 3)));
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int sum = 2 * (PL - 1); sum >= 0; --sum)
#pragma unroll
                        for (int ka = 0; ka < PL; ++ka) {
                            const int kb = sum - ka;
                            if (kb >= 0 && kb < PL && form_keep_term<PL>(ka, kb))
                                acc[rb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[ka], bfrag[ks][nb][kb], acc[rb][nb], 0, 0, 0);
                        }
            }
        load_b(chunk_at(it + 1), bfrag);
        load_tile(chunk_at(it + 2), x);
        __syncthreads();
    };
    for (int it = 0; it < n_loc; it += 2) {          // (an odd walk ends with a step whose tile is dropped)
        step(it, xa);
        step(it + 1, xb);
    }
    // ---- the 256 x cp result tile goes out in two halves of 128 rows through LDS (the operand buffer is free: the
    // loop ends in a barrier); half h holds the rows of waves 2 h and 2 h + 1
    float* otile = reinterpret_cast<float*>(smem);            // [128][cp + 1]
    constexpr int tw = cp + 1;
    const ThinRef T = L.thin[out_role];
    const int w = T.width;
#pragma unroll 1
    for (int h = 0; h < 2; ++h) {
        if (h) __syncthreads();
        if ((wv >> 1) == h) {
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        otile[(64 * (wv & 1) + 32 * rb + 8 * (v >> 2) + 4 * lg + (v & 3)) * tw + 32 * nb + li] = acc[rb][nb][v];
        }
        __syncthreads();
        const int r0 = col0 + 128 * h;                        // first result row of this half
        if (r0 >= L.colsP) break;                             // (uniform)
        if (n_split > 1) {
            // one of n_split partial sums, [split][column][row]; finish_kernel adds them in split order
            PSGD_GLOBAL float* dst = as_global(L.part[SIDE_W]) + (int64_t)sp * L.colsP * w + r0;
            for (int i = t; i < 128 * w; i += kThreads) {
                const int row = i & 127, c = i >> 7;
                dst[(int64_t)c * L.colsP + row] = otile[row * tw + c];
            }
            continue;
        }
        if (T.ld == w && (w & 3) == 0) {
            // (rows of the result are one run of memory: 16-byte stores over the flat range)
            const int n_valid = (min(L.cols, r0 + 128) - r0) * w;
            const float inv_w = 1.0f / (float)w;
            PSGD_GLOBAL float* yp = as_global(T.ptr) + (int64_t)r0 * w;
            for (int f = 4 * t; f < n_valid; f += 4 * kThreads) {
                int row = (int)(((float)f + 0.5f) * inv_w);
                int c = f - row * w;
                if (c < 0) { --row; c += w; } else if (c >= w) { ++row; c -= w; }
                const float* __restrict__ sr = otile + row * tw + c;
                *reinterpret_cast<PSGD_GLOBAL floatx4*>(yp + f) = floatx4{sr[0], sr[1], sr[2], sr[3]};
            }
        } else {
            for (int i = t; i < 128 * w; i += kThreads) {
                const int row = i / w, c = i - row * w;
                if (r0 + row < L.cols) as_global(T.ptr)[(int64_t)(r0 + row) * T.ld + c] = otile[row * tw + c];
            }
        }
        // the partial Gram matrix or the operand copies of the result, per 128 rows as the other kernels expect them
        if (epi == EPI_GRAM) gram_tile_f64(otile, tw, 128, w, L.gram + (int64_t)(r0 / 128) * ((w * (w + 1)) / 2));
        else if (epi == EPI_PACK) write_packs<PL>(L.pack[SIDE_W], L.planes, otile, tw, cp, r0, 128, L.colsP, 3, (epi_flags & EPI_KEPT) ? L.lzf[SIDE_W] : nullptr);
    }
}

template <int NB, int PL>
static hipError_t launch_colprod_nb(const LayerDev* layers, const int* ids, int n_ids, int max_tiles, int out_role,
                                    int epi, int gate, int nt_s, const int* xtab, int xstride, int xtiles,
                                    hipStream_t st) {
    dim3 grid(max_tiles, n_ids), block(kThreads);
    if (xtab) grid = dim3(8 * xtiles, 1);
    auto kfn = col_prod_kernel<NB, PL>;
    const size_t lds = colprod_lds_bytes<NB, PL>();
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kfn), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kfn, grid, block, lds, st, layers, ids, out_role, epi, gate, nt_s, xtab, xstride);
    return hipGetLastError();
}

// (width 96 with three planes: the fragments of a step and two tiles do not fit the registers)
bool col_prod_supported(int nb, int planes) { return nb == 1 || nb == 2 || (nb == 3 && planes == 2); }

// max_tiles: max over the layers of ceil(padded cols / 256) * split_col_v2; nt_s: read S with the non-temporal hint
hipError_t launch_col_prod(int nb, int planes, const LayerDev* layers, const int* ids, int n_ids, int max_tiles,
                           int out_role, int epi, int gate, int nt_s, const int* xtab, int xstride, int xtiles,
                           hipStream_t st) {
    if (n_ids <= 0 || max_tiles <= 0) return hipSuccess;
    if (nb == 1) return planes == 2 ? launch_colprod_nb<1, 2>(layers, ids, n_ids, max_tiles, out_role, epi, gate, nt_s, xtab, xstride, xtiles, st)
                                    : launch_colprod_nb<1, 3>(layers, ids, n_ids, max_tiles, out_role, epi, gate, nt_s, xtab, xstride, xtiles, st);
    if (nb == 2) return planes == 2 ? launch_colprod_nb<2, 2>(layers, ids, n_ids, max_tiles, out_role, epi, gate, nt_s, xtab, xstride, xtiles, st)
                                    : launch_colprod_nb<2, 3>(layers, ids, n_ids, max_tiles, out_role, epi, gate, nt_s, xtab, xstride, xtiles, st);
    if (nb == 3 && planes == 2) return launch_colprod_nb<3, 2>(layers, ids, n_ids, max_tiles, out_role, epi, gate, nt_s, xtab, xstride, xtiles, st);
    return hipErrorInvalidValue;
}

template <int NB, int PL>
static hipError_t launch_rowprod_nb(const LayerDev* layers, const int* ids, int n_ids, int max_tiles, int out_role,
                                    int epi, int gate, int nt_s, const int* xtab, int xstride, int xtiles,
                                    hipStream_t st) {
    dim3 grid(max_tiles, n_ids), block(kThreads);
    if (xtab) grid = dim3(8 * xtiles, 1);
    auto kfn = row_prod_kernel<NB, PL>;
    const size_t lds = rowprod_lds_bytes<NB, PL>();
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kfn), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kfn, grid, block, lds, st, layers, ids, out_role, epi, gate, nt_s, xtab, xstride);
    return hipGetLastError();
}

// (not at width 96: every 32 rows fetch the thin operand again, 12 bytes from L2 per 4 bytes of S with two planes,
// and the pass is L2-bound there: 7.1 ms on the 7B-shaped set against 6.4 for prod_kernel's 128-row tiles)
bool row_prod_supported(int nb, int planes) { (void)planes; return nb == 1 || nb == 2; }

// thin[out_role] = S X on row-major layers, S read only.  max_tiles, xtab, xstride, xtiles as for launch_form_row;
// gate: iteration gate of the refresh (-1: none)
hipError_t launch_row_prod(int nb, int planes, const LayerDev* layers, const int* ids, int n_ids, int max_tiles,
                           int out_role, int epi, int gate, int nt_s, const int* xtab, int xstride, int xtiles,
                           hipStream_t st) {
    if (n_ids <= 0 || max_tiles <= 0) return hipSuccess;
    if (nb == 1) return planes == 2 ? launch_rowprod_nb<1, 2>(layers, ids, n_ids, max_tiles, out_role, epi, gate, nt_s, xtab, xstride, xtiles, st)
                                    : launch_rowprod_nb<1, 3>(layers, ids, n_ids, max_tiles, out_role, epi, gate, nt_s, xtab, xstride, xtiles, st);
    if (nb == 2) return planes == 2 ? launch_rowprod_nb<2, 2>(layers, ids, n_ids, max_tiles, out_role, epi, gate, nt_s, xtab, xstride, xtiles, st)
                                    : launch_rowprod_nb<2, 3>(layers, ids, n_ids, max_tiles, out_role, epi, gate, nt_s, xtab, xstride, xtiles, st);
    return hipErrorInvalidValue;
}

template <int NB, int PL>
static hipError_t launch_form_nb(bool gbf, bool onew, int lazy, const LayerDev* layers, const int* ids, int n_ids,
                                 int max_tiles, int out_role, int epi, int nt_m, const int* xtab, int xstride,
                                 int xtiles, hipStream_t st) {
    dim3 grid(max_tiles, n_ids), block(kThreads);
    if (xtab) grid = dim3(8 * xtiles, 1);
#define PSGD_FORM(GBF, ONEW, LAZY)                                                                             \
    do {                                                                                                       \
        auto kfn = form_row_kernel<NB, PL, GBF, ONEW, LAZY>;                                                   \
        const size_t lds = form_lds_bytes<NB, PL, LAZY>();                                                     \
        if (lds > 48 * 1024) {                                                                                 \
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kfn),                             \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);          \
            if (e != hipSuccess) return e;                                                                     \
        }                                                                                                      \
        hipLaunchKernelGGL(kfn, grid, block, lds, st, layers, ids, out_role, epi, nt_m, xtab, xstride);        \
    } while (0)
    if (lazy == 2) {
        if (gbf) { if (onew) PSGD_FORM(true, true, 2); else PSGD_FORM(true, false, 2); }
        else     { if (onew) PSGD_FORM(false, true, 2); else PSGD_FORM(false, false, 2); }
    } else if (lazy) {
        if (gbf) { if (onew) PSGD_FORM(true, true, 1); else PSGD_FORM(true, false, 1); }
        else     { if (onew) PSGD_FORM(false, true, 1); else PSGD_FORM(false, false, 1); }
    } else {
        if (gbf) { if (onew) PSGD_FORM(true, true, 0); else PSGD_FORM(true, false, 0); }
        else     { if (onew) PSGD_FORM(false, true, 0); else PSGD_FORM(false, false, 0); }
    }
#undef PSGD_FORM
    return hipGetLastError();
}

// Variants this kernel is built for: the thin operand fragments of a whole step live in registers next to the tile,
// which the wider and the several-fp32-worker variants cannot afford without spilling.
bool form_row_supported(int nb, int planes, bool gbf, bool onew, bool lazy) {
    if (nb < 1 || nb > 3) return false;
    const bool f32_multi = !gbf && !onew;
    if (nb == 1) return true;
    if (nb == 3) return planes == 2 && gbf && onew && !lazy;
    if (planes == 2) return !(lazy && f32_multi);
    return !lazy && !f32_multi;
}

// nb = width / 32 of the thin operand (1 or 2); gbf: every layer of the launch has bf16 gradients (else every layer
// fp32); onew: one worker; lazy: apply the owed residual on the way in (2: the kept Q is what the transposed operand
// copies of the product hold, and is taken from those); nt_m: store M with the non-temporal hint
// (matrices too large to be found in a cache by the second pass).  max_tiles: max over the layers of
// (padded rows / 32) * split_row_v2.  xtab (device, nullable): the XCD table described in the kernel, 16 rows of
// xstride ints; xtiles: the largest tile total of an XCD.
hipError_t launch_form_row(int nb, int planes, bool gbf, bool onew, int lazy, const LayerDev* layers, const int* ids,
                           int n_ids, int max_tiles, int out_role, int epi, int nt_m, const int* xtab, int xstride,
                           int xtiles, hipStream_t st) {
    if (n_ids <= 0 || max_tiles <= 0) return hipSuccess;
    if (nb == 1) return planes == 2 ? launch_form_nb<1, 2>(gbf, onew, lazy, layers, ids, n_ids, max_tiles, out_role, epi, nt_m, xtab, xstride, xtiles, st)
                                    : launch_form_nb<1, 3>(gbf, onew, lazy, layers, ids, n_ids, max_tiles, out_role, epi, nt_m, xtab, xstride, xtiles, st);
    if (nb == 2) return planes == 2 ? launch_form_nb<2, 2>(gbf, onew, lazy, layers, ids, n_ids, max_tiles, out_role, epi, nt_m, xtab, xstride, xtiles, st)
                                    : launch_form_nb<2, 3>(gbf, onew, lazy, layers, ids, n_ids, max_tiles, out_role, epi, nt_m, xtab, xstride, xtiles, st);
    if (nb == 3 && planes == 2 && gbf && onew && !lazy) {
        dim3 grid(max_tiles, n_ids), block(kThreads);
        if (xtab) grid = dim3(8 * xtiles, 1);
        auto kfn = form_row_kernel<3, 2, true, true, 0>;
        const size_t lds = form_lds_bytes<3, 2, 0>();
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kfn), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(kfn, grid, block, lds, st, layers, ids, out_role, epi, nt_m, xtab, xstride);
        return hipGetLastError();
    }
    return hipErrorInvalidValue;
}

}  // namespace psgd
