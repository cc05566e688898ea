// Rank-w outer product on MFMA fused with the error-feedback residual (gfx950).
//
//   residual    S <- S - X_L X_W^T     E_{t+1} = M - P~ Q_t^T        (Algorithm 2, error update)
//               (FORM: S holds E_t, not M; M = mean G + E is formed again on the way, Eq. (7a))
//   decompress  out <- X_L X_W^T       Delta_hat = P~ Q_t^T          (Algorithm 1, return value)
//   msgd        m <- mu m + X_L X_W^T;  X <- X - eta m               (Eq. (7c): momentum SGD on Delta_hat)
//   adam        Adam / AdamW moments and weights from X_L X_W^T      (the base optimizer of Section 5's runs)
//
// Both thin operands arrive pre-split into two or three bf16 planes (row-major [len][cp]); the
// product keeps the 3 (two planes) or 6 (three planes) largest plane products, accumulated in fp32 by
// v_mfma_f32_32x32x16_bf16.  A workgroup owns a
// 128 x 128 tile; wave v owns rows 32v..32v+31 and all 128 columns as four 32 x 32 MFMA blocks.
// MFMA block q, column lane i is bound to matrix column 4*i + q, so that after the four blocks each
// lane holds 4 consecutive columns of 16 rows: S is then read and written with 16-byte accesses
// straight from/to the accumulator layout and never goes through LDS.
#include <type_traits>

#include "psgd_dev.h"

namespace psgd {

constexpr int RT = 128;   // tile rows and columns

template <int PL> __device__ inline bool keep_term(int ka, int kb) { return PL == 2 ? (ka + kb <= 1) : (ka + kb <= 2); }

// KGH = half the k-steps whose row operand is held in registers at a time with two planes (a quarter with three):
// small for the kernels that also hold a tile of M or of the optimizer state, or that want more workgroups per CU
// KEPT: the kept copies of a deferred-residual step instead of the row-major operand copies (a compile-time choice: as a
// run-time one it cost the decompress kernel a tenth of its time)
template <int NB, int PL, int KGH = 2, int KEPT = 0>   // cp = 32*NB columns of the thin operands (reduction length), PL bf16 planes
__device__ inline void outer_tile(const LayerDev& L, int rb, int cb, int cp, bf16_t* b_pl, floatx16 (&acc)[4]) {
    constexpr int CPW = 32 * NB + 8;   // LDS row stride (bf16)
    constexpr int BPL = RT * CPW;      // one plane
    constexpr int KS = 2 * NB;         // k-steps of 16
    constexpr int KG = (PL == 2 ? 2 * KGH : KGH) > 0 ? (PL == 2 ? 2 * KGH : KGH) : 1;
    constexpr int NG = (KS + KG - 1) / KG;
    constexpr int NI = 2 * NB;         // 16-byte pieces of the column operand per thread and plane
    constexpr int SB = KGH < 2 ? 2 : (NI < 4 ? NI : 4);   // pieces requested together
    const int t = threadIdx.x;
    const int lane = t & 63, wv = t >> 6;
    const int li = lane & 31, lg = lane >> 5;
    const PSGD_GLOBAL bf16_t* wk[PL];
    const PSGD_GLOBAL bf16_t* lk[PL];
    // kept: the fragment-order copies that a compress step with a deferred residual leaves of its P~ and Q (in the
    // layers that defer: the launch addresses only those) instead of the row-major ones
    constexpr bool kept = KEPT == 1;
#pragma unroll
    for (int k = 0; k < PL; ++k) {
        wk[k] = as_global(kept ? L.lzf[SIDE_W][k] : L.pack[SIDE_W].n[k]);
        lk[k] = as_global(kept ? L.lzf[SIDE_L][k] : L.pack[SIDE_L].n[k]);
    }
    // Every global round trip on the way to the first MFMA is a stretch in which this workgroup moves no
    // matrix bytes, so the requests go out together: the first group of this wave's row operand, then the
    // column operand of the tile in batches of SB pieces per thread.
    // (offsets of 16-byte pieces: row-major copies by row and column, the kept ones in fragment order)
    const int arow = rb * RT + 32 * wv + li;
    auto piece = [&](int row, int g8) { return kept ? frag_piece(row, g8, cp) * 8 : (int64_t)row * cp + 8 * g8; };
    bf16x8 av[2][KG][PL];
    auto load_rows = [&](int g, bf16x8 (&dst)[KG][PL]) {
#pragma unroll
        for (int j = 0; j < KG; ++j)
            if (g * KG + j < KS) {
#pragma unroll
                for (int k = 0; k < PL; ++k)
                    dst[j][k] = *reinterpret_cast<const PSGD_GLOBAL bf16x8*>(lk[k] + piece(arow, 2 * (g * KG + j) + lg));
            }
    };
    load_rows(0, av[0]);
    // stage the W-side tile: matrix column j = cb*128 + jj goes to LDS row (jj & 3) * 32 + (jj >> 2)
#pragma unroll
    for (int i0 = 0; i0 < NI; i0 += SB) {
        uintx4 tmp[SB][PL];
#pragma unroll
        for (int i = 0; i < SB; ++i) {
            const int v = t + (i0 + i) * kThreads;
            // (kept copies: the tile's 128 rows are one run of whole fragments, thread v takes its v-th piece)
            const int64_t goff = kept ? ((int64_t)cb * (RT / 32) * KS * 64 + v) * 8 : piece(cb * RT + v / (NB * 4), v % (NB * 4));
#pragma unroll
            for (int k = 0; k < PL; ++k)
                if (i0 + i < NI) tmp[i][k] = *reinterpret_cast<const PSGD_GLOBAL uintx4*>(wk[k] + goff);
        }
#pragma unroll
        for (int i = 0; i < SB; ++i) {
            const int v = t + (i0 + i) * kThreads;
            int jj = v / (NB * 4), part = v % (NB * 4);
            if (kept) {
                const int frag = v >> 6, blk = frag / KS;
                jj = 32 * blk + (v & 31);
                part = 2 * (frag - blk * KS) + ((v >> 5) & 1);
            }
            const int lrow = (jj & 3) * 32 + (jj >> 2);
#pragma unroll
            for (int k = 0; k < PL; ++k)
                if (i0 + i < NI) *reinterpret_cast<uintx4*>(b_pl + k * BPL + lrow * CPW + 8 * part) = tmp[i][k];
        }
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[q][v] = 0.f;
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        if (g + 1 < NG) load_rows(g + 1, av[(g + 1) & 1]);      // next group in flight during this one's MFMAs
#pragma unroll
        for (int j = 0; j < KG; ++j) {
            const int ks = g * KG + j;
            if (ks >= KS) continue;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int boff = (32 * q + li) * CPW + 16 * ks + 8 * lg;
                bf16x8 bv[PL];
#pragma unroll
                for (int k = 0; k < PL; ++k) bv[k] = *reinterpret_cast<const bf16x8*>(b_pl + k * BPL + boff);
#pragma unroll
                for (int sum = 2 * (PL - 1); sum >= 0; --sum)
#pragma unroll
                    for (int ka = 0; ka < PL; ++ka) {
                        const int kb = sum - ka;
                        if (kb >= 0 && kb < PL && keep_term<PL>(ka, kb))
                            acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[g & 1][j][ka], bv[kb], acc[q], 0, 0, 0);
                    }
            }
        }
    }
}

// 16 bytes of worker w's gradient at element offset off, widened to fp32
__device__ inline floatx4 load_grad4(const LayerDev& L, int w, int64_t off) {
    const PSGD_GLOBAL void* gw = as_global(as_global(L.G)[w]);
    if (L.gdt == 0) return ld_stream<NT_G>(reinterpret_cast<const PSGD_GLOBAL floatx4*>(reinterpret_cast<const PSGD_GLOBAL float*>(gw) + off));
    const uintx2 v = ld_stream<NT_G>(reinterpret_cast<const PSGD_GLOBAL uintx2*>(reinterpret_cast<const PSGD_GLOBAL bf16_t*>(gw) + off));
    return floatx4{__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xffff0000u), __uint_as_float(v.y << 16),
                   __uint_as_float(v.y & 0xffff0000u)};
}

template <int NB, int PL, bool FORM, bool KEPT>
__global__ __launch_bounds__(kThreads, 2) void residual_kernel(const LayerDev* __restrict__ layers,
                                                                       const int* __restrict__ ids, int cp) {
    const LayerDev& L = layers[ids[blockIdx.y]];
    const int n_rb = (L.rows + RT - 1) / RT, n_cb = (L.cols + RT - 1) / RT;
    const int tile = blockIdx.x;
    if (tile >= n_rb * n_cb) return;
    const int cb = tile % n_cb, rb = tile / n_cb;
    extern __shared__ __align__(16) unsigned char smem[];
    bf16_t* b_pl = reinterpret_cast<bf16_t*>(smem);

    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int li = lane & 31, lg = lane >> 5;
    // (the layer's numbers are read once, here: the compiler cannot move a scalar load across a store that might alias
    // it, and read in place every store of the epilogue waited for a round trip to the scalar cache of its own)
    const int rows = L.rows, cols = L.cols;
    const int64_t ld = L.ld;
    const int col = cb * RT + 4 * li;
    const bool col_ok = col < cols;
    const bool interior = rb * RT + RT <= rows && cb * RT + RT <= cols;     // (uniform) nothing to decide per lane
    // issue the 16 loads of M first; the operand staging and the MFMAs hide their latency
    // addresses = uniform base of tile row 8*(v>>2) + (v&3) (scalar registers) + one per-lane offset
    PSGD_GLOBAL float* tile0 = as_global(L.S) + (int64_t)(rb * RT) * ld + cb * RT;
    const unsigned lane_byte = ((unsigned)(32 * wv + 4 * lg) * (unsigned)ld + 4 * li) * 4u;   // < 2^32: 128 rows
    const int row_lane = rb * RT + 32 * wv + 4 * lg;
    auto at = [&](int k) {
        return reinterpret_cast<PSGD_GLOBAL float*>(reinterpret_cast<PSGD_GLOBAL char*>(tile0 + (int64_t)k * ld) + lane_byte);
    };
    floatx4 m[16];
    auto load_m = [&](auto whole) {
        const int nw = FORM ? L.n_workers : 1;
        const float inv_n = 1.0f / (float)nw;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int k = 8 * (v >> 2) + (v & 3);
            m[v] = floatx4{0.f, 0.f, 0.f, 0.f};
            if (decltype(whole)::value || (col_ok && row_lane + k < rows)) {
                m[v] = ld_stream<NT_M_RES>(reinterpret_cast<const PSGD_GLOBAL floatx4*>(at(k)));
                if (FORM) {
                    // same arithmetic and order as the product kernel's FORM path: (sum of workers) / N + E
                    const int64_t off = (int64_t)(rb * RT + k) * ld + cb * RT + (lane_byte >> 2);
                    floatx4 g = load_grad4(L, 0, off);
                    for (int w = 1; w < nw; ++w) g += load_grad4(L, w, off);
                    m[v] = g * inv_n + m[v];
                }
            }
        }
    };
    if (interior) load_m(std::true_type{}); else load_m(std::false_type{});
    floatx16 acc[4];
    outer_tile<NB, PL, 1, KEPT ? 1 : 0>(L, rb, cb, cp, b_pl, acc);
    if (interior) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const floatx4 e = {m[v].x - acc[0][v], m[v].y - acc[1][v], m[v].z - acc[2][v], m[v].w - acc[3][v]};
            st_stream<NT_E_OUT>(reinterpret_cast<PSGD_GLOBAL floatx4*>(at(8 * (v >> 2) + (v & 3))), e);
        }
        return;
    }
    if (!col_ok) return;
    const bool full = col + 3 < cols;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int k = 8 * (v >> 2) + (v & 3);
        if (row_lane + k >= rows) continue;
        floatx4 e;
        e.x = m[v].x - acc[0][v]; e.y = m[v].y - acc[1][v]; e.z = m[v].z - acc[2][v]; e.w = m[v].w - acc[3][v];
        PSGD_GLOBAL float* p = at(k);
        if (full) {
            st_stream<NT_E_OUT>(reinterpret_cast<PSGD_GLOBAL floatx4*>(p), e);
        } else {
            p[0] = e.x;
            if (col + 1 < cols) p[1] = e.y;
            if (col + 2 < cols) p[2] = e.z;
        }
    }
}

// Write-only: nothing but other workgroups' stores hides this one's operand round trip and MFMA phase, so as many
// workgroups per compute unit as the operand tile in LDS allows (four at NB * PL <= 6).
template <int NB, int PL, bool KEPT>
__global__ __launch_bounds__(kThreads, (NB * PL <= 6 ? 4 : 2)) void decompress_kernel(const LayerDev* __restrict__ layers,
                                                              const int* __restrict__ ids, int cp,
                                                              void* const* __restrict__ outs, int out_bf16) {
    const int lid = ids[blockIdx.y];
    const LayerDev& L = layers[lid];
    const int n_rb = (L.rows + RT - 1) / RT, n_cb = (L.cols + RT - 1) / RT;
    const int tile = blockIdx.x;
    if (tile >= n_rb * n_cb) return;
    const int cb = tile % n_cb, rb = tile / n_cb;
    extern __shared__ __align__(16) unsigned char smem[];
    bf16_t* b_pl = reinterpret_cast<bf16_t*>(smem);
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int li = lane & 31, lg = lane >> 5;
    const int col = cb * RT + 4 * li;
    const int row_base = rb * RT + 32 * wv + 4 * lg;
    // (what the stores need is read before them: the compiler cannot move a scalar load across a store that might
    // alias it, and left in place every one of the 16 stores waited for its own round trip to the scalar cache)
    const int rows = L.rows, cols = L.cols;
    const int64_t ld = L.ld;
    void* const outp = outs[lid];
    floatx16 acc[4];
    outer_tile<NB, PL, 2, KEPT ? 1 : 0>(L, rb, cb, cp, b_pl, acc);
    const int64_t off0 = (int64_t)row_base * ld + col;
    if (rb * RT + RT <= rows && cb * RT + RT <= cols) {
        // interior tile: sixteen stores, nothing to decide
        if (out_bf16) {
            PSGD_GLOBAL bf16_t* p = as_global(reinterpret_cast<bf16_t*>(outp)) + off0;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                bf16x4 o;
                o[0] = (bf16_t)acc[0][v]; o[1] = (bf16_t)acc[1][v]; o[2] = (bf16_t)acc[2][v]; o[3] = (bf16_t)acc[3][v];
                st_stream<NT_DEC>(reinterpret_cast<PSGD_GLOBAL bf16x4*>(p + (int64_t)(8 * (v >> 2) + (v & 3)) * ld), o);
            }
        } else {
            PSGD_GLOBAL float* p = as_global(reinterpret_cast<float*>(outp)) + off0;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const floatx4 o = {acc[0][v], acc[1][v], acc[2][v], acc[3][v]};
                st_stream<NT_DEC>(reinterpret_cast<PSGD_GLOBAL floatx4*>(p + (int64_t)(8 * (v >> 2) + (v & 3)) * ld), o);
            }
        }
        return;
    }
    if (col >= cols) return;
    const bool full = col + 3 < cols;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int row = row_base + 8 * (v >> 2) + (v & 3);
        if (row >= rows) continue;
        const float d[4] = {acc[0][v], acc[1][v], acc[2][v], acc[3][v]};
        const int64_t off = (int64_t)row * ld + col;
        if (out_bf16) {
            PSGD_GLOBAL bf16_t* p = as_global(reinterpret_cast<bf16_t*>(outp)) + off;
            if (full) {
                bf16x4 o;
                o[0] = (bf16_t)d[0]; o[1] = (bf16_t)d[1]; o[2] = (bf16_t)d[2]; o[3] = (bf16_t)d[3];
                st_stream<NT_DEC>(reinterpret_cast<PSGD_GLOBAL bf16x4*>(p), o);
            } else {
                for (int q = 0; q < 4; ++q) if (col + q < cols) p[q] = (bf16_t)d[q];
            }
        } else {
            PSGD_GLOBAL float* p = as_global(reinterpret_cast<float*>(outp)) + off;
            if (full) {
                floatx4 o = {d[0], d[1], d[2], d[3]};
                st_stream<NT_DEC>(reinterpret_cast<PSGD_GLOBAL floatx4*>(p), o);
            } else {
                for (int q = 0; q < 4; ++q) if (col + q < cols) p[q] = d[q];
            }
        }
    }
}

// Decompress fused with the momentum-SGD update of Eq. (7c): Delta_hat never goes to memory.
//   m_t = mu m_{t-1} + P~ Q^T,   X_{t+1} = X_t - eta m_t      (both rows x cols fp32 with the layer's ld, in place)
template <int NB, int PL, bool KEPT>
__global__ __launch_bounds__(kThreads, 2) void msgd_kernel(const LayerDev* __restrict__ layers,
                                                           const int* __restrict__ ids, int cp,
                                                           float* const* __restrict__ moms,
                                                           float* const* __restrict__ xs, float mu, float eta) {
    const int lid = ids[blockIdx.y];
    const LayerDev& L = layers[lid];
    const int n_rb = (L.rows + RT - 1) / RT, n_cb = (L.cols + RT - 1) / RT;
    const int tile = blockIdx.x;
    if (tile >= n_rb * n_cb) return;
    const int cb = tile % n_cb, rb = tile / n_cb;
    extern __shared__ __align__(16) unsigned char smem[];
    bf16_t* b_pl = reinterpret_cast<bf16_t*>(smem);
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int li = lane & 31, lg = lane >> 5;
    const int rows = L.rows, cols = L.cols;          // (read once, before any store: see residual_kernel)
    const int64_t ld = L.ld;
    const int col = cb * RT + 4 * li;
    const bool col_ok = col < cols;
    const bool interior = rb * RT + RT <= rows && cb * RT + RT <= cols;
    const int64_t tile_off = (int64_t)(rb * RT) * ld + cb * RT;
    PSGD_GLOBAL float* m0 = as_global(moms[lid]) + tile_off;
    PSGD_GLOBAL float* x0 = as_global(xs[lid]) + tile_off;
    const unsigned lane_byte = ((unsigned)(32 * wv + 4 * lg) * (unsigned)ld + 4 * li) * 4u;   // < 2^32: 128 rows
    const int row_lane = rb * RT + 32 * wv + 4 * lg;
    auto at = [&](PSGD_GLOBAL float* base, int k) {
        return reinterpret_cast<PSGD_GLOBAL float*>(reinterpret_cast<PSGD_GLOBAL char*>(base + (int64_t)k * ld) + lane_byte);
    };
    // momentum and weights of the tile are requested first; the operand staging and the MFMAs hide the latency
    floatx4 mo[16], xo[16];
    auto load_state = [&](auto whole) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int k = 8 * (v >> 2) + (v & 3);
            mo[v] = floatx4{0.f, 0.f, 0.f, 0.f};
            xo[v] = floatx4{0.f, 0.f, 0.f, 0.f};
            if (decltype(whole)::value || (col_ok && row_lane + k < rows)) {
                mo[v] = ld_stream<NT_OPT_IN>(reinterpret_cast<const PSGD_GLOBAL floatx4*>(at(m0, k)));
                xo[v] = ld_stream<NT_OPT_IN>(reinterpret_cast<const PSGD_GLOBAL floatx4*>(at(x0, k)));
            }
        }
    };
    if (interior) load_state(std::true_type{}); else load_state(std::false_type{});
    floatx16 acc[4];
    outer_tile<NB, PL, 1, KEPT ? 1 : 0>(L, rb, cb, cp, b_pl, acc);
    if (interior) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int k = 8 * (v >> 2) + (v & 3);
            const floatx4 d = {acc[0][v], acc[1][v], acc[2][v], acc[3][v]};
            const floatx4 mn = mo[v] * mu + d;
            const floatx4 xn = xo[v] - mn * eta;
            st_stream<NT_OPT_OUT>(reinterpret_cast<PSGD_GLOBAL floatx4*>(at(m0, k)), mn);
            st_stream<NT_OPT_OUT>(reinterpret_cast<PSGD_GLOBAL floatx4*>(at(x0, k)), xn);
        }
        return;
    }
    if (!col_ok) return;
    const bool full = col + 3 < cols;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int k = 8 * (v >> 2) + (v & 3);
        if (row_lane + k >= rows) continue;
        const floatx4 d = {acc[0][v], acc[1][v], acc[2][v], acc[3][v]};
        const floatx4 mn = mo[v] * mu + d;
        const floatx4 xn = xo[v] - mn * eta;
        PSGD_GLOBAL float* pm = at(m0, k);
        PSGD_GLOBAL float* px = at(x0, k);
        if (full) {
            st_stream<NT_OPT_OUT>(reinterpret_cast<PSGD_GLOBAL floatx4*>(pm), mn);
            st_stream<NT_OPT_OUT>(reinterpret_cast<PSGD_GLOBAL floatx4*>(px), xn);
        } else {
            for (int q = 0; q < 4; ++q)
                if (col + q < cols) { pm[q] = mn[q]; px[q] = xn[q]; }
        }
    }
}

// Decompress fused with Adam on Delta_hat (the base optimizer of the paper's pre-training and fine-tuning runs,
// Section 5 and Appendix C; the update itself is the published one, with decoupled weight decay):
//   m <- b1 m + (1 - b1) D,  v <- b2 v + (1 - b2) D^2,  X <- X - step m / (sqrt(v) rs2 + eps) - decay X
// with step = eta / (1 - b1^t), rs2 = 1 / sqrt(1 - b2^t), decay = eta lambda folded by the host.
struct AdamArgs { float b1, b2, c1, c2, step, rs2, eps, decay; };

template <int NB, int PL, bool KEPT>
__global__ __launch_bounds__(kThreads, 2) void adam_kernel(const LayerDev* __restrict__ layers,
                                                           const int* __restrict__ ids, int cp,
                                                           float* const* __restrict__ m1s,
                                                           float* const* __restrict__ m2s,
                                                           float* const* __restrict__ xs, AdamArgs a) {
    const int lid = ids[blockIdx.y];
    const LayerDev& L = layers[lid];
    const int n_rb = (L.rows + RT - 1) / RT, n_cb = (L.cols + RT - 1) / RT;
    const int tile = blockIdx.x;
    if (tile >= n_rb * n_cb) return;
    const int cb = tile % n_cb, rb = tile / n_cb;
    extern __shared__ __align__(16) unsigned char smem[];
    bf16_t* b_pl = reinterpret_cast<bf16_t*>(smem);
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int li = lane & 31, lg = lane >> 5;
    const int rows = L.rows, cols = L.cols;          // (read once, before any store: see residual_kernel)
    const int64_t ld = L.ld;
    const int col = cb * RT + 4 * li;
    const bool col_ok = col < cols;
    const bool interior = rb * RT + RT <= rows && cb * RT + RT <= cols;
    const int64_t tile_off = (int64_t)(rb * RT) * ld + cb * RT;
    PSGD_GLOBAL float* m0 = as_global(m1s[lid]) + tile_off;
    PSGD_GLOBAL float* v0 = as_global(m2s[lid]) + tile_off;
    PSGD_GLOBAL float* x0 = as_global(xs[lid]) + tile_off;
    const unsigned lane_byte = ((unsigned)(32 * wv + 4 * lg) * (unsigned)ld + 4 * li) * 4u;   // < 2^32: 128 rows
    const int row_lane = rb * RT + 32 * wv + 4 * lg;
    auto at = [&](PSGD_GLOBAL float* base, int k) {
        return reinterpret_cast<PSGD_GLOBAL float*>(reinterpret_cast<PSGD_GLOBAL char*>(base + (int64_t)k * ld) + lane_byte);
    };
    // the two moments of the tile are requested before the product (its staging and MFMAs hide their latency);
    // the weights, needed last, are read in the epilogue
    floatx4 mo[16], vo[16];
    auto load_state = [&](auto whole) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int k = 8 * (v >> 2) + (v & 3);
            mo[v] = floatx4{0.f, 0.f, 0.f, 0.f};
            vo[v] = floatx4{0.f, 0.f, 0.f, 0.f};
            if (decltype(whole)::value || (col_ok && row_lane + k < rows)) {
                mo[v] = ld_stream<NT_OPT_IN>(reinterpret_cast<const PSGD_GLOBAL floatx4*>(at(m0, k)));
                vo[v] = ld_stream<NT_OPT_IN>(reinterpret_cast<const PSGD_GLOBAL floatx4*>(at(v0, k)));
            }
        }
    };
    if (interior) load_state(std::true_type{}); else load_state(std::false_type{});
    floatx16 acc[4];
    outer_tile<NB, PL, 1, KEPT ? 1 : 0>(L, rb, cb, cp, b_pl, acc);
    auto update = [&](int v, const floatx4& xo, floatx4& mn, floatx4& vn, floatx4& xn) {
        const floatx4 d = {acc[0][v], acc[1][v], acc[2][v], acc[3][v]};
        mn = mo[v] * a.b1 + d * a.c1;
        vn = vo[v] * a.b2 + (d * d) * a.c2;
#pragma unroll
        for (int q = 0; q < 4; ++q)
            xn[q] = xo[q] - a.step * (mn[q] / (sqrtf(vn[q]) * a.rs2 + a.eps)) - a.decay * xo[q];
    };
    if (interior) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            floatx4 xo[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) xo[u] = ld_stream<NT_OPT_IN>(reinterpret_cast<const PSGD_GLOBAL floatx4*>(at(x0, 8 * g + u)));
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int v = 4 * g + u, k = 8 * g + u;
                floatx4 mn, vn, xn;
                update(v, xo[u], mn, vn, xn);
                st_stream<NT_OPT_OUT>(reinterpret_cast<PSGD_GLOBAL floatx4*>(at(m0, k)), mn);
                st_stream<NT_OPT_OUT>(reinterpret_cast<PSGD_GLOBAL floatx4*>(at(v0, k)), vn);
                st_stream<NT_OPT_OUT>(reinterpret_cast<PSGD_GLOBAL floatx4*>(at(x0, k)), xn);
            }
        }
        return;
    }
    if (!col_ok) return;
    const bool full = col + 3 < cols;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        floatx4 xo[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int k = 8 * g + u;
            xo[u] = floatx4{0.f, 0.f, 0.f, 0.f};
            if (row_lane + k < rows) {
                if (full) xo[u] = ld_stream<NT_OPT_IN>(reinterpret_cast<const PSGD_GLOBAL floatx4*>(at(x0, k)));
                else for (int q = 0; q < 4; ++q) if (col + q < cols) xo[u][q] = at(x0, k)[q];
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int v = 4 * g + u, k = 8 * g + u;
            if (row_lane + k >= rows) continue;
            floatx4 mn, vn, xn;
            update(v, xo[u], mn, vn, xn);
            PSGD_GLOBAL float* pm = at(m0, k);
            PSGD_GLOBAL float* pv = at(v0, k);
            PSGD_GLOBAL float* px = at(x0, k);
            if (full) {
                st_stream<NT_OPT_OUT>(reinterpret_cast<PSGD_GLOBAL floatx4*>(pm), mn);
                st_stream<NT_OPT_OUT>(reinterpret_cast<PSGD_GLOBAL floatx4*>(pv), vn);
                st_stream<NT_OPT_OUT>(reinterpret_cast<PSGD_GLOBAL floatx4*>(px), xn);
            } else {
                for (int q = 0; q < 4; ++q)
                    if (col + q < cols) { pm[q] = mn[q]; pv[q] = vn[q]; px[q] = xn[q]; }
            }
        }
    }
}

static size_t outer_lds_bytes(int nb, int planes) { return (size_t)planes * RT * (32 * nb + 8) * sizeof(bf16_t); }

template <int NB, int PL>
static hipError_t launch_outer_nb(bool decomp, bool form, bool kept, const LayerDev* layers, const int* ids, int n_ids,
                                  int max_tiles, void* const* outs, int out_bf16, hipStream_t st) {
    dim3 grid(max_tiles, n_ids), block(kThreads);
    const size_t lds = outer_lds_bytes(NB, PL);
    const int cp = 32 * NB;
    // (kept copies exist up to width 128)
    if (kept && NB > 4) return hipErrorInvalidValue;
    if (decomp) {
        auto kfn = (kept && NB <= 4) ? decompress_kernel<NB, PL, (NB <= 4)> : decompress_kernel<NB, PL, false>;
        if (lds > 48 * 1024) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kfn),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL(kfn, grid, block, lds, st, layers, ids, cp, outs, out_bf16);
    } else if (form) {
        if (kept) return hipErrorInvalidValue;      // (the deferred residual lives in the stored M)
        auto kfn = residual_kernel<NB, PL, true, false>;
        if (lds > 48 * 1024) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kfn),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL(kfn, grid, block, lds, st, layers, ids, cp);
    } else {
        auto kfn = (kept && NB <= 4) ? residual_kernel<NB, PL, false, (NB <= 4)> : residual_kernel<NB, PL, false, false>;
        if (lds > 48 * 1024) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kfn),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL(kfn, grid, block, lds, st, layers, ids, cp);
    }
    return hipGetLastError();
}

template <int NB, int PL>
static hipError_t launch_msgd_nb(const LayerDev* layers, const int* ids, int n_ids, int max_tiles, float* const* moms,
                                 float* const* xs, float mu, float eta, bool kept, hipStream_t st) {
    dim3 grid(max_tiles, n_ids), block(kThreads);
    const size_t lds = outer_lds_bytes(NB, PL);
    if (kept && NB > 4) return hipErrorInvalidValue;
    auto kfn = (kept && NB <= 4) ? msgd_kernel<NB, PL, (NB <= 4)> : msgd_kernel<NB, PL, false>;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kfn),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kfn, grid, block, lds, st, layers, ids, 32 * NB, moms, xs, mu, eta);
    return hipGetLastError();
}

// moms, xs: device arrays of per-layer device pointers; kept: as for launch_outer
hipError_t launch_msgd(int nb, int planes, const LayerDev* layers, const int* ids, int n_ids, int max_tiles,
                       float* const* moms, float* const* xs, float mu, float eta, bool kept, hipStream_t st) {
    if (n_ids <= 0 || max_tiles <= 0) return hipSuccess;
#define PSGD_CASE(N)                                                                                       \
    case N:                                                                                                \
        return planes == 2 ? launch_msgd_nb<N, 2>(layers, ids, n_ids, max_tiles, moms, xs, mu, eta, kept, st)   \
                           : launch_msgd_nb<N, 3>(layers, ids, n_ids, max_tiles, moms, xs, mu, eta, kept, st);
    switch (nb) {
        PSGD_CASE(1) PSGD_CASE(2) PSGD_CASE(3) PSGD_CASE(4) PSGD_CASE(5) PSGD_CASE(6)
        default: return hipErrorInvalidValue;
    }
#undef PSGD_CASE
}

template <int NB, int PL>
static hipError_t launch_adam_nb(const LayerDev* layers, const int* ids, int n_ids, int max_tiles, float* const* m1s,
                                 float* const* m2s, float* const* xs, const AdamArgs& a, bool kept, hipStream_t st) {
    dim3 grid(max_tiles, n_ids), block(kThreads);
    const size_t lds = outer_lds_bytes(NB, PL);
    if (kept && NB > 4) return hipErrorInvalidValue;
    auto kfn = (kept && NB <= 4) ? adam_kernel<NB, PL, (NB <= 4)> : adam_kernel<NB, PL, false>;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kfn),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kfn, grid, block, lds, st, layers, ids, 32 * NB, m1s, m2s, xs, a);
    return hipGetLastError();
}

// m1s, m2s, xs: device arrays of per-layer device pointers; coef = {b1, b2, 1 - b1, 1 - b2, eta / (1 - b1^t),
// 1 / sqrt(1 - b2^t), eps, eta * weight decay}
hipError_t launch_adam(int nb, int planes, const LayerDev* layers, const int* ids, int n_ids, int max_tiles,
                       float* const* m1s, float* const* m2s, float* const* xs, const float* coef, bool kept,
                       hipStream_t st) {
    if (n_ids <= 0 || max_tiles <= 0) return hipSuccess;
    const AdamArgs a = {coef[0], coef[1], coef[2], coef[3], coef[4], coef[5], coef[6], coef[7]};
#define PSGD_CASE(N)                                                                                       \
    case N:                                                                                                \
        return planes == 2 ? launch_adam_nb<N, 2>(layers, ids, n_ids, max_tiles, m1s, m2s, xs, a, kept, st)     \
                           : launch_adam_nb<N, 3>(layers, ids, n_ids, max_tiles, m1s, m2s, xs, a, kept, st);
    switch (nb) {
        PSGD_CASE(1) PSGD_CASE(2) PSGD_CASE(3) PSGD_CASE(4) PSGD_CASE(5) PSGD_CASE(6)
        default: return hipErrorInvalidValue;
    }
#undef PSGD_CASE
}

// kept: the factors are the fragment-order copies that the last compress step left in the addressed layers (all of
// them defer their residual)
hipError_t launch_outer(int nb, int planes, bool decomp, bool form, bool kept, const LayerDev* layers, const int* ids,
                        int n_ids, int max_tiles, void* const* outs, int out_bf16, hipStream_t st) {
    if (n_ids <= 0 || max_tiles <= 0) return hipSuccess;
#define PSGD_CASE(N)                                                                                              \
    case N:                                                                                                       \
        return planes == 2 ? launch_outer_nb<N, 2>(decomp, form, kept, layers, ids, n_ids, max_tiles, outs, out_bf16, st) \
                           : launch_outer_nb<N, 3>(decomp, form, kept, layers, ids, n_ids, max_tiles, outs, out_bf16, st);
    switch (nb) {
        PSGD_CASE(1) PSGD_CASE(2) PSGD_CASE(3) PSGD_CASE(4) PSGD_CASE(5) PSGD_CASE(6)
        default: return hipErrorInvalidValue;
    }
#undef PSGD_CASE
}

}  // namespace psgd
