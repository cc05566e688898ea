// Tall-skinny products of the power iteration on MFMA (gfx950), one streaming pass over S each.
//
//   row mode    Y_L = S   X_W      (rows x w) = (rows x cols)(cols x w)     e.g. P = M Q      (Algorithm 1)
//   column mode Y_W = S^T X_L      (cols x w) = (cols x rows)(rows x w)     e.g. Q = M^T P~   (Algorithm 1)
//
// With FORM the pass also forms M = (1/N) sum_i G^(i) + E (Eq. (7a) averaged over the workers)
// from the gradient buffers and the error buffer, uses it for the product and stores it in place
// of E, so that the second pass and the residual read 4 bytes per element instead of N*sizeof(G)+4.
//
// Arithmetic: M and X are split into two bf16 halves each (x = hi + lo, |x - hi - lo| <= 2^-17 |x|)
// and the product is accumulated in fp32 as hi*hi + lo*hi + hi*lo with v_mfma_f32_32x32x16_bf16.
// The S tile goes global -> registers (coalesced 16-byte loads, summed over workers) -> LDS in the
// k-contiguous layout the MFMA A operand wants; the thin operand arrives pre-split and transposed.
#include "psgd_dev.h"

namespace psgd {

constexpr int BK = 64;          // reduction chunk
constexpr int BT = 128;         // output rows per workgroup (4 waves x 32)
constexpr int LDSW = BK + 8;    // LDS row stride in bf16 elements (144 bytes)

__device__ inline float4 ld_f32x4(const float* p) { return *reinterpret_cast<const float4*>(p); }

__device__ inline float4 ld_bf16x4(const bf16_t* p) {
    uint2 v = *reinterpret_cast<const uint2*>(p);
    float4 o;
    o.x = __uint_as_float(v.x << 16);
    o.y = __uint_as_float(v.x & 0xffff0000u);
    o.z = __uint_as_float(v.y << 16);
    o.w = __uint_as_float(v.y & 0xffff0000u);
    return o;
}

// Eight 4-element pieces of M (or of S when !FORM), piece u at (row0 + u*row_step, col); zero outside
// the matrix.  The loop over the workers is outermost so that the eight loads of one worker are in
// flight together.  Addresses are clamped into the matrix and masked afterwards (no divergent loads).
template <bool FORM>
__device__ inline void load_m4x8(const LayerDev& L, int row0, int row_step, int col, float inv_n, float4 (&m)[8]) {
    const bool col_ok = col < L.cols;
    const int colc = col_ok ? col : 0;
    int64_t off[8];
    bool ok[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const int row = row0 + u * row_step;
        ok[u] = col_ok && row < L.rows;
        off[u] = (int64_t)min(row, L.rows - 1) * L.ld + colc;
    }
    if (FORM) {
#pragma unroll
        for (int u = 0; u < 8; ++u) m[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (L.gdt == 0) {
            for (int w = 0; w < L.n_workers; ++w) {
                const float* __restrict__ g = reinterpret_cast<const float*>(L.G[w]);
                float4 x[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) x[u] = ld_f32x4(g + off[u]);
#pragma unroll
                for (int u = 0; u < 8; ++u) { m[u].x += x[u].x; m[u].y += x[u].y; m[u].z += x[u].z; m[u].w += x[u].w; }
            }
        } else {
            for (int w = 0; w < L.n_workers; ++w) {
                const bf16_t* __restrict__ g = reinterpret_cast<const bf16_t*>(L.G[w]);
                float4 x[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) x[u] = ld_bf16x4(g + off[u]);
#pragma unroll
                for (int u = 0; u < 8; ++u) { m[u].x += x[u].x; m[u].y += x[u].y; m[u].z += x[u].z; m[u].w += x[u].w; }
            }
        }
        float4 e[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) e[u] = ld_f32x4(L.S + off[u]);
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            m[u].x = m[u].x * inv_n + e[u].x; m[u].y = m[u].y * inv_n + e[u].y;
            m[u].z = m[u].z * inv_n + e[u].z; m[u].w = m[u].w * inv_n + e[u].w;
        }
    } else {
#pragma unroll
        for (int u = 0; u < 8; ++u) m[u] = ld_f32x4(L.S + off[u]);
    }
    const bool k1 = col + 1 < L.cols, k2 = col + 2 < L.cols, k3 = col + 3 < L.cols;
#pragma unroll
    for (int u = 0; u < 8; ++u) {   // ragged edges: padding up to ld and rows past the end are not data
        m[u].x = ok[u] ? m[u].x : 0.f;
        m[u].y = (ok[u] && k1) ? m[u].y : 0.f;
        m[u].z = (ok[u] && k2) ? m[u].z : 0.f;
        m[u].w = (ok[u] && k3) ? m[u].w : 0.f;
    }
}

__device__ inline void store_m4(const LayerDev& L, int row, int col, float4 m) {
    if (row >= L.rows || col >= L.cols) return;
    float* p = L.S + (int64_t)row * L.ld + col;
    if (col + 3 < L.cols) {
        *reinterpret_cast<float4*>(p) = m;
    } else {
        p[0] = m.x;
        if (col + 1 < L.cols) p[1] = m.y;
        if (col + 2 < L.cols) p[2] = m.z;
    }
}

__device__ inline void split_bf16(float x, bf16_t& hi, bf16_t& lo) {
    hi = (bf16_t)x;
    lo = (bf16_t)(x - (float)hi);
}

template <int NB, bool COLMODE, bool FORM>
__global__ __launch_bounds__(kThreads) void prod_kernel(const LayerDev* __restrict__ layers,
                                                        const int* __restrict__ ids, int cp) {
    const LayerDev& L = layers[ids[blockIdx.y]];
    const int out_side = COLMODE ? SIDE_W : SIDE_L;
    const int src_side = COLMODE ? SIDE_L : SIDE_W;
    const int out_len = COLMODE ? L.cols : L.rows;
    const int red_len = COLMODE ? L.rows : L.cols;
    const int n_ob = (out_len + BT - 1) / BT;
    const int n_split = COLMODE ? L.split_col : L.split_row;
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
    bf16_t* a_hi = reinterpret_cast<bf16_t*>(smem);
    bf16_t* a_lo = a_hi + BT * LDSW;
    bf16_t* b_hi = a_lo + BT * LDSW;
    bf16_t* b_lo = b_hi + NB * 32 * LDSW;

    const int t = threadIdx.x;
    const int lane = t & 63, wv = t >> 6;
    const int li = lane & 31, lg = lane >> 5;
    const float inv_n = 1.0f / (float)L.n_workers;
    const int src_lenP = side_lenP(L, src_side);
    const bf16_t* __restrict__ xt_hi = L.pack[src_side].t_hi;
    const bf16_t* __restrict__ xt_lo = L.pack[src_side].t_lo;

    floatx16 acc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[nb][v] = 0.f;

    for (int ch = ch0; ch < ch1; ++ch) {
        const int k0 = ch * BK;
        // ---- S tile: global -> registers -> (store M) -> split -> LDS
        if (!COLMODE) {
            const int c4 = t & 15, r0 = t >> 4;
            const int col = k0 + 4 * c4;
            float4 m[8];
            load_m4x8<FORM>(L, ob * BT + r0, 16, col, inv_n, m);
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int row = r0 + 16 * u;
                if (FORM) store_m4(L, ob * BT + row, col, m[u]);
                bf16x4 h, l;
                bf16_t hh, ll;
                split_bf16(m[u].x, hh, ll); h[0] = hh; l[0] = ll;
                split_bf16(m[u].y, hh, ll); h[1] = hh; l[1] = ll;
                split_bf16(m[u].z, hh, ll); h[2] = hh; l[2] = ll;
                split_bf16(m[u].w, hh, ll); h[3] = hh; l[3] = ll;
                *reinterpret_cast<bf16x4*>(a_hi + row * LDSW + 4 * c4) = h;
                *reinterpret_cast<bf16x4*>(a_lo + row * LDSW + 4 * c4) = l;
            }
        } else {
            const int c4 = t & 31, rg = t >> 5;
            const int col = ob * BT + 4 * c4;
            float4 m[8];
            load_m4x8<FORM>(L, k0 + 8 * rg, 1, col, inv_n, m);
            if (FORM) {
#pragma unroll
                for (int u = 0; u < 8; ++u) store_m4(L, k0 + 8 * rg + u, col, m[u]);
            }
            bf16x8 h[4], l[4];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                bf16_t hh, ll;
                split_bf16(m[u].x, hh, ll); h[0][u] = hh; l[0][u] = ll;
                split_bf16(m[u].y, hh, ll); h[1][u] = hh; l[1][u] = ll;
                split_bf16(m[u].z, hh, ll); h[2][u] = hh; l[2][u] = ll;
                split_bf16(m[u].w, hh, ll); h[3][u] = hh; l[3][u] = ll;
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                *reinterpret_cast<bf16x8*>(a_hi + (4 * c4 + q) * LDSW + 8 * rg) = h[q];
                *reinterpret_cast<bf16x8*>(a_lo + (4 * c4 + q) * LDSW + 8 * rg) = l[q];
            }
        }
        // ---- thin operand chunk: pre-split, transposed [cp][lenP] -> LDS [cp][LDSW]
#pragma unroll
        for (int it = 0; it < NB; ++it) {
            const int v = t + it * kThreads;        // 0 .. 32*NB*8-1
            const int c = v >> 3, part = v & 7;
            const int64_t goff = (int64_t)c * src_lenP + k0 + 8 * part;
            *reinterpret_cast<uint4*>(b_hi + c * LDSW + 8 * part) = *reinterpret_cast<const uint4*>(xt_hi + goff);
            *reinterpret_cast<uint4*>(b_lo + c * LDSW + 8 * part) = *reinterpret_cast<const uint4*>(xt_lo + goff);
        }
        __syncthreads();
        // ---- MFMA: 32 output rows per wave, NB blocks of 32 columns, 4 k-steps of 16
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            const int aoff = (32 * wv + li) * LDSW + 16 * ks + 8 * lg;
            const bf16x8 ah = *reinterpret_cast<const bf16x8*>(a_hi + aoff);
            const bf16x8 al = *reinterpret_cast<const bf16x8*>(a_lo + aoff);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const int boff = (32 * nb + li) * LDSW + 16 * ks + 8 * lg;
                const bf16x8 bh = *reinterpret_cast<const bf16x8*>(b_hi + boff);
                const bf16x8 bl = *reinterpret_cast<const bf16x8*>(b_lo + boff);
                acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bh, acc[nb], 0, 0, 0);
                acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, bh, acc[nb], 0, 0, 0);
                acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bl, acc[nb], 0, 0, 0);
            }
        }
        __syncthreads();
    }
    // ---- partial product of this split: part[out_side][sp][lenP][cp]
    const int out_lenP = side_lenP(L, out_side);
    float* __restrict__ dst = L.part[out_side] + ((int64_t)sp * out_lenP + (int64_t)ob * BT + 32 * wv) * cp;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = 8 * (v >> 2) + 4 * lg + (v & 3);
            dst[(int64_t)row * cp + 32 * nb + li] = acc[nb][v];
        }
}

size_t prod_lds_bytes(int nb) { return (size_t)(2 * BT * LDSW + 2 * nb * 32 * LDSW) * sizeof(bf16_t); }

template <int NB>
static hipError_t launch_nb(bool colmode, bool form, const LayerDev* layers, const int* ids, int n_ids,
                            int max_tiles, hipStream_t st) {
    if (n_ids <= 0 || max_tiles <= 0) return hipSuccess;
    dim3 grid(max_tiles, n_ids), block(kThreads);
    const size_t lds = prod_lds_bytes(NB);
    const int cp = 32 * NB;
#define PSGD_LAUNCH(C, F)                                                                              \
    do {                                                                                               \
        auto kfn = prod_kernel<NB, C, F>;                                                              \
        if (lds > 48 * 1024) {                                                                         \
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kfn),                     \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);  \
            if (e != hipSuccess) return e;                                                             \
        }                                                                                              \
        hipLaunchKernelGGL(kfn, grid, block, lds, st, layers, ids, cp);                                \
    } while (0)
    if (colmode) { if (form) PSGD_LAUNCH(true, true); else PSGD_LAUNCH(true, false); }
    else         { if (form) PSGD_LAUNCH(false, true); else PSGD_LAUNCH(false, false); }
#undef PSGD_LAUNCH
    return hipGetLastError();
}

// nb = width / 32 of the thin operand (1..8).
hipError_t launch_prod(int nb, bool colmode, bool form, const LayerDev* layers, const int* ids, int n_ids,
                       int max_tiles, hipStream_t st) {
    switch (nb) {
        case 1: return launch_nb<1>(colmode, form, layers, ids, n_ids, max_tiles, st);
        case 2: return launch_nb<2>(colmode, form, layers, ids, n_ids, max_tiles, st);
        case 3: return launch_nb<3>(colmode, form, layers, ids, n_ids, max_tiles, st);
        case 4: return launch_nb<4>(colmode, form, layers, ids, n_ids, max_tiles, st);
        case 5: return launch_nb<5>(colmode, form, layers, ids, n_ids, max_tiles, st);
        case 6: return launch_nb<6>(colmode, form, layers, ids, n_ids, max_tiles, st);
        case 7: return launch_nb<7>(colmode, form, layers, ids, n_ids, max_tiles, st);
        case 8: return launch_nb<8>(colmode, form, layers, ids, n_ids, max_tiles, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace psgd
