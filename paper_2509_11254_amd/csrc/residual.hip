// Rank-w outer product on MFMA fused with the error-feedback residual (gfx950).
//
//   residual    S <- S - X_L X_W^T     E_{t+1} = M - P~ Q_t^T        (Algorithm 2, error update)
//   decompress  out <- X_L X_W^T       Delta_hat = P~ Q_t^T          (Algorithm 1, return value)
//
// Both thin operands arrive pre-split into bf16 halves (row-major [len][cp]); the product is
// hi*hi + lo*hi + hi*lo accumulated in fp32 by v_mfma_f32_32x32x16_bf16.  A workgroup owns a
// 128 x 128 tile; wave v owns rows 32v..32v+31 and all 128 columns as four 32 x 32 MFMA blocks.
// MFMA block q, column lane i is bound to matrix column 4*i + q, so that after the four blocks each
// lane holds 4 consecutive columns of 16 rows: S is then read and written with 16-byte accesses
// straight from/to the accumulator layout and never goes through LDS.
#include "psgd_dev.h"

namespace psgd {

constexpr int RT = 128;   // tile rows and columns

template <int NB>   // cp = 32*NB columns of the thin operands (reduction length)
__device__ inline void outer_tile(const LayerDev& L, int rb, int cb, int cp, bf16_t* b_hi, bf16_t* b_lo,
                                  floatx16 (&acc)[4]) {
    constexpr int CPW = 32 * NB + 8;   // LDS row stride (bf16)
    const int t = threadIdx.x;
    const int lane = t & 63, wv = t >> 6;
    const int li = lane & 31, lg = lane >> 5;
    const bf16_t* __restrict__ wn_hi = L.pack[SIDE_W].n_hi;
    const bf16_t* __restrict__ wn_lo = L.pack[SIDE_W].n_lo;
    // stage the W-side tile: matrix column j = cb*128 + jj goes to LDS row (jj & 3) * 32 + (jj >> 2)
    for (int v = t; v < RT * NB * 4; v += kThreads) {
        const int jj = v / (NB * 4), part = v % (NB * 4);
        const int lrow = (jj & 3) * 32 + (jj >> 2);
        const int64_t goff = (int64_t)(cb * RT + jj) * cp + 8 * part;
        *reinterpret_cast<uint4*>(b_hi + lrow * CPW + 8 * part) = *reinterpret_cast<const uint4*>(wn_hi + goff);
        *reinterpret_cast<uint4*>(b_lo + lrow * CPW + 8 * part) = *reinterpret_cast<const uint4*>(wn_lo + goff);
    }
    __syncthreads();
    const bf16_t* __restrict__ ln_hi = L.pack[SIDE_L].n_hi + (int64_t)(rb * RT + 32 * wv + li) * cp + 8 * lg;
    const bf16_t* __restrict__ ln_lo = L.pack[SIDE_L].n_lo + (int64_t)(rb * RT + 32 * wv + li) * cp + 8 * lg;
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[q][v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 2 * NB; ++ks) {
        const bf16x8 ah = *reinterpret_cast<const bf16x8*>(ln_hi + 16 * ks);
        const bf16x8 al = *reinterpret_cast<const bf16x8*>(ln_lo + 16 * ks);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int boff = (32 * q + li) * CPW + 16 * ks + 8 * lg;
            const bf16x8 bh = *reinterpret_cast<const bf16x8*>(b_hi + boff);
            const bf16x8 bl = *reinterpret_cast<const bf16x8*>(b_lo + boff);
            acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bh, acc[q], 0, 0, 0);
            acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, bh, acc[q], 0, 0, 0);
            acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bl, acc[q], 0, 0, 0);
        }
    }
}

template <int NB>
__global__ __launch_bounds__(kThreads) void residual_kernel(const LayerDev* __restrict__ layers,
                                                            const int* __restrict__ ids, int cp) {
    const LayerDev& L = layers[ids[blockIdx.y]];
    const int n_rb = (L.rows + RT - 1) / RT, n_cb = (L.cols + RT - 1) / RT;
    const int tile = blockIdx.x;
    if (tile >= n_rb * n_cb) return;
    const int cb = tile % n_cb, rb = tile / n_cb;
    extern __shared__ __align__(16) unsigned char smem[];
    bf16_t* b_hi = reinterpret_cast<bf16_t*>(smem);
    bf16_t* b_lo = b_hi + RT * (32 * NB + 8);

    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int li = lane & 31, lg = lane >> 5;
    const int col = cb * RT + 4 * li;
    const int row_base = rb * RT + 32 * wv + 4 * lg;
    const bool col_ok = col < L.cols;
    // issue the 16 loads of M first; the operand staging and the MFMAs hide their latency
    float4 m[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int row = row_base + 8 * (v >> 2) + (v & 3);
        const int64_t off = (int64_t)min(row, L.rows - 1) * L.ld + (col_ok ? col : 0);
        m[v] = *reinterpret_cast<const float4*>(L.S + off);
    }
    floatx16 acc[4];
    outer_tile<NB>(L, rb, cb, cp, b_hi, b_lo, acc);
    if (!col_ok) return;
    const bool full = col + 3 < L.cols;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int row = row_base + 8 * (v >> 2) + (v & 3);
        if (row >= L.rows) continue;
        float4 e;
        e.x = m[v].x - acc[0][v]; e.y = m[v].y - acc[1][v]; e.z = m[v].z - acc[2][v]; e.w = m[v].w - acc[3][v];
        float* p = L.S + (int64_t)row * L.ld + col;
        if (full) {
            *reinterpret_cast<float4*>(p) = e;
        } else {
            p[0] = e.x;
            if (col + 1 < L.cols) p[1] = e.y;
            if (col + 2 < L.cols) p[2] = e.z;
        }
    }
}

template <int NB>
__global__ __launch_bounds__(kThreads) void decompress_kernel(const LayerDev* __restrict__ layers,
                                                              const int* __restrict__ ids, int cp,
                                                              void* const* __restrict__ outs, int out_bf16) {
    const int lid = ids[blockIdx.y];
    const LayerDev& L = layers[lid];
    const int n_rb = (L.rows + RT - 1) / RT, n_cb = (L.cols + RT - 1) / RT;
    const int tile = blockIdx.x;
    if (tile >= n_rb * n_cb) return;
    const int cb = tile % n_cb, rb = tile / n_cb;
    extern __shared__ __align__(16) unsigned char smem[];
    bf16_t* b_hi = reinterpret_cast<bf16_t*>(smem);
    bf16_t* b_lo = b_hi + RT * (32 * NB + 8);
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int li = lane & 31, lg = lane >> 5;
    const int col = cb * RT + 4 * li;
    const int row_base = rb * RT + 32 * wv + 4 * lg;
    floatx16 acc[4];
    outer_tile<NB>(L, rb, cb, cp, b_hi, b_lo, acc);
    if (col >= L.cols) return;
    const bool full = col + 3 < L.cols;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int row = row_base + 8 * (v >> 2) + (v & 3);
        if (row >= L.rows) continue;
        const float d[4] = {acc[0][v], acc[1][v], acc[2][v], acc[3][v]};
        const int64_t off = (int64_t)row * L.ld + col;
        if (out_bf16) {
            bf16_t* p = reinterpret_cast<bf16_t*>(outs[lid]) + off;
            if (full) {
                bf16x4 o;
                o[0] = (bf16_t)d[0]; o[1] = (bf16_t)d[1]; o[2] = (bf16_t)d[2]; o[3] = (bf16_t)d[3];
                *reinterpret_cast<bf16x4*>(p) = o;
            } else {
                for (int q = 0; q < 4; ++q) if (col + q < L.cols) p[q] = (bf16_t)d[q];
            }
        } else {
            float* p = reinterpret_cast<float*>(outs[lid]) + off;
            if (full) {
                *reinterpret_cast<float4*>(p) = make_float4(d[0], d[1], d[2], d[3]);
            } else {
                for (int q = 0; q < 4; ++q) if (col + q < L.cols) p[q] = d[q];
            }
        }
    }
}

static size_t outer_lds_bytes(int nb) { return (size_t)2 * RT * (32 * nb + 8) * sizeof(bf16_t); }

template <int NB>
static hipError_t launch_outer_nb(bool decomp, const LayerDev* layers, const int* ids, int n_ids, int max_tiles,
                                  void* const* outs, int out_bf16, hipStream_t st) {
    dim3 grid(max_tiles, n_ids), block(kThreads);
    const size_t lds = outer_lds_bytes(NB);
    const int cp = 32 * NB;
    if (decomp) {
        auto kfn = decompress_kernel<NB>;
        if (lds > 48 * 1024) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kfn),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL(kfn, grid, block, lds, st, layers, ids, cp, outs, out_bf16);
    } else {
        auto kfn = residual_kernel<NB>;
        if (lds > 48 * 1024) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kfn),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL(kfn, grid, block, lds, st, layers, ids, cp);
    }
    return hipGetLastError();
}

hipError_t launch_outer(int nb, bool decomp, const LayerDev* layers, const int* ids, int n_ids, int max_tiles,
                        void* const* outs, int out_bf16, hipStream_t st) {
    if (n_ids <= 0 || max_tiles <= 0) return hipSuccess;
    switch (nb) {
        case 1: return launch_outer_nb<1>(decomp, layers, ids, n_ids, max_tiles, outs, out_bf16, st);
        case 2: return launch_outer_nb<2>(decomp, layers, ids, n_ids, max_tiles, outs, out_bf16, st);
        case 3: return launch_outer_nb<3>(decomp, layers, ids, n_ids, max_tiles, outs, out_bf16, st);
        case 4: return launch_outer_nb<4>(decomp, layers, ids, n_ids, max_tiles, outs, out_bf16, st);
        case 5: return launch_outer_nb<5>(decomp, layers, ids, n_ids, max_tiles, outs, out_bf16, st);
        case 6: return launch_outer_nb<6>(decomp, layers, ids, n_ids, max_tiles, outs, out_bf16, st);
        case 7: return launch_outer_nb<7>(decomp, layers, ids, n_ids, max_tiles, outs, out_bf16, st);
        case 8: return launch_outer_nb<8>(decomp, layers, ids, n_ids, max_tiles, outs, out_bf16, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace psgd
