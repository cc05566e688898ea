// Kernels on the thin (len x w) matrices of the compressor: operand packing, reduction of the
// split products, the orthonormaliser, the Rayleigh-Ritz step of the refresh, random start blocks.
//
// The small factorisation of the orthonormaliser (CholeskyQR2) is in thin_dev.h.
#include <string.h>

#include "thin_dev.h"

namespace psgd {

// --------------------------------------------------------------------------------------------
// pack: thin fp32 (len x width, ld) -> split-bf16 operand copies, row-major and transposed.
// --------------------------------------------------------------------------------------------
// grid.z walks the roles to pack (role_a, then role_b when two are asked for); which: 1 = row-major copies (what
// the outer-product kernels read), 2 = transposed copies (what the products read), 3 = both
__global__ __launch_bounds__(kThreads) void pack_kernel(const LayerDev* __restrict__ layers,
                                                        const int* __restrict__ ids, int role_a, int role_b,
                                                        int cp, int which) {
    const LayerDev& L = layers[ids[blockIdx.y]];
    const int role = blockIdx.z == 0 ? role_a : role_b;
    const int side = side_of_role(L.transposed, role);
    const int len = side_len(L, side), lenP = side_lenP(L, side);
    const int i0 = blockIdx.x * 64;
    if (i0 >= lenP) return;
    const ThinRef T = L.thin[role];
    extern __shared__ __align__(16) unsigned char smem[];
    float* tile = reinterpret_cast<float*>(smem);      // [64][cp + 1]
    const int tw = cp + 1;
    // eight loads per thread are issued before their LDS stores
    const PSGD_GLOBAL float* src = as_global(T.ptr);
    for (int e0 = 0; e0 < 64 * cp; e0 += 8 * kThreads) {
        float v[8];
#pragma unroll
        for (int d = 0; d < 8; ++d) {
            const int e = e0 + d * kThreads + threadIdx.x;
            const int i = e / cp, c = e % cp;
            v[d] = (e < 64 * cp && i0 + i < len && c < T.width) ? src[(int64_t)(i0 + i) * T.ld + c] : 0.f;
        }
#pragma unroll
        for (int d = 0; d < 8; ++d) {
            const int e = e0 + d * kThreads + threadIdx.x;
            if (e < 64 * cp) tile[(e / cp) * tw + e % cp] = v[d];
        }
    }
    __syncthreads();
    write_packs(L.pack[side], L.planes, tile, tw, cp, i0, 64, lenP, which);
}

// role_b < 0: one role
hipError_t launch_pack(const LayerDev* layers, const int* ids, int n_ids, int max_lenP, int role_a, int role_b,
                       int cp, int which, hipStream_t st) {
    if (n_ids <= 0) return hipSuccess;
    dim3 grid(max_lenP / 64, n_ids, role_b >= 0 ? 2 : 1), block(kThreads);
    const size_t lds = (size_t)64 * (cp + 1) * sizeof(float);
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(pack_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(pack_kernel, grid, block, lds, st, layers, ids, role_a, role_b, cp, which);
    return hipGetLastError();
}

// --------------------------------------------------------------------------------------------
// iterations the next refresh of these layers will run: the largest and the smallest per-layer count.  The host
// fetches them asynchronously, stops launching iterations past the largest (they would find every gate closed) and
// leaves out the second-pass launches of the iterations before the smallest (no layer has its last one there).
// --------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void max_iterations_kernel(const LayerDev* __restrict__ layers, const int* __restrict__ ids,
                                                            int n_ids, int mx, int* __restrict__ out) {
    int k = 1, kmin = 255;
    for (int i = threadIdx.x; i < n_ids; i += 64) {
        const int ki = refresh_iterations(layers[ids[i]], mx);
        k = max(k, ki);
        kmin = min(kmin, ki);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) { k = max(k, __shfl_xor(k, off)); kmin = min(kmin, __shfl_xor(kmin, off)); }
    if (threadIdx.x == 0) out[0] = k | (min(kmin, k) << 16);     // largest count, and the smallest in the high half
}

hipError_t launch_max_iterations(const LayerDev* layers, const int* ids, int n_ids, int mx, int* out, hipStream_t st) {
    if (n_ids <= 0) return hipSuccess;
    hipLaunchKernelGGL(max_iterations_kernel, dim3(1), dim3(64), 0, st, layers, ids, n_ids, mx, out);
    return hipGetLastError();
}

// --------------------------------------------------------------------------------------------
// chol: one workgroup per layer runs the factorisation on the partial Gram matrices that the producing
// kernel has left (used when that kernel cannot hand over to it itself).
// --------------------------------------------------------------------------------------------
// after_finish: the launch follows a split product's finish_kernel, which has factorised every layer itself except
// the wide ones with many Gram slots: those it has only added up in groups (grouped_slot_sum) and left to this
// kernel, which brings 512 threads to the serial part instead of the 256 of a finish workgroup.
template <int NT>
__global__ __launch_bounds__(NT) void chol_kernel(const LayerDev* __restrict__ layers,
                                                  const int* __restrict__ ids, int role, double tol2,
                                                  int pass, int slot_rows, int gate, int a2gate,
                                                  int local_ok, int after_finish) {
    const LayerDev& L = layers[ids[blockIdx.y]];
    if (!gate_open(L, gate)) return;
    if (pass == 2 && L.status[1] == 0) return;
    if (pass == 1 && local_chol(L, role, local_ok)) return;       // the apply kernel factorises for itself
    int stride = after_finish > 1 ? after_finish : 1;     // (> 1: slot_sum_kernel has added the slots up in such groups)
    if (after_finish == 1) {
        const int n_slots = (side_len(L, side_of_role(L.transposed, role)) + slot_rows - 1) / slot_rows;
        if (!grouped_slot_sum(L.thin[role].width, n_slots)) return;
        stride = kSlotGroup;
    }
    extern __shared__ __align__(16) unsigned char smem[];
    chol_body(L, role, tol2, pass, slot_rows, allow2_of(L, a2gate), smem, L.tmat, true, nullptr, stride);
}

// --------------------------------------------------------------------------------------------
// slot sum: the partial Gram matrices of thin[role] added up in groups of `group` consecutive slots, each sum left in
// its group's first slot (fixed order).  For producers that leave many small slots (one per 32 rows): the
// factorisation's one workgroup per layer then adds up one matrix per group.
// --------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void slot_sum_kernel(const LayerDev* __restrict__ layers, const int* __restrict__ ids,
                                                            int role, int slot_rows, int group, int gate) {
    typedef double doublex2 __attribute__((ext_vector_type(2)));
    const LayerDev& L = layers[ids[blockIdx.y]];
    if (!gate_open(L, gate)) return;       // (the slots of a layer whose iteration is over hold what its Ritz step needs)
    const int len = side_len(L, side_of_role(L.transposed, role));
    const int n_slots = (len + slot_rows - 1) / slot_rows;
    const int first = blockIdx.x * group;
    if (first >= n_slots) return;
    const int cnt = min(group, n_slots - first);
    const int w = L.thin[role].width;
    const int ntri = (w * (w + 1)) / 2;
    PSGD_GLOBAL double* g0 = as_global(L.gram) + (int64_t)first * ntri;
    const int t = threadIdx.x;
    if ((ntri & 1) == 0 && (((int64_t)first * ntri) & 1) == 0) {
        for (int e = 2 * t; e < ntri; e += 2 * kThreads) {
            doublex2 x[16];
#pragma unroll
            for (int d = 0; d < 16; ++d)
                x[d] = *reinterpret_cast<const PSGD_GLOBAL doublex2*>(g0 + (int64_t)(d < cnt ? d : 0) * ntri + e);
            doublex2 sacc = x[0];
#pragma unroll
            for (int d = 1; d < 16; ++d) if (d < cnt) sacc += x[d];
            *reinterpret_cast<PSGD_GLOBAL doublex2*>(g0 + e) = sacc;
        }
    } else {
        for (int e = t; e < ntri; e += kThreads) {
            double sacc = g0[e];
            for (int d = 1; d < cnt; ++d) sacc += g0[(int64_t)d * ntri + e];
            g0[e] = sacc;
        }
    }
}

// group <= 16; gate: iteration gate of the refresh (-1: none)
hipError_t launch_slot_sum(const LayerDev* layers, const int* ids, int n_ids, int max_len, int role, int slot_rows,
                           int group, int gate, hipStream_t st) {
    if (n_ids <= 0 || group < 2 || group > 16) return n_ids <= 0 ? hipSuccess : hipErrorInvalidValue;
    const int groups = ((max_len + slot_rows - 1) / slot_rows + group - 1) / group;
    hipLaunchKernelGGL(slot_sum_kernel, dim3(groups, n_ids), dim3(kThreads), 0, st, layers, ids, role, slot_rows, group, gate);
    return hipGetLastError();
}

// Widths that take the blocked factorisation get 512 threads: its panels, trailing updates, the blocked inverse and
// the slot sum are dealt to the waves (1024 threads halve the registers a thread may hold, and measured slower).
hipError_t launch_chol(const LayerDev* layers, const int* ids, int n_ids, int w, int role, double tol2, int pass,
                       int slot_rows, int gate, int a2gate, int local_ok, int after_finish, hipStream_t st) {
    if (n_ids <= 0) return hipSuccess;
    const bool wide = w > 32;
    dim3 grid(1, n_ids), block(wide ? 512 : kThreads);
    const size_t lds = chol_lds_bytes_upto(w);
    auto kfn = wide ? chol_kernel<512> : chol_kernel<kThreads>;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kfn),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kfn, grid, block, lds, st, layers, ids, role, tol2, pass, slot_rows, gate, a2gate,
                       local_ok, after_finish);
    return hipGetLastError();
}

// --------------------------------------------------------------------------------------------
// apply: thin[dst] (len x w_out) <- thin[src] (len x w_in) * tmat[:, :w_out]   (fp64 accumulate);
// w_in and w_out are the widths of the two thin matrices, tmat is w_in x w_in row-major.
// In place (dst == src) is allowed: a workgroup reads its 64 rows completely before writing them.
// Fused follow-ups, chosen by `mode` and the layer's second-pass flag:
//   APPLY_PASS1  (upper-triangular tmat): flag set   -> also the partial Gram matrix of the result, and the
//                                                       last workgroup to finish factorises their sum
//                                         flag clear -> result is final: operand copies if cp > 0
//   APPLY_PASS2  (upper-triangular tmat): flag clear -> nothing to do; else final + operand copies
//   APPLY_RITZ   (full tmat)            : final + operand copies if cp > 0
// --------------------------------------------------------------------------------------------
enum ApplyMode { APPLY_PASS1 = 1, APPLY_PASS2 = 2, APPLY_RITZ = 3 };

// LDS bytes of the tmat block, the x tile and the result tile (what every mode needs), 16-byte rounded
__host__ __device__ inline size_t apply_main_lds(int w_in, int w_out, int cp) {
    const int ow = (cp > w_out ? cp : w_out) + 1;
    const int kpad = (w_in + 3) & ~3;
    const size_t b = (size_t)kGramRows2 * (ow + w_in + 1) * sizeof(float) + (size_t)kpad * 32 * sizeof(double);
    return (b + 15) & ~(size_t)15;
}

// SMALL: the variant for launches whose layers are all narrow (width <= 16) -- it carries the per-workgroup
// factorisation and the hand-over to the second-pass factorisation, which cost registers the plain variant
// (wide blocks, where the kernel is a streaming pass and wants occupancy) does without; there the
// second-pass factorisation is a launch of its own.
template <bool SMALL>
__global__ __launch_bounds__(kThreads) void apply_kernel(const LayerDev* __restrict__ layers,
                                                         const int* __restrict__ ids, int src_role, int dst_role,
                                                         int mode, int cp, int gate, int a2gate, double tol2,
                                                         int which) {
    __shared__ int s_last;
    __shared__ int s_need2;
    const LayerDev& L = layers[ids[blockIdx.y]];
    if (!gate_open(L, gate)) return;
    const int side = side_of_role(L.transposed, src_role);
    const int len = side_len(L, side), lenP = side_lenP(L, side);
    const int i0 = blockIdx.x * kGramRows2;
    if (i0 >= lenP) return;
    const ThinRef X = L.thin[src_role];
    const ThinRef Y = L.thin[dst_role];
    const int w_in = X.width, w_out = Y.width;
    extern __shared__ __align__(16) unsigned char smem[];
    const size_t main_lds = apply_main_lds(w_in, w_out, cp);
    const double* __restrict__ tm = L.tmat;
    int need2;
    // x tile (64 x w_in): one contiguous block of the thin matrix when ld == width (always the case for the
    // library's own buffers and for P, Q), fetched with 16-byte loads over the flat range
    const bool flat_x = X.ld == w_in && (w_in & 3) == 0;
    const int64_t xbase = (int64_t)i0 * X.ld;
    const int n_valid_x = (min(len, i0 + kGramRows2) - i0) * w_in;          // elements that exist
    float4 xpre = make_float4(0.f, 0.f, 0.f, 0.f);
    bool have_pre = false;
    if (SMALL && mode == APPLY_PASS1 && local_chol(L, src_role, 1)) {
        // small factorisation repeated by every workgroup; the first one records the outcome.  The
        // workgroup's own rows are requested first so that their latency overlaps the factorisation.
        if (flat_x) {
            have_pre = true;
            if (4 * (int)threadIdx.x < n_valid_x) xpre = *reinterpret_cast<const float4*>(X.ptr + xbase + 4 * threadIdx.x);
        }
        double* tml = reinterpret_cast<double*>(smem + main_lds);
        chol_body<true>(L, src_role, tol2, 1, kGramRows1, allow2_of(L, a2gate), smem + main_lds + w_in * w_in * sizeof(double),
                  tml, blockIdx.x == 0, &s_need2);
        __syncthreads();
        need2 = s_need2;
        tm = tml;
    } else {
        need2 = L.status[1];
    }
    if (mode == APPLY_PASS2 && !need2) return;
    const bool do_gram = (mode == APPLY_PASS1) && need2;
    const bool do_pack = !do_gram && cp > 0;
    if (i0 >= (do_pack ? lenP : len)) return;
    const bool upper = mode != APPLY_RITZ;
    const int ow = (cp > w_out ? cp : w_out) + 1;     // stride of the output tile (zero padded to cp)
    // The product runs on the fp64 matrix cores (v_mfma_f64_16x16x4_f64): wave v owns rows 16v..16v+15
    // of the 64-row tile and walks the 16-column tiles of the result.  A operand = x (fp32 in LDS,
    // widened per use), B operand = a block of tmat columns staged in LDS.
    const int xs = w_in + 1;                                         // row stride of the x tile
    const int kpad = (w_in + 3) & ~3;                                // reduction length padded to the MFMA k
    const int cbw = 32;                                              // output columns per pass
    double* st = reinterpret_cast<double*>(smem);                    // [kpad][cbw] block of tmat columns
    float* sx = reinterpret_cast<float*>(st + (size_t)kpad * cbw);    // [64][xs]  x tile
    float* so = sx + (size_t)kGramRows2 * xs;                        // [64][ow]  result tile
    const int t = threadIdx.x;
    const int tx = t & 63, ty = t >> 6;
    {
        const float inv_w = 1.0f / (float)w_in;
        if (flat_x) {
            // up to eight 16-byte loads per thread in flight before the first LDS store (w_in <= 128 in one go)
            for (int f0 = 0; f0 < kGramRows2 * w_in; f0 += 32 * kThreads) {
                floatx4 xv[8];
#pragma unroll
                for (int d = 0; d < 8; ++d) {
                    const int f = f0 + 4 * (d * kThreads + t);
                    xv[d] = floatx4{0.f, 0.f, 0.f, 0.f};
                    if (have_pre && f == 4 * t) xv[d] = floatx4{xpre.x, xpre.y, xpre.z, xpre.w};
                    else if (f < n_valid_x) xv[d] = *reinterpret_cast<const PSGD_GLOBAL floatx4*>(as_global(X.ptr) + xbase + f);
                }
#pragma unroll
                for (int d = 0; d < 8; ++d) {
                    const int f = f0 + 4 * (d * kThreads + t);
                    if (f >= kGramRows2 * w_in) continue;
                    int row = (int)(((float)f + 0.5f) * inv_w);
                    int c = f - row * w_in;
                    if (c < 0) { --row; c += w_in; } else if (c >= w_in) { ++row; c -= w_in; }
                    float* dd = sx + row * xs + c;
                    dd[0] = xv[d].x; dd[1] = xv[d].y; dd[2] = xv[d].z; dd[3] = xv[d].w;
                }
            }
        } else {
            for (int i = ty; i < kGramRows2; i += 4) {
                const bool in = i0 + i < len;
                const float* __restrict__ xr = X.ptr + (int64_t)(in ? i0 + i : 0) * X.ld;
                for (int c = tx; c < w_in; c += 64) sx[i * xs + c] = in ? xr[c] : 0.f;
            }
        }
        for (int e = t; e < kGramRows2 * ow; e += kThreads) so[e] = 0.f;
    }
    const int li = tx & 15, lk = tx >> 4;                             // MFMA lane: row/column index, k index
    for (int cb = 0; cb < w_out; cb += cbw) {
        __syncthreads();
        const int jmax = upper ? min(cb + cbw, w_in) : w_in;          // below-diagonal entries of tmat are zero
        const int jpad = (jmax + 3) & ~3;
        // block of tmat -> LDS; eight loads per thread are issued before their LDS stores so that they are
        // in flight together (a load-store-load-store chain costs a round trip to L2 per row)
        for (int e0 = 0; e0 < jpad * cbw; e0 += 8 * kThreads) {
            double tv[8];
#pragma unroll
            for (int d = 0; d < 8; ++d) {
                const int e = e0 + d * kThreads + t;
                const int j = e / cbw, c = e % cbw;             // cbw is a power of two
                tv[d] = (e < jpad * cbw && j < w_in && cb + c < w_in) ? tm[(int64_t)j * w_in + cb + c] : 0.0;
            }
#pragma unroll
            for (int d = 0; d < 8; ++d) {
                const int e = e0 + d * kThreads + t;
                if (e < jpad * cbw) st[e] = tv[d];
            }
        }
        __syncthreads();
        const float* __restrict__ xa = sx + (16 * ty + li) * xs + lk;
        for (int ct = 0; ct < cbw / 16 && cb + 16 * ct < w_out; ++ct) {
            doublex4 acc = {0.0, 0.0, 0.0, 0.0};
            const int kend = upper ? min(jpad, (cb + 16 * ct + 16 + 3) & ~3) : jpad;
            const double* __restrict__ sb = st + lk * cbw + 16 * ct + li;
            for (int k = 0; k < kend; k += 4) {
                const double a = (k + lk < w_in) ? (double)xa[k] : 0.0;
                const double b = sb[k * cbw];
                acc = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, acc, 0, 0, 0);
            }
            const int col = cb + 16 * ct + li;
            if (col < w_out) {
#pragma unroll
                for (int v = 0; v < 4; ++v) so[(16 * ty + 4 * v + lk) * ow + col] = (float)acc[v];
            }
        }
    }
    __syncthreads();
    if (Y.ld == w_out && (w_out & 3) == 0) {
        // contiguous result block: 16-byte stores (rows past the end are cut off)
        const int n_valid = (min(len, i0 + kGramRows2) - i0) * w_out;
        const float inv_w = 1.0f / (float)w_out;
        for (int f = 4 * t; f < n_valid; f += 4 * kThreads) {
            int row = (int)(((float)f + 0.5f) * inv_w);
            int c = f - row * w_out;
            if (c < 0) { --row; c += w_out; } else if (c >= w_out) { ++row; c -= w_out; }
            const float* __restrict__ sr = so + row * ow + c;
            *reinterpret_cast<float4*>(Y.ptr + (int64_t)i0 * Y.ld + f) = make_float4(sr[0], sr[1], sr[2], sr[3]);
        }
    } else {
        for (int i = ty; i < kGramRows2; i += 4) {
            if (i0 + i >= len) break;
            float* __restrict__ yr = Y.ptr + (int64_t)(i0 + i) * Y.ld;
            for (int c = tx; c < w_out; c += 64) yr[c] = so[i * ow + c];
        }
    }
    if (do_gram) {
        gram_tile_f64(so, ow, kGramRows2, w_out, L.gram + (int64_t)blockIdx.x * ((w_out * (w_out + 1)) / 2));
        if (SMALL) {
            const int n_wg = (len + kGramRows2 - 1) / kGramRows2;
            if (last_to_arrive(&L.status[7], n_wg, &s_last)) chol_body<true>(L, dst_role, tol2, 2, kGramRows2, false, smem, L.tmat);
        }
    } else if (do_pack) {
        write_packs(L.pack[side], L.planes, so, ow, cp, i0, kGramRows2, lenP, which & 3, (which & 4) ? L.lzf[side] : nullptr);
    }
}

// --------------------------------------------------------------------------------------------
// The same product for blocks up to 96 wide that are not `small`, as a streaming pass: at these widths the kernel above
// spends its time on latency, not bytes -- a workgroup stages a block of tmat per 32 output columns from L2 behind
// barriers, and its 66 KB of LDS let two workgroups run per compute unit (config 4, 1.58 M rows of width 64: 0.70 ms
// for 1.6 GB of traffic).  Here a workgroup keeps the part of tmat it needs in LDS for its whole life -- per
// 16-column tile of the result only the rows above the diagonal block when tmat is triangular -- and walks over
// many 64-row tiles of its layer; the rows of the next tile are requested before the MFMA phase of the current one.
// --------------------------------------------------------------------------------------------
constexpr int kApplyStreamMaxWidth = 96;
constexpr int kTmStride = 17;        // doubles per row of a 16-column tile of tmat in LDS

__host__ __device__ inline int apply_tm_rows(int ct, int kpad, bool upper) {
    const int k = 16 * (ct + 1);
    return (upper && k < kpad) ? k : kpad;
}
// kp16 > 0: the variant with tmat in registers (reduction length padded to 16 kp16, no tmat in LDS)
__host__ __device__ inline size_t apply_stream_lds(int w_in, int w_out, int cp, bool upper, int kp16) {
    const int kpad = kp16 > 0 ? 16 * kp16 : ((w_in + 3) & ~3), n_ct = (w_out + 15) / 16;
    size_t rows = 0;
    for (int ct = 0; ct < n_ct && kp16 == 0; ++ct) rows += (size_t)apply_tm_rows(ct, kpad, upper);
    const int ow = (cp > 16 * n_ct ? cp : 16 * n_ct) + 1;
    return rows * kTmStride * sizeof(double) + (size_t)kGramRows2 * (kpad + 1 + ow) * sizeof(float);
}

// KP16 > 0: for a triangular tmat of width <= 16 KP16 the wave's fragments of it (tile ct: 4 (ct + 1) steps of the
// reduction) stay in registers for the workgroup's whole life and the MFMA phase reads nothing but them and the rows:
// with the fragments in LDS every MFMA waits on two LDS reads, and the phase ran at a third of the matrix cores' rate.
// KP16 = 0: fragments from LDS (a full tmat, the Ritz step, or widths whose fragments do not fit the registers).
template <int KP16>
__global__ __launch_bounds__(kThreads) void apply_stream_kernel(const LayerDev* __restrict__ layers,
                                                                const int* __restrict__ ids, int src_role, int dst_role,
                                                                int mode, int cp, int gate, int w_out_max, int which) {
    const LayerDev& L = layers[ids[blockIdx.y]];
    if (!gate_open(L, gate)) return;
    const int need2 = L.status[1];
    if (mode == APPLY_PASS2 && !need2) return;
    const bool do_gram = (mode == APPLY_PASS1) && need2;
    const bool do_pack = !do_gram && cp > 0;
    const int side = side_of_role(L.transposed, src_role);
    const int len = side_len(L, side), lenP = side_lenP(L, side);
    const int n_tiles = ((do_pack ? lenP : len) + kGramRows2 - 1) / kGramRows2;
    if ((int)blockIdx.x >= n_tiles) return;
    const ThinRef X = L.thin[src_role];
    const ThinRef Y = L.thin[dst_role];
    const int w_in = X.width, w_out = Y.width;
    const bool upper = mode != APPLY_RITZ;
    const int kpad = KP16 > 0 ? 16 * KP16 : ((w_in + 3) & ~3);
    const int n_ct = (w_out + 15) / 16;
    const int n_ct_max = (w_out_max + 15) / 16;
    const int ow = (cp > 16 * n_ct_max ? cp : 16 * n_ct_max) + 1;    // stride of the result tile (zero padded to cp)
    const int xs = kpad + 1;
    extern __shared__ __align__(16) unsigned char smem[];
    double* tl = reinterpret_cast<double*>(smem);                    // tiles of tmat, tile ct: apply_tm_rows x 17
    int tm_rows_all = 0;
    int tm_rows[kApplyStreamMaxWidth / 16], tm_off[kApplyStreamMaxWidth / 16];     // (uniform)
#pragma unroll
    for (int ct = 0; ct < kApplyStreamMaxWidth / 16; ++ct) {
        tm_rows[ct] = (KP16 == 0 && ct < n_ct) ? apply_tm_rows(ct, kpad, upper) : 0;
        tm_off[ct] = tm_rows_all;
        tm_rows_all += tm_rows[ct];
    }
    float* sx = reinterpret_cast<float*>(tl + (size_t)tm_rows_all * kTmStride);   // [64][xs]  x tile
    float* so = sx + (size_t)kGramRows2 * xs;                                     // [64][ow]  result tile
    const int t = threadIdx.x;
    const int lane = t & 63, wv = t >> 6;
    const int li = lane & 15, lk = lane >> 4;
    // ---- tmat -> LDS (eight loads per thread in flight), zero where the matrix ends
    {
        const double* __restrict__ tm = L.tmat;
        const int tcols = min(w_out, w_in);
        int off = 0;
        for (int ct = 0; ct < n_ct && KP16 == 0; ++ct) {
            const int rows = apply_tm_rows(ct, kpad, upper);
            for (int e0 = 0; e0 < rows * 16; e0 += 8 * kThreads) {
                double tv[8];
#pragma unroll
                for (int d = 0; d < 8; ++d) {
                    const int e = e0 + d * kThreads + t;
                    const int k = e >> 4, c = 16 * ct + (e & 15);
                    tv[d] = (e < rows * 16 && k < w_in && c < tcols) ? tm[(int64_t)k * w_in + c] : 0.0;
                }
#pragma unroll
                for (int d = 0; d < 8; ++d) {
                    const int e = e0 + d * kThreads + t;
                    if (e < rows * 16) tl[(off + (e >> 4)) * kTmStride + (e & 15)] = tv[d];
                }
            }
            off += rows;
        }
        for (int e = t; e < kGramRows2 * ow; e += kThreads) so[e] = 0.f;
    }
    constexpr int NTB = KP16 > 0 ? 2 * KP16 * (KP16 + 1) : 1;
    double tb[NTB];                                              // tile ct, step ks at 2 ct (ct + 1) + ks
    if (KP16 > 0) {
        const double* __restrict__ tm = L.tmat;
        const int tcols = min(w_out, w_in);
#pragma unroll
        for (int ct = 0; ct < KP16; ++ct)
#pragma unroll
            for (int ks = 0; ks < 4 * (ct + 1); ++ks) {
                const int k = 4 * ks + lk, c = 16 * ct + li;
                tb[2 * ct * (ct + 1) + ks] = (k < w_in && c < tcols) ? tm[(int64_t)k * w_in + c] : 0.0;
            }
    }
    // ---- the rows of a tile: one contiguous block of the thin matrix when ld == width, fetched with 16-byte loads
    const bool flat_x = X.ld == w_in && (w_in & 3) == 0;
    const bool flat_y = Y.ld == w_out && (w_out & 3) == 0;
    const float inv_wi = 1.0f / (float)w_in, inv_wo = 1.0f / (float)w_out;
    constexpr int XP = kApplyStreamMaxWidth / 16;          // 16-byte pieces per thread at the widest
    floatx4 xr[XP];
    auto load_x = [&](int tile) {
        const int i0 = tile * kGramRows2;
        const int n_valid = (min(len, i0 + kGramRows2) - i0) * w_in;
        const PSGD_GLOBAL float* xp = as_global(X.ptr) + (int64_t)i0 * X.ld;
#pragma unroll
        for (int d = 0; d < XP; ++d) {
            const int f = 4 * (d * kThreads + t);
            xr[d] = floatx4{0.f, 0.f, 0.f, 0.f};
            if (f < n_valid) xr[d] = *reinterpret_cast<const PSGD_GLOBAL floatx4*>(xp + f);
        }
    };
    int tile = blockIdx.x;
    if (flat_x) load_x(tile);
    for (; tile < n_tiles; tile += gridDim.x) {
        const int i0 = tile * kGramRows2;
        // ---- x tile -> LDS (zero beyond the matrix and in the columns up to the padded reduction length)
        if (flat_x) {
#pragma unroll
            for (int d = 0; d < XP; ++d) {
                const int f = 4 * (d * kThreads + t);
                if (f >= kGramRows2 * w_in) continue;
                int row = (int)(((float)f + 0.5f) * inv_wi);
                int c = f - row * w_in;
                if (c < 0) { --row; c += w_in; } else if (c >= w_in) { ++row; c -= w_in; }
                float* dd = sx + row * xs + c;
                dd[0] = xr[d].x; dd[1] = xr[d].y; dd[2] = xr[d].z; dd[3] = xr[d].w;
            }
            if (kpad > w_in)
                for (int e = t; e < kGramRows2 * (kpad - w_in); e += kThreads)
                    sx[(e / (kpad - w_in)) * xs + w_in + e % (kpad - w_in)] = 0.f;        // (uniform widths: rarely)
        } else {
            for (int i = wv; i < kGramRows2; i += 4) {
                const bool in = i0 + i < len;
                const float* __restrict__ xrow = X.ptr + (int64_t)(in ? i0 + i : 0) * X.ld;
                for (int c = lane; c < kpad; c += 64) sx[i * xs + c] = (in && c < w_in) ? xrow[c] : 0.f;
            }
        }
        __syncthreads();
        if (flat_x && tile + (int)gridDim.x < n_tiles) load_x(tile + gridDim.x);
        // ---- wave v: rows 16 v .. 16 v + 15 of the tile (fp64 matrix cores).  All column tiles advance together along
        // the reduction index: one read of the row operand serves them all, and their accumulators are independent
        // chains (a tile by itself is a chain of dependent MFMAs, each behind two LDS reads).
        if constexpr (KP16 > 0) {
            const float* __restrict__ xa = sx + (16 * wv + li) * xs + lk;
            double a[4 * KP16];
#pragma unroll
            for (int ks = 0; ks < 4 * KP16; ++ks) a[ks] = (double)xa[4 * ks];
            doublex4 acc[KP16];
#pragma unroll
            for (int ct = 0; ct < KP16; ++ct) acc[ct] = doublex4{0.0, 0.0, 0.0, 0.0};
#pragma unroll
            for (int ks = 0; ks < 4 * KP16; ++ks)
#pragma unroll
                for (int ct = ks / 4; ct < KP16; ++ct)
                    acc[ct] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[ks], tb[2 * ct * (ct + 1) + ks], acc[ct], 0, 0, 0);
#pragma unroll
            for (int ct = 0; ct < KP16; ++ct)
                if (ct < n_ct) {
#pragma unroll
                    for (int v = 0; v < 4; ++v) so[(16 * wv + 4 * v + lk) * ow + 16 * ct + li] = (float)acc[ct][v];
                }
        } else {
            const float* __restrict__ xa = sx + (16 * wv + li) * xs + lk;
            const double* __restrict__ sb = tl + lk * kTmStride + li;
            doublex4 acc[kApplyStreamMaxWidth / 16];
#pragma unroll
            for (int ct = 0; ct < kApplyStreamMaxWidth / 16; ++ct) acc[ct] = doublex4{0.0, 0.0, 0.0, 0.0};
#pragma unroll 2
            for (int k = 0; k < kpad; k += 4) {
                const double a = (double)xa[k];
#pragma unroll
                for (int ct = 0; ct < kApplyStreamMaxWidth / 16; ++ct)
                    if (ct < n_ct && k < tm_rows[ct])
                        acc[ct] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, sb[(tm_off[ct] + k) * kTmStride], acc[ct], 0, 0, 0);
            }
#pragma unroll
            for (int ct = 0; ct < kApplyStreamMaxWidth / 16; ++ct)
                if (ct < n_ct) {
#pragma unroll
                    for (int v = 0; v < 4; ++v) so[(16 * wv + 4 * v + lk) * ow + 16 * ct + li] = (float)acc[ct][v];
                }
        }
        __syncthreads();
        // ---- rows of the result
        const int rows_valid = min(len, i0 + kGramRows2) - i0;
        if (flat_y) {
            const int n_valid = rows_valid * w_out;
            PSGD_GLOBAL float* yp = as_global(Y.ptr) + (int64_t)i0 * Y.ld;
            for (int f = 4 * t; f < n_valid; f += 4 * kThreads) {
                int row = (int)(((float)f + 0.5f) * inv_wo);
                int c = f - row * w_out;
                if (c < 0) { --row; c += w_out; } else if (c >= w_out) { ++row; c -= w_out; }
                const float* __restrict__ sr = so + row * ow + c;
                *reinterpret_cast<PSGD_GLOBAL floatx4*>(yp + f) = floatx4{sr[0], sr[1], sr[2], sr[3]};
            }
        } else {
            for (int i = wv; i < rows_valid; i += 4) {
                float* __restrict__ yr = Y.ptr + (int64_t)(i0 + i) * Y.ld;
                for (int c = lane; c < w_out; c += 64) yr[c] = so[i * ow + c];
            }
        }
        if (do_gram) gram_tile_f64(so, ow, kGramRows2, w_out, L.gram + (int64_t)tile * ((w_out * (w_out + 1)) / 2));
        else if (do_pack) write_packs(L.pack[side], L.planes, so, ow, cp, i0, kGramRows2, lenP, which & 3, (which & 4) ? L.lzf[side] : nullptr);
        __syncthreads();
    }
}

// w_in / w_out: upper bounds of the operand widths over the addressed layers (LDS sizing only)
// small: every layer of the launch is narrow (w_in <= 16) and the chain runs the per-workgroup factorisation
// which: operand copies to leave when cp > 0 (1 = row-major, 2 = transposed, 3 = both; + 4: the row-major pieces go to
// the layer's kept copies in fragment order where it has them -- the P~ of a compress step with a deferred residual)
hipError_t launch_apply(const LayerDev* layers, const int* ids, int n_ids, int max_lenP, int w_in, int w_out,
                        int src_role, int dst_role, int mode, int cp, int gate, int a2gate, double tol2,
                        bool small, int which, hipStream_t st) {
    if (n_ids <= 0) return hipSuccess;
    dim3 grid(max_lenP / kGramRows2, n_ids), block(kThreads);
    if (!small && w_in <= kApplyStreamMaxWidth && w_out <= w_in) {
        // a few rounds of workgroups over the whole launch, each walking several tiles of its layer
        // (config 4, width 64: 0.54 ms with one round of 512 workgroups, 0.43 with four, 0.42 with eight, 0.45 with 16)
        int per_layer = (8 * 512 + n_ids - 1) / n_ids;
        if (per_layer > (int)grid.x) per_layer = grid.x;
        if (per_layer < 1) per_layer = 1;
        // (triangular tmat up to width 80: its fragments fit the registers)
        const int kp16 = (mode != APPLY_RITZ && w_in <= 80) ? (w_in + 15) / 16 : 0;
        const size_t lds = apply_stream_lds(w_in, w_out, cp, mode != APPLY_RITZ, kp16);
        // (widths up to 16 are the `small` chain's: kp16 >= 2 here)
        auto kfn = kp16 == 2 ? apply_stream_kernel<2> : kp16 == 3 ? apply_stream_kernel<3>
                 : kp16 == 4 ? apply_stream_kernel<4> : kp16 == 5 ? apply_stream_kernel<5> : apply_stream_kernel<0>;
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kfn),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(kfn, dim3(per_layer, n_ids), block, lds, st, layers, ids, src_role, dst_role,
                           mode, cp, gate, w_out, which);
        return hipGetLastError();
    }
    // w_in / w_out are upper bounds over the layers: sizes that grow with them cover every layer
    size_t lds = apply_main_lds(w_in, w_out, cp);
    if (small && mode == APPLY_PASS1) {
        if (chol_lds_bytes_upto(w_out) > lds) lds = chol_lds_bytes_upto(w_out);          // second-pass factorisation
        const int wl = w_in < kCholRegWidth ? w_in : kCholRegWidth;             // per-workgroup factorisation
        lds += (size_t)wl * wl * sizeof(double) + chol_lds_bytes_upto(wl);
    }
    auto kfn = small ? apply_kernel<true> : apply_kernel<false>;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kfn),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kfn, grid, block, lds, st, layers, ids, src_role, dst_role, mode, cp, gate, a2gate, tol2, which);
    return hipGetLastError();
}

// --------------------------------------------------------------------------------------------
// start block of the subspace iteration: columns [0, n_copy) from thin[src_role] (warm start),
// the others uniform in (-1, 1) from a counter-based hash of (seed, layer, row, column).
// --------------------------------------------------------------------------------------------
__device__ inline uint32_t mix32(uint32_t x) {
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}

__global__ __launch_bounds__(kThreads) void init_block_kernel(const LayerDev* __restrict__ layers,
                                                              const int* __restrict__ ids, int dst_role,
                                                              int src_role, int warm, uint32_t seed) {
    const int lid = ids[blockIdx.y];
    const LayerDev& L = layers[lid];
    const int side = side_of_role(L.transposed, dst_role);
    const int len = side_len(L, side);
    const ThinRef Y = L.thin[dst_role];
    const ThinRef X = L.thin[src_role];
    const int n_copy = warm ? min(X.width, Y.width) : 0;
    const int64_t total = (int64_t)len * Y.width;
    for (int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x; e < total; e += (int64_t)gridDim.x * kThreads) {
        const int i = (int)(e / Y.width), c = (int)(e % Y.width);
        float v;
        if (c < n_copy) {
            v = X.ptr[(int64_t)i * X.ld + c];
        } else {
            uint32_t h = mix32(seed ^ mix32((uint32_t)lid * 0x9e3779b9u + 0x85ebca6bu));
            h = mix32(h ^ mix32((uint32_t)i + 0x632be5abu) ^ mix32((uint32_t)c * 0xc2b2ae35u + 0x27d4eb2fu));
            v = (float)(h >> 8) * (2.0f / 16777216.0f) - 1.0f;
        }
        Y.ptr[(int64_t)i * Y.ld + c] = v;
    }
}

hipError_t launch_init_block(const LayerDev* layers, const int* ids, int n_ids, int max_len, int w, int dst_role,
                             int src_role, int warm, uint32_t seed, hipStream_t st) {
    if (n_ids <= 0) return hipSuccess;
    const int64_t total = (int64_t)max_len * w;
    int gx = (int)((total + kThreads * 4 - 1) / (kThreads * 4));
    if (gx < 1) gx = 1;
    dim3 grid(gx, n_ids), block(kThreads);
    hipLaunchKernelGGL(init_block_kernel, grid, block, 0, st, layers, ids, dst_role, src_role, warm, seed);
    return hipGetLastError();
}

// --------------------------------------------------------------------------------------------
// Rayleigh-Ritz: eigen-decomposition of the w x w Gram matrix H = Y^T Y (Y = M^T Z, Z orthonormal)
// by cyclic two-sided Jacobi in fp64 with a round-robin ordering (w/2 disjoint rotations per round).
// One workgroup per layer.  One copy of each entry of the symmetric H is kept in LDS (layout: sym_idx); in a round the 2 x 2 blocks
// (pair k1 rows) x (pair k2 columns), k1 <= k2, are independent of each other and are rotated in
// place.  The accumulated rotations V live in LDS when they fit, else in the layer's scratch matrix.
// On exit tmat[:, k] is the eigenvector of the k-th largest eigenvalue, so that P~ = Z tmat[:, :r] are
// the leading left singular vectors (Definition 3) and Q = Y tmat[:, :r] = M^T P~.  status gets
// sigma_1 and sigma_r = sqrt(eigenvalue), and the iteration count the next refresh needs.
// --------------------------------------------------------------------------------------------
constexpr int kJacobiMaxSweeps = 30;

// Storage of the symmetric matrix H of even order n in LDS: n rows of S doubles, S the odd one of n / 2 + 1 and
// n / 2 + 2; entry (i, j) lives in row i at column d = (j - i) mod n if d <= n / 2 (for d = n / 2 in the row of the
// smaller index), otherwise it is entry (j, i) of row j.  About as many doubles as a packed triangle.  The lanes
// of a rotation step hold neighbouring rotation pairs at a fixed distance, so the entries they touch together
// move along a diagonal: by +-1 in both indices (address stride S) or by +1 and -1 (stride S - 2).  Both are
// odd, so 32 lanes reading doubles fall on 32 different even banks; the packed triangle's strides vary with the
// row and collide.
__host__ __device__ inline int sym_stride(int n) { return (n / 2 + 1) | 1; }
__device__ inline int sym_idx(int i, int j, int n) {
    int d = j - i;
    d += d < 0 ? n : 0;
    const bool own = 2 * d < n || (2 * d == n && i < j);
    return own ? __mul24(i, sym_stride(n)) + d : __mul24(j, sym_stride(n)) + (n - d);      // (24-bit multiply: full rate)
}

// The round-robin tournament on n players (n even): n / 2 slots, slot k pairs the players at positions 2k ("top")
// and 2k + 1 ("bottom").  Position 0 keeps its player; after every round the others move one place round the ring
// top[1] -> bottom[0] -> bottom[1] -> ... -> bottom[n/2 - 1] -> top[n/2 - 1] -> ... -> top[2] -> top[1].
// In round rd the players (matrix indices) in slot k are
//   top: n - 1 for k = 0, else (rd + k) mod (n - 1);   bottom: (rd - k) mod (n - 1),
// and after n - 1 rounds everybody is back where round 0 had them.
__device__ inline int jacobi_next_pos(int x, int n) {
    const int half = n / 2, k = x >> 1;
    if (x == 0 || n <= 2) return x;
    if ((x & 1) == 0) return k == 1 ? 1 : x - 2;            // top[k] -> top[k - 1], top[1] -> bottom[0]
    return k == half - 1 ? n - 2 : x + 2;                   // bottom[k] -> bottom[k + 1], the last one -> top[half - 1]
}
__device__ inline int jacobi_top(int k, int rd, int n) {
    if (k == 0) return n - 1;
    const int p = rd + k;
    return p >= n - 1 ? p - (n - 1) : p;
}
__device__ inline int jacobi_bottom(int k, int rd, int n) {
    const int q = rd - k;
    return q < 0 ? q + (n - 1) : q;
}
// position in round 0 of matrix index j (inverse of jacobi_top / jacobi_bottom at rd = 0)
__device__ inline int jacobi_pos0(int j, int n) {
    const int half = n / 2;
    if (j == n - 1) return 0;
    if (j == 0) return 1;
    return j < half ? 2 * j : 2 * (n - 1 - j) + 1;
}

// Rotation that annihilates the off-diagonal entry of slot k's 2 x 2 diagonal block (H is stored by position);
// also notes which columns of V the slot holds in round rd.
__device__ inline void jacobi_rotation(const double* a, int n, int rd, int k, double* cs, int* pq) {
    const int half = n / 2;
    const double app = a[sym_idx(2 * k, 2 * k, n)], aqq = a[sym_idx(2 * k + 1, 2 * k + 1, n)];
    const double apq = a[sym_idx(2 * k, 2 * k + 1, n)];
    double c = 1.0, sn = 0.0;
    if (fabs(apq) > 1e-300 && apq * apq > 1e-36 * fabs(app * aqq)) {
        // t = sgn(tau) / (|tau| + sqrt(1 + tau^2)), tau = (aqq - app) / (2 apq), written with one division
        // (square root and quotient from the hardware estimates with Newton steps: this sits on the critical path
        // of every round.  b^2 is a normal number by the test above.)
        const double d = aqq - app, b = 2.0 * apq;
        const double h2 = __builtin_fma(d, d, b * b);
        const double tt = (d >= 0.0 ? b : -b) * rcp_nr(fabs(d) + h2 * rsqrt_nr(h2));
        c = rsqrt_nr(__builtin_fma(tt, tt, 1.0));
        sn = tt * c;
    }
    cs[k] = c; cs[half + k] = sn;
    pq[k] = jacobi_top(k, rd, n); pq[half + k] = jacobi_bottom(k, rd, n);
}

// grid = (slices, layers): every workgroup of a layer repeats the (deterministic) iteration on H and
// accumulates the rotations into its own slice of v_rows rows of V, which is independent of the other rows.
//
// H is stored by POSITION in the tournament, not by matrix index: the 2 x 2 block (slot k1) x (slot k2) sits at
// the same LDS addresses in every round, is rotated by the two slots' rotations, and its four entries are written
// to where the tournament moves their row and column players.  Source and destination addresses of a thread's
// blocks are therefore computed once; a round is: read and rotate (registers) | barrier | write | barrier | the
// next rotations from the diagonal blocks, and V <- V J on the columns the slots hold | barrier.
// V stays indexed by matrix index.
// NBLK: 2 x 2 blocks of H per thread, at least (w/2)(w/2 + 1)/2 over the workgroup's threads.
template <int NBLK>
__global__ __launch_bounds__(1024) void jacobi_kernel(const LayerDev* __restrict__ layers,
                                                      const int* __restrict__ ids, int role, int v_rows,
                                                      float* __restrict__ sigma_out) {
    __shared__ int s_ke;
    __shared__ double s_sum;
    const LayerDev& L = layers[ids[blockIdx.y]];
    const int w = L.thin[role].width;
    const int n_slots = (side_len(L, side_of_role(L.transposed, role)) + kGramRows1 - 1) / kGramRows1;
    const int n = (w + 1) & ~1;      // even size for the round-robin schedule (a zero row/column is added)
    const int half = n / 2;
    const int row0 = blockIdx.x * v_rows;
    const int nv = min(v_rows, n - row0);              // rows of V kept by this workgroup
    extern __shared__ __align__(16) unsigned char smem[];
    double* csb = reinterpret_cast<double*>(smem);     // two buffers of [half] cos, [half] sin
    double* red = csb + 2 * n;                         // [2][16] per-wave partial sums of the convergence test
    double* a = red + 32;                              // H, n rows of sym_stride(n) (see sym_idx)
    double* v = a + n * sym_stride(n);                 // v_rows x n slice of the accumulated rotations
    int* pqb = reinterpret_cast<int*>(v + v_rows * n); // two buffers of [half] top, [half] bottom matrix indices
    const int t = threadIdx.x;
    const int nt = blockDim.x;
    const int txw = nt >= 512 ? 32 : 16, tyw = nt / txw;   // threads as a tyw x txw grid: no integer division
    const int tx = t & (txw - 1), ty = t / txw;
    // H = sum of the partial Gram matrices (upper triangle) left by the last product's epilogue, entry
    // (position x, position y) = H of the matrix indices that round 0 puts there
    const int ntri = (w * (w + 1)) / 2;
    for (int x = ty; x < n; x += tyw) {
        const int k = x >> 1, i = (x & 1) ? jacobi_bottom(k, 0, n) : jacobi_top(k, 0, n);
        for (int y = x + tx; y < n; y += txw) {
            const int ky = y >> 1, j = (y & 1) ? jacobi_bottom(ky, 0, n) : jacobi_top(ky, 0, n);
            double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
            if (i < w && j < w) {
                const double* g = L.gram + tri_idx(min(i, j), max(i, j), w);
                int sp = 0;
                for (; sp + 4 <= n_slots; sp += 4) {
                    s0 += g[(int64_t)sp * ntri]; s1 += g[(int64_t)(sp + 1) * ntri];
                    s2 += g[(int64_t)(sp + 2) * ntri]; s3 += g[(int64_t)(sp + 3) * ntri];
                }
                for (; sp < n_slots; ++sp) s0 += g[(int64_t)sp * ntri];
            }
            a[sym_idx(x, y, n)] = (s0 + s1) + (s2 + s3);
        }
    }
    for (int i = ty; i < nv; i += tyw)
        for (int j = tx; j < n; j += txw) v[i * n + j] = (row0 + i == j) ? 1.0 : 0.0;
    // The unordered pairs {k1, k2} of slots (k1 = k2 included), i.e. the 2 x 2 blocks of H that hold one stored
    // copy each, dealt evenly to the threads once: block e is k1 = e mod half, k2 = k1 + e / half (mod half); the
    // distances e / half = 0 .. half / 2 reach every pair once (the last distance, for even half, only from the
    // lower k1).  Per entry: source address | destination address << 16 (both below 2^16 doubles).
    int bk[NBLK], n_blk = 0;                                   // k1 | k2 << 8
    unsigned adr[NBLK][4];
    {
        const int total = (half * (half + 1)) / 2;
#pragma unroll
        for (int b = 0; b < NBLK; ++b) {
            const int e = t + b * nt;
            bk[b] = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) adr[b][q] = 0;
            if (e < total) {
                const int dk = e / half, k1 = e - dk * half;
                int k2 = k1 + dk;
                k2 -= k2 >= half ? half : 0;
                bk[b] = k1 | (k2 << 8);
                n_blk = b + 1;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    // entry q of the block: row 2 k1 + (q >> 1), column 2 k2 + (q & 1); a diagonal block's entry 2
                    // (bottom, top) is the stored entry 1 again and is left out when the block is written
                    const int x = 2 * k1 + (q >> 1), y = 2 * k2 + (q & 1);
                    adr[b][q] = (unsigned)sym_idx(x, y, n) |
                                ((unsigned)sym_idx(jacobi_next_pos(x, n), jacobi_next_pos(y, n), n) << 16);
                }
            }
        }
    }
    __syncthreads();
    int cur = 0, sweeps = 0;
    for (int sweep = 0; sweep < kJacobiMaxSweeps; ++sweep) {
        // convergence: off-diagonal mass relative to the diagonal.  The per-wave partial sums are added in wave order
        // by every thread for itself: the same bits in every thread and in every workgroup of the layer, whose
        // slices of V only fit together if all of them run the same number of sweeps.
        double off = 0.0, dia = 0.0;
        for (int i = ty; i < n; i += tyw)
            for (int j = i + tx; j < n; j += txw) {
                const double x = a[sym_idx(i, j, n)];
                if (i == j) dia += x * x; else off += 2.0 * x * x;
            }
        for (int o = 32; o > 0; o >>= 1) { off += __shfl_down(off, o); dia += __shfl_down(dia, o); }
        if ((t & 63) == 0) { red[t >> 6] = off; red[16 + (t >> 6)] = dia; }
        __syncthreads();
        double off_all = 0.0, dia_all = 0.0;
        for (int wq = 0; wq < (nt >> 6); ++wq) { off_all += red[wq]; dia_all += red[16 + wq]; }
        const bool done = off_all <= 1e-20 * dia_all;
        if (done) break;
        sweeps = sweep + 1;
        if (t < half) jacobi_rotation(a, n, 0, t, csb + cur * n, pqb + cur * n);
        __syncthreads();
        for (int rd = 0; rd < n - 1; ++rd) {
            const double* cs = csb + cur * n;
            const int* pq = pqb + cur * n;
            // H <- J^T H J on this thread's blocks: rows by slot k1's rotation, columns by slot k2's
            double o[NBLK][4];
#pragma unroll
            for (int b = 0; b < NBLK; ++b) {
                if (b >= n_blk) break;
                const int k1 = bk[b] & 0xff, k2 = bk[b] >> 8;
                const double c1 = cs[k1], s1 = cs[half + k1];
                const double app = a[adr[b][0] & 0xffffu], apq = a[adr[b][1] & 0xffffu];
                const double aqp = a[adr[b][2] & 0xffffu], aqq = a[adr[b][3] & 0xffffu];
                if (k1 == k2) {
                    // (aqp is apq here)
                    o[b][0] = c1 * c1 * app - 2.0 * c1 * s1 * apq + s1 * s1 * aqq;
                    o[b][1] = (c1 * c1 - s1 * s1) * apq + c1 * s1 * (app - aqq);
                    o[b][2] = 0.0;
                    o[b][3] = s1 * s1 * app + 2.0 * c1 * s1 * apq + c1 * c1 * aqq;
                } else {
                    const double c2 = cs[k2], s2 = cs[half + k2];
                    // rows: (top, bottom) <- (c1 top - s1 bottom, s1 top + c1 bottom)
                    const double rpp = c1 * app - s1 * aqp, rpq = c1 * apq - s1 * aqq;
                    const double rqp = s1 * app + c1 * aqp, rqq = s1 * apq + c1 * aqq;
                    // columns: likewise with slot k2's rotation
                    o[b][0] = c2 * rpp - s2 * rpq;
                    o[b][1] = s2 * rpp + c2 * rpq;
                    o[b][2] = c2 * rqp - s2 * rqq;
                    o[b][3] = s2 * rqp + c2 * rqq;
                }
            }
            __syncthreads();
#pragma unroll
            for (int b = 0; b < NBLK; ++b) {
                if (b >= n_blk) break;
                const bool diag = (bk[b] & 0xff) == (bk[b] >> 8);
                a[adr[b][0] >> 16] = o[b][0];
                a[adr[b][1] >> 16] = o[b][1];
                if (!diag) a[adr[b][2] >> 16] = o[b][2];
                a[adr[b][3] >> 16] = o[b][3];
            }
            __syncthreads();
            // the next round's rotations (from the updated H) while the other waves finish V <- V J
            if (rd + 1 < n - 1 && t < half) jacobi_rotation(a, n, rd + 1, t, csb + (cur ^ 1) * n, pqb + (cur ^ 1) * n);
            for (int i = ty; i < nv; i += tyw)
                for (int k = tx; k < half; k += txw) {
                    const int p = pq[k], q = pq[half + k];
                    const double c = cs[k], sn = cs[half + k];
                    const double vx = v[i * n + p], vy = v[i * n + q];
                    v[i * n + p] = c * vx - sn * vy;
                    v[i * n + q] = sn * vx + c * vy;
                }
            __syncthreads();
            cur ^= 1;
        }
    }
    __syncthreads();
    // eigenvalue of matrix index j (= column j of V): the diagonal entry at the position round 0 gives j, where
    // every sweep ends
    double* lam = csb;                                 // [n], the rotation buffers are free now
    for (int j = t; j < n; j += nt) { const int x = jacobi_pos0(j, n); lam[j] = a[sym_idx(x, x, n)]; }
    __syncthreads();
    // sort: rank of eigenvalue j = number of eigenvalues that come before it (ties by index)
    int* rank_of = pqb;
    double* __restrict__ tm = L.tmat;
    for (int j = t; j < w; j += nt) {
        const double lj = lam[j];
        int rank = 0;
        for (int k = 0; k < w; ++k) {
            const double lk = lam[k];
            rank += (lk > lj || (lk == lj && k < j)) ? 1 : 0;
        }
        rank_of[j] = rank;     // 2n entries available
        if (blockIdx.x == 0) L.eval[rank] = lj;
    }
    __syncthreads();
    for (int i = ty; i < nv; i += tyw)
        if (row0 + i < w)
            for (int j = tx; j < w; j += txw) tm[(int64_t)(row0 + i) * w + rank_of[j]] = v[i * n + j];
    if (blockIdx.x != 0) return;
    const int r = L.r;
    // Iterations for a cut without a gap (see refresh_iterations).  Where the count that the subspace needs is out of
    // reach, what is asked of the step is its error (Lemma 2 / Eq. (6): ||M - P~ P~^T M||^2 = sum_{i > r} sigma_i^2
    // at the optimum).  Direction i <= r of the block, still off by sin(theta_i) <= (theta_b / theta_i)^k after k
    // iterations from any start (theta: Ritz values = squared singular value estimates), costs at most
    // sin^2(theta_i) (theta_i - theta_b) on top of the optimum: the directions well above the cut cost nothing after
    // two iterations, the ones in the cluster at the cut have little to lose.  The count is the smallest k for which
    // the sum of these is below 1e-5 of ||M||^2 >= sum of the Ritz values: a tenth of the 1e-4 the step is held to,
    // because the Ritz values are those of the layer's previous refresh and error feedback has flattened the spectrum
    // further since (with 5e-5 the counts came out at 3 to 10 and left 1e-4 to 3e-4).
    // Measured on 7B-shaped bf16 layers (sigma_{b+1} / sigma_r = 0.98): after 3 steps of error feedback 2 iterations
    // leave 3e-6 ||M||^2; after 60 steps, with ||E|| = 0.3 ||M||, 4 leave 1.8e-4, 8 leave 5.8e-5, 16 leave 1.5e-5.
    if (t == 0) s_ke = 255;
    {
        double tr = 0.0;
        for (int j = 0; j < w; ++j) tr += fmax(lam[j], 0.0);
        const double lb = w > r ? L.eval[w - 1] : 0.0, target = 1e-5 * tr;
        for (int k = 2; k <= 64; ++k) {
            if (t == 0) s_sum = 0.0;
            __syncthreads();
            double part = 0.0;
            for (int i = t; i < r; i += nt) {
                const double li = L.eval[i];
                if (lb > 0.0 && li > lb) part += pow(lb / li, 2.0 * k) * (li - lb);
            }
            if (part > 0.0) atomicAdd(&s_sum, part);
            __syncthreads();
            const bool ok = s_sum <= target;          // (the same value in every thread)
            __syncthreads();
            if (ok) {
                if (t == 0) s_ke = k;
                break;
            }
        }
    }
    __syncthreads();
    for (int k = t; k < r; k += nt) {
        const float sg = (float)sqrt(fmax(L.eval[k], 0.0));
        if (sigma_out) sigma_out[k] = sg;
        if (k == 0) L.status[2] = __float_as_int(sg);
        if (k == r - 1) L.status[3] = __float_as_int(sg);
    }
    if (t == 0) {
        // The iteration contracts the error of the leading r-dimensional subspace by about
        // rho = (theta_b / theta_r)^2 per step (theta = Ritz values, the smallest one of the block standing
        // in for sigma_{b+1}); the next refresh of this layer needs as many steps as 1e-5 takes (a tenth of
        // the 1e-4 bar on the subspace), plus one.  (Error feedback drives M towards rho = 1: what is not
        // sent accumulates in E until it is as large as what is.  The launches cap the count, see gate_open.)
        int k_next = 255;
        const double lr = L.eval[r - 1], lb = L.eval[w - 1];
        if (w > r && lr > 0.0 && lb >= 0.0) {
            const double rho = lb / lr;
            if (rho < 0.999) k_next = (rho <= 1e-12) ? 2 : (int)ceil(log(1e-5) / log(rho)) + 1;
        }
        L.status[4] = max(2, min(255, k_next));
        L.status[25] = s_ke;
        L.status[5] = sweeps;
        L.status[24] = min(L.status[24] + 1, 1 << 20);
    }
}

size_t jacobi_lds_bytes(int w, int v_rows) {
    const int n = (w + 1) & ~1;
    return (size_t)(2 * n + 32 + n * sym_stride(n) + v_rows * n) * sizeof(double) + (size_t)2 * n * sizeof(int);
}

hipError_t launch_jacobi(const LayerDev* layers, const int* ids, int n_ids, int w, int role, float* sigma_out,
                         hipStream_t st) {
    if (n_ids <= 0) return hipSuccess;
    const int n = (w + 1) & ~1;
    // rows of V per workgroup: as few as 8 while the chip has idle compute units, and no more than fit in LDS
    int slices = 256 / n_ids;
    slices = slices < 1 ? 1 : slices;
    int v_rows = (n + slices - 1) / slices;
    v_rows = v_rows < 8 ? 8 : v_rows;
    constexpr size_t kLdsCap = 159 * 1024;     // of the 160 KB a workgroup can have
    while (v_rows > 1 && jacobi_lds_bytes(w, v_rows) > kLdsCap) --v_rows;
    if (jacobi_lds_bytes(w, v_rows) > kLdsCap) return hipErrorInvalidValue;
    v_rows = v_rows > n ? n : v_rows;
    const size_t lds = jacobi_lds_bytes(w, v_rows);
    const int n_blocks = ((n / 2) * (n / 2 + 1)) / 2;
    // 256 threads for narrow blocks (the rounds are latency-bound there), else 1024.  (With three to five blocks
    // per thread the kernel spills a few registers; 512 threads with twice the registers measured slower.)
    const int threads = w <= 48 ? 256 : 1024;
    dim3 grid((n + v_rows - 1) / v_rows, n_ids), block(threads);
    const int per_thread = (n_blocks + threads - 1) / threads;
    void (*kfn)(const LayerDev*, const int*, int, int, float*) = nullptr;
    switch (per_thread) {
        case 1: kfn = jacobi_kernel<1>; break;
        case 2: kfn = jacobi_kernel<2>; break;
        case 3: kfn = jacobi_kernel<3>; break;
        case 4: kfn = jacobi_kernel<4>; break;
        case 5: kfn = jacobi_kernel<5>; break;
        default: break;
    }
    if (!kfn) return hipErrorInvalidValue;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kfn),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kfn, grid, block, lds, st, layers, ids, role, v_rows, sigma_out);
    return hipGetLastError();
}

// --------------------------------------------------------------------------------------------
// Host tables (layer descriptors, pointer tables, id lists) reach the workspace as kernel arguments: the runtime
// copies a launch's arguments before the launch call returns, so the host arrays may be rewritten or go out of
// scope at once, nothing depends on how the runtime stages copies from pageable memory, and no copy node ever
// re-reads a host array.  One launch carries kPutBytes bytes.
// --------------------------------------------------------------------------------------------
constexpr int kPutBytes = 2048;
struct PutChunk { uint4 w[kPutBytes / 16]; };

__global__ __launch_bounds__(kPutBytes / 16) void put_kernel(uint4* __restrict__ dst, PutChunk c, int n16) {
    if ((int)threadIdx.x < n16) dst[threadIdx.x] = c.w[threadIdx.x];
}

// dst: device, 16-byte aligned, with room for `bytes` rounded up to 16 (the tail is written as zeros)
hipError_t launch_put(void* dst, const void* src_host, size_t bytes, hipStream_t st) {
    const unsigned char* src = static_cast<const unsigned char*>(src_host);
    unsigned char* d = static_cast<unsigned char*>(dst);
    for (size_t o = 0; o < bytes; o += kPutBytes) {
        const size_t n = bytes - o < (size_t)kPutBytes ? bytes - o : (size_t)kPutBytes;
        PutChunk c;
        memset(&c, 0, sizeof(c));
        memcpy(&c, src + o, n);
        hipLaunchKernelGGL(put_kernel, dim3(1), dim3(kPutBytes / 16), 0, st, reinterpret_cast<uint4*>(d + o), c,
                           (int)((n + 15) / 16));
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// status words of the addressed layers <- 0 (a workspace seen for the first time: "iterations the next refresh
// needs" = unknown, arrival counters at rest)
__global__ __launch_bounds__(64) void clear_status_kernel(const LayerDev* __restrict__ layers, const int* __restrict__ ids) {
    const LayerDev& L = layers[ids[blockIdx.x]];
    if (threadIdx.x < kStatusWords) as_global(L.status)[threadIdx.x] = 0;
}

hipError_t launch_clear_status(const LayerDev* layers, const int* ids, int n_ids, hipStream_t st) {
    if (n_ids <= 0) return hipSuccess;
    hipLaunchKernelGGL(clear_status_kernel, dim3(n_ids), dim3(64), 0, st, layers, ids);
    return hipGetLastError();
}

// plain copy, 16 bytes per thread per iteration (profiler calibration / attainable copy bandwidth)
__global__ __launch_bounds__(kThreads) void copy_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src,
                                                        size_t n_vec) {
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n_vec; i += (size_t)gridDim.x * kThreads)
        dst[i] = src[i];
}

hipError_t launch_copy(void* dst, const void* src, size_t n_bytes, hipStream_t st) {
    const size_t n_vec = n_bytes / 16;
    if (n_vec == 0) return hipSuccess;
    size_t gx = (n_vec + kThreads - 1) / kThreads;
    if (gx > 256 * 64) gx = 256 * 64;
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned)gx), dim3(kThreads), 0, st, reinterpret_cast<uint4*>(dst),
                       reinterpret_cast<const uint4*>(src), n_vec);
    return hipGetLastError();
}

}  // namespace psgd
