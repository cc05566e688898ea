// Device code of the small (w x w) factorisation behind the orthonormaliser, shared by the kernels
// that can run it: the stand-alone chol kernel and, as the last workgroup to arrive, the kernel that
// wrote the partial Gram matrices.
//
// Orthonormalisation (Section 2, "QR decomposition": Q-factor of the economic QR) is CholeskyQR2:
//   G = X^T X (fp64, exact products of the fp32 entries);  G_s = D G D with D = diag(G)^{-1/2};
//   G_s = R_s^T R_s (Cholesky, fp64);  X <- X (D R_s^{-1});  then the same once more on the result.
// The Q-factor it converges to is the one with a positive diagonal of R.  A pivot of the scaled
// Cholesky at step k equals (norm of column k's part orthogonal to the earlier columns / norm of
// column k)^2; if it is <= rank_tol^2 the column is declared dependent and its P~ column is zero.
#pragma once
#include "psgd_dev.h"

namespace psgd {

// The first pass leaves an orthogonality error of about 1e-16/pivot (the smallest pivot of the scaled
// factorisation is about 1/cond^2 of the column-scaled matrix); below kSecondPassPivot the flag
// status[1] is set and the pass-2 code (which exits at once otherwise) does its work.
constexpr double kSecondPassPivot = 1e-6;
constexpr int kCholMaxGroups = 8;
constexpr int kCholRegWidth = 16;      // widths up to this are factorised by one wavefront in registers

// slot groups that sum the partial Gram matrices side by side (all kThreads threads busy for small w)
__host__ __device__ inline int chol_groups(int w) {
    const int ntri = (w * (w + 1)) / 2;
    int g = kThreads / ntri;
    return g < 1 ? 1 : (g > kCholMaxGroups ? kCholMaxGroups : g);
}
// LDS doubles of chol_body besides the blocked inverse's panel, and whether the panel fits as well
__host__ __device__ inline size_t chol_lds_doubles(int w) {
    const int ntri = (w * (w + 1)) / 2;
    const int g = chol_groups(w);
    const int wp = (w + 15) & ~15;
    return (size_t)(g > 1 ? g + 1 : 1) * ntri + 2 * w + wp;
}
__host__ __device__ inline bool chol_blocked_inverse(int w) {
    const int wp = (w + 15) & ~15;
    return w > kCholRegWidth && (chol_lds_doubles(w) + (size_t)wp * 16) * sizeof(double) + (w + 2) * sizeof(int) <= 150 * 1024;
}
// LDS bytes chol_body needs
__host__ __device__ inline size_t chol_lds_bytes(int w) {
    const int wp = (w + 15) & ~15;
    return (chol_lds_doubles(w) + (chol_blocked_inverse(w) ? (size_t)wp * 16 : 0)) * sizeof(double) +
           (size_t)(w + 2) * sizeof(int);
}
// the same for a launch that serves layers of any width up to w (the need is not monotone in w)
inline size_t chol_lds_bytes_upto(int w) {
    size_t b = 0;
    for (int v = 1; v <= w; ++v) b = chol_lds_bytes(v) > b ? chol_lds_bytes(v) : b;
    return b;
}

// squared column norms at or below this count as zero (far below anything fp32 data can produce, and
// keeps the reciprocal square root away from subnormal arguments)
constexpr double kTinyNorm2 = 1e-280;

// 1 / sqrt(x) for finite normal x > 0: hardware estimate refined by two Newton steps (full fp64 accuracy)
__device__ inline double rsqrt_nr(double x) {
    double y = __builtin_amdgcn_rsq(x);
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const double e = __builtin_fma(-(x * y), y, 1.0);
        y = __builtin_fma(0.5 * y, e, y);
    }
    return y;
}

// 1 / x for finite normal x: hardware estimate refined by two Newton steps (full fp64 accuracy)
__device__ inline double rcp_nr(double x) {
    double y = __builtin_amdgcn_rcp(x);
#pragma unroll
    for (int it = 0; it < 2; ++it) y = __builtin_fma(__builtin_fma(-x, y, 1.0), y, y);
    return y;
}

// Ordering point for LDS traffic inside one wavefront (its LDS accesses execute in program order; this
// keeps the compiler from moving them across).
__device__ inline void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Value of v on lane `lane`, the same lane for the whole wavefront (a constant or a uniform value): two scalar
// lane reads instead of the LDS-routed general shuffle, whose latency would sit on the critical path of every
// step of the in-register factorisations below.  All lanes of the wave must be active.
__device__ inline double bcast_lane(double v, int lane) {
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), lane);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), lane);
    return __hiloint2double(hi, lo);
}

// Second-pass permission carried by a launch: -1 always, -2 never, else an iteration gate (kind 2).
__device__ inline bool allow2_of(const LayerDev& L, int a2gate) {
    if (a2gate == -1) return true;
    if (a2gate == -2) return false;
    return gate_open(L, a2gate);
}

// The factorisation for w <= 16 by one wavefront without LDS traffic or barriers: lane j < 16 holds column j
// of the scaled matrix in registers, lane 16 + c holds column c of an identity matrix, and the steps
// exchange values with cross-lane reads.  The row operations of the right-looking Cholesky A = R^T R turn
// the identity columns into R^{-T}, so lane 16 + c ends up with row c of T = R^{-1} and no separate
// inversion is needed.  g: the summed Gram matrix (packed upper triangle, LDS).  Same arithmetic and
// outputs as the general path of chol_body.  W: compiled width (w <= W); rows and columns w .. W-1 are
// those of an identity matrix.
template <int W>
__device__ inline void chol_in_registers_w(const LayerDev& L, const double* g, int w, double tol2, int pass,
                                           bool allow2, double* tm, bool write_status, int* need2_out) {
    const int j = threadIdx.x & 63;
    const bool aug = j >= 16;                          // identity column c = j - 16
    const int c = (j - 16) & 15;
    const int jc = j < w ? j : 0;                      // matrix lanes >= w hold identity columns
    const double djj = g[tri_idx(jc, jc, w)];
    const double dsc_own = djj > kTinyNorm2 ? rsqrt_nr(djj) : 0.0;
    const double dsc_row = __shfl(dsc_own, c < w ? c : 0);    // scaling of row c (used by lane 16 + c)
    // a[i]: entry (i, j) of the scaled matrix, later of R; on lane 16 + c entry (i, c) of R^{-T}
    double a[W];
    int badmask = 0;
#pragma unroll
    for (int i = 0; i < W; ++i) {
        const double dsi = bcast_lane(dsc_own, i < w ? i : 0);
        if (i < w && !(dsi > 0.0)) badmask |= 1 << i;
        double x = (i == (aug ? c : j)) ? 1.0 : 0.0;
        if (!aug && i < w && j < w && i <= j) x = g[tri_idx(i, jc, w)] * dsi * dsc_own;
        a[i] = x;
    }
    double min_piv = 1.0;
    // Written without branches (selects on the wave-uniform `dep`): with branches the compiler copies the whole
    // register array at every merge point, which cost more than the arithmetic.  Rows k >= w are rows of the
    // identity: pivot 1, multipliers 0, nothing changes.  A dependent column (pivot not above tol2) makes row k of
    // R the k-th row of the identity and skips the update (multiplier 0).
#pragma unroll
    for (int k = 0; k < W; ++k) {
        const double piv = bcast_lane(a[k], k);
        const bool dep = ((badmask >> k) & 1) || !(piv > tol2);
        badmask |= dep ? (1 << k) : 0;
        min_piv = (!dep && piv < min_piv) ? piv : min_piv;
        const double rinv = rsqrt_nr(dep ? 1.0 : piv);
        const double ak = dep ? (aug ? a[k] : (j == k ? 1.0 : 0.0)) : a[k] * rinv;   // row k <- row k / R_kk
        a[k] = ak;
        const double mult = dep ? 0.0 : ak;
#pragma unroll
        for (int i = k + 1; i < W; ++i)
            a[i] = __builtin_fma(-bcast_lane(ak, i), mult, a[i]);   // row i <- row i - R[k][i] row k  (on a matrix lane
                                                                    // j < i an entry below the diagonal: never read)
    }
    // lane 16 + c: row c of tmat = D T with the dependent columns zeroed
    if (aug && j < 16 + w) {
#pragma unroll
        for (int i = 0; i < W; ++i)
            if (i < w) tm[(int64_t)c * w + i] = ((badmask >> i) & 1) ? 0.0 : a[i] * dsc_row;
    }
    if (j == 0) {
        const int nbad = __popc(badmask & ((1 << w) - 1));
        const int need2 = (allow2 && min_piv < kSecondPassPivot) ? 1 : 0;
        if (need2_out) *need2_out = need2;
        if (write_status) {
            if (pass == 1) {
                L.status[0] = nbad;
                L.status[1] = need2;
            } else {
                L.status[0] = max(L.status[0], nbad);
            }
        }
    }
}

__device__ inline void chol_in_registers(const LayerDev& L, const double* g, int w, double tol2, int pass,
                                         bool allow2, double* tm, bool write_status, int* need2_out) {
    if (w <= 4) chol_in_registers_w<4>(L, g, w, tol2, pass, allow2, tm, write_status, need2_out);
    else if (w <= 8) chol_in_registers_w<8>(L, g, w, tol2, pass, allow2, tm, write_status, need2_out);
    else if (w <= 12) chol_in_registers_w<12>(L, g, w, tol2, pass, allow2, tm, write_status, need2_out);
    else chol_in_registers_w<16>(L, g, w, tol2, pass, allow2, tm, write_status, need2_out);
}

// Diagonal 16 x 16 block of the blocked factorisation, by one wavefront in registers (same scheme as above):
// factorises the block at rows/columns r0 .. r0 + bw - 1 of the packed triangle `a` (order w), leaves the
// strict upper part of T_JJ = R_JJ^{-1} in its place, 1 / R_kk in rdiag, and updates the dependent-column
// flags and the smallest accepted pivot.  All 64 lanes of the wave call it.
__device__ inline void chol_block16(double* a, int w, int r0, int bw, double tol2, double* rdiag, int* bad,
                                    double& min_piv) {
    constexpr int W = 16;
    const int j = threadIdx.x & 63;
    const bool aug = j >= 16;
    const int c = (j - 16) & 15;
    double x[W];
    int badmask = 0;
#pragma unroll
    for (int i = 0; i < W; ++i) {
        if (i < bw && bad[r0 + i]) badmask |= 1 << i;
        double v = (i == (aug ? c : j)) ? 1.0 : 0.0;
        if (!aug && i <= j && j < bw) v = a[tri_idx(r0 + i, r0 + j, w)];
        x[i] = v;
    }
    // (branch-free for the same reason as above; rows k >= bw are rows of the identity)
#pragma unroll
    for (int k = 0; k < W; ++k) {
        const double piv = bcast_lane(x[k], k);
        const bool dep = ((badmask >> k) & 1) || !(piv > tol2);
        badmask |= dep ? (1 << k) : 0;
        min_piv = (!dep && piv < min_piv) ? piv : min_piv;
        const double rinv = rsqrt_nr(dep ? 1.0 : piv);
        const double xk = dep ? (aug ? x[k] : (j == k ? 1.0 : 0.0)) : x[k] * rinv;
        x[k] = xk;
        const double mult = dep ? 0.0 : xk;
#pragma unroll
        for (int i = k + 1; i < W; ++i) x[i] = __builtin_fma(-bcast_lane(xk, i), mult, x[i]);
    }
    // lane 16 + c holds row c of T_JJ
    if (aug && j < 16 + bw) {
        rdiag[r0 + c] = x[c];
#pragma unroll
        for (int i = 1; i < W; ++i)
            if (i > c && i < bw) a[tri_idx(r0 + c, r0 + i, w)] = x[i];
    }
    if (j < bw) bad[r0 + j] = (badmask >> j) & 1;
}

// Layers whose factorisation is cheap enough for every workgroup of the apply kernel to repeat it for
// itself (one kernel boundary less): register path, and few partial Gram matrices to add up.
constexpr int kLocalCholMaxSlots = 64;
// local_ok: launch-wide permission (all layers of the launch are narrow), the same in every kernel of the chain
__device__ inline bool local_chol(const LayerDev& L, int role, int local_ok) {
    const int len = side_len(L, side_of_role(L.transposed, role));
    return local_ok && L.thin[role].width <= kCholRegWidth &&
           (len + kGramRows1 - 1) / kGramRows1 <= kLocalCholMaxSlots;
}

// Sums the partial Gram matrices of thin[role] (packed upper triangles, slots of `slot_rows` rows, fixed
// order), scales to unit diagonal, Cholesky-factorises (upper, packed in LDS), inverts the factor in
// place and writes tmat = D R_s^{-1}.  pass 1 also decides whether the second CholeskyQR pass runs.
// Called by all threads of one workgroup per layer (256 or 1024: a multiple of 256 and a power of two); smem:
// chol_lds_bytes(w), 8-byte aligned.
// tm: where the w x w factor goes (the layer's tmat, or LDS of the caller); need2_out: optional LDS word
// that receives the second-pass decision; write_status: whether this caller owns the layer's status words.
// NARROW: compiled for widths <= 16 only (the register path; nothing else is generated).
template <bool NARROW = false>
__device__ inline void chol_body(const LayerDev& L, int role, double tol2, int pass, int slot_rows, bool allow2,
                                 unsigned char* smem, double* tm, bool write_status = true,
                                 int* need2_out = nullptr, int slot_stride = 1) {
    const int side = side_of_role(L.transposed, role);
    // slot_stride > 1: the slots were already added up in groups of that many, each sum left in its group's
    // first slot (sum_slot_groups); what remains is one matrix per group
    const int n_slots = (side_len(L, side) + slot_rows * slot_stride - 1) / (slot_rows * slot_stride);
    const int w = L.thin[role].width;
    const int ntri = (w * (w + 1)) / 2;
    const int64_t sstr = (int64_t)slot_stride * ntri;      // distance between the matrices to add
    const int G = chol_groups(w);
    double* a = reinterpret_cast<double*>(smem);          // packed upper triangle
    double* ps = a + ntri;                                // [G][ntri] partial slot sums (G > 1)
    double* dsc = ps + (G > 1 ? G * ntri : 0);            // [w] scaling
    double* rdiag = dsc + w;                              // [w] diagonal of the inverse factor
    double* tcol = rdiag + w;                             // [w up to 16] copy of the column of R being replaced
    const int wp = (w + 15) & ~15;
    const bool blocked = chol_blocked_inverse(w);
    double* panel = tcol + wp;                            // [wp][16] original block column (blocked inverse)
    int* bad = reinterpret_cast<int*>(panel + (blocked ? wp * 16 : 0));    // [w] dependent-column flags
    const int t = threadIdx.x;
    const int nt = blockDim.x, nw = nt >> 6, nty = nt >> 4;      // threads, wavefronts, rows of the 16-wide thread grid
    const double* __restrict__ gram = L.gram;
    if (G > 1 || NARROW) {
        // thread (e, g): entries e of slots g, g + G, ...; sixteen loads in flight, those past the end
        // re-read slot g and do not count
        const int g = t / ntri, e = t - g * ntri;
        if (g < G) {
            double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
            for (int sl = g; sl < n_slots; sl += 16 * G) {
                double x[16];
#pragma unroll
                for (int d = 0; d < 16; ++d) {
                    const int sd = sl + d * G;
                    x[d] = gram[(int64_t)(sd < n_slots ? sd : g) * sstr + e];
                }
#pragma unroll
                for (int d = 0; d < 16; ++d)
                    if (sl + d * G >= n_slots) x[d] = 0.0;
#pragma unroll
                for (int d = 0; d < 16; d += 4) { s0 += x[d]; s1 += x[d + 1]; s2 += x[d + 2]; s3 += x[d + 3]; }
            }
            (G > 1 ? ps + g * ntri : a)[e] = (s0 + s1) + (s2 + s3);
        }
        if (G > 1) {
            __syncthreads();
            if (t < ntri) {
                double s = 0.0;
                for (int g2 = 0; g2 < G; ++g2) s += ps[g2 * ntri + t];
                a[t] = s;
            }
        }
    } else {
        // one workgroup adds up everything: keep many loads in flight (four entries x 16 slots per thread, as
        // 16-byte loads where the slot stride keeps them aligned); the order of the sum is fixed
        typedef double doublex2 __attribute__((ext_vector_type(2)));
        const PSGD_GLOBAL double* gg = as_global(gram);
        if ((ntri & 1) == 0) {
            for (int e = 2 * t; e < ntri; e += 4 * nt) {
                const bool two = e + 2 * nt < ntri;
                const PSGD_GLOBAL double* g0 = gg + e;
                const PSGD_GLOBAL double* g1 = gg + (two ? e + 2 * nt : e);
                doublex2 p0 = {0.0, 0.0}, p1 = p0, p2 = p0, p3 = p0, q0 = p0, q1 = p0, q2 = p0, q3 = p0;
                int sl = 0;
                for (; sl + 16 <= n_slots; sl += 16) {
                    doublex2 x[16], y[16];
#pragma unroll
                    for (int d = 0; d < 16; ++d) {
                        x[d] = *reinterpret_cast<const PSGD_GLOBAL doublex2*>(g0 + (int64_t)(sl + d) * sstr);
                        y[d] = *reinterpret_cast<const PSGD_GLOBAL doublex2*>(g1 + (int64_t)(sl + d) * sstr);
                    }
#pragma unroll
                    for (int d = 0; d < 16; d += 4) {
                        p0 += x[d]; p1 += x[d + 1]; p2 += x[d + 2]; p3 += x[d + 3];
                        q0 += y[d]; q1 += y[d + 1]; q2 += y[d + 2]; q3 += y[d + 3];
                    }
                }
                for (; sl < n_slots; ++sl) {
                    p0 += *reinterpret_cast<const PSGD_GLOBAL doublex2*>(g0 + (int64_t)sl * sstr);
                    q0 += *reinterpret_cast<const PSGD_GLOBAL doublex2*>(g1 + (int64_t)sl * sstr);
                }
                const doublex2 ps2 = (p0 + p1) + (p2 + p3), qs2 = (q0 + q1) + (q2 + q3);
                a[e] = ps2.x; a[e + 1] = ps2.y;
                if (two) { a[e + 2 * nt] = qs2.x; a[e + 2 * nt + 1] = qs2.y; }
            }
        } else {
            for (int e = t; e < ntri; e += nt) {
                const PSGD_GLOBAL double* g0 = gg + e;
                double p0 = 0.0, p1 = 0.0, p2 = 0.0, p3 = 0.0;
                int sl = 0;
                for (; sl + 16 <= n_slots; sl += 16) {
                    double x[16];
#pragma unroll
                    for (int d = 0; d < 16; ++d) x[d] = g0[(int64_t)(sl + d) * sstr];
#pragma unroll
                    for (int d = 0; d < 16; d += 4) { p0 += x[d]; p1 += x[d + 1]; p2 += x[d + 2]; p3 += x[d + 3]; }
                }
                for (; sl < n_slots; ++sl) p0 += g0[(int64_t)sl * sstr];
                a[e] = (p0 + p1) + (p2 + p3);
            }
        }
    }
    __syncthreads();
    if (w <= kCholRegWidth) {
        if (t < 64) chol_in_registers(L, a, w, tol2, pass, allow2, tm, write_status, need2_out);
        return;
    }
    if constexpr (NARROW) return;
    for (int i = t; i < w; i += nt) {
        const double d = a[tri_idx(i, i, w)];
        dsc[i] = d > kTinyNorm2 ? rsqrt_nr(d) : 0.0;
        bad[i] = d > kTinyNorm2 ? 0 : 1;
    }
    __syncthreads();
    // threads as a 16 x 16 grid over (row, column): no integer division in the loops over the triangle
    const int tx = t & 15, ty = t >> 4;
    for (int i = ty; i < w; i += nty) {
        const int base = tri_idx(i, i, w) - i;
        for (int j = i + tx; j < w; j += 16) a[base + j] *= dsc[i] * dsc[j];
    }
    __syncthreads();
    // right-looking Cholesky, A = R^T R, R overwrites the strict upper triangle; 1 / R_kk goes to rdiag
    double min_piv = 1.0;
    const int lane = t & 63, wv = t >> 6, li = lane & 15, lk = lane >> 4;
    if (!blocked) {
        for (int k = 0; k < w; ++k) {
            // every thread reads the pivot itself; the pivot entry is never overwritten, so two barriers
            // per step are enough
            const double piv = a[tri_idx(k, k, w)];
            const bool dep = bad[k] || !(piv > tol2);
            if (!dep && piv < min_piv) min_piv = piv;
            const int kbase = tri_idx(k, k, w) - k;             // a[tri_idx(k, j)] = a[kbase + j]
            if (dep) {
                if (t == 0) { bad[k] = 1; rdiag[k] = 1.0; }
                for (int j = k + 1 + t; j < w; j += nt) a[kbase + j] = 0.0;
            } else {
                const double rinv = rsqrt_nr(piv);
                if (t == 0) rdiag[k] = rinv;
                for (int j = k + 1 + t; j < w; j += nt) a[kbase + j] *= rinv;
            }
            __syncthreads();
            if (!dep) {
                for (int i = k + 1 + ty; i < w; i += nty) {
                    const double rki = a[kbase + i];
                    const int base = tri_idx(i, i, w) - i;
                    for (int j = i + tx; j < w; j += 16) a[base + j] -= rki * a[kbase + j];
                }
            }
            __syncthreads();
        }
    } else {
        // The same in 16 x 16 blocks: per block row J, (1) one wave factorises the diagonal block and
        // inverts its factor (needed below and by the inverse of R), (2) R_JK = T_JJ^T A_JK for K > J and
        // (3) A_IK -= R_JI^T R_JK for J < I <= K run on the fp64 matrix cores, blocks dealt to the waves.
        const int nbk = wp / 16;
        for (int J = 0; J < nbk; ++J) {
            const int r0 = 16 * J;
            const int bw = min(16, w - r0);
            if (t < 64) chol_block16(a, w, r0, bw, tol2, rdiag, bad, min_piv);
            __syncthreads();
            // (2) row panel; rows of dependent columns are zero.  (Block J is complete: K > J exists.)
            for (int K = J + 1 + wv; K < nbk; K += nw) {
                doublex4 d = {0.0, 0.0, 0.0, 0.0};
                const int col = 16 * K + li;
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const int kk = r0 + 4 * c + lk, ii = r0 + li;
                    const double av = kk < ii ? a[tri_idx(kk, ii, w)] : (kk == ii ? rdiag[ii] : 0.0);   // T_JJ[kk][ii]
                    const double bv = col < w ? a[tri_idx(kk, col, w)] : 0.0;                           // A_JK[kk][col]
                    d = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bv, d, 0, 0, 0);
                }
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int row = r0 + 4 * v + lk;
                    if (col < w) a[tri_idx(row, col, w)] = bad[row] ? 0.0 : d[v];
                }
            }
            __syncthreads();
            // (3) trailing update
            int pair = 0;
            for (int I = J + 1; I < nbk; ++I)
                for (int K = I; K < nbk; ++K, ++pair) {
                    if ((pair & (nw - 1)) != wv) continue;
                    doublex4 acc = {0.0, 0.0, 0.0, 0.0};
                    const int ci = 16 * I + li, ck = 16 * K + li;
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const int kk = r0 + 4 * c + lk;
                        const double av = ci < w ? a[tri_idx(kk, ci, w)] : 0.0;     // R_JI[kk][ci]
                        const double bv = ck < w ? a[tri_idx(kk, ck, w)] : 0.0;     // R_JK[kk][ck]
                        acc = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bv, acc, 0, 0, 0);
                    }
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int row = 16 * I + 4 * v + lk;
                        if (row <= ck && ck < w) a[tri_idx(row, ck, w)] -= acc[v];
                    }
                }
            __syncthreads();
        }
    }
    // inverse T of the upper-triangular factor, in place in the packed triangle (T_jj = 1 / R_jj is in rdiag):
    //   T_ij = -T_jj * sum_{l=i}^{j-1} T_il R_lj   (i < j; T_il already in place)
    if (!blocked) {
        // column by column, one thread per row i of the new column
        for (int j = 1; j < w; ++j) {
            for (int i = t; i < j; i += nt) tcol[i] = a[tri_idx(i, j, w)];
            __syncthreads();
            const double tjj = rdiag[j];
            for (int i = t; i < j; i += nt) {
                const int base = tri_idx(i, i, w) - i;
                double sacc = rdiag[i] * tcol[i];
                for (int l = i + 1; l < j; ++l) sacc += a[base + l] * tcol[l];
                a[base + j] = -tjj * sacc;
            }
            __syncthreads();
        }
    } else {
        // 16 x 16 blocks; the diagonal blocks of T were left by the factorisation,
        const int nbk = wp / 16;
        // then block column after block column, T_IJ = -(sum_{K=I}^{J-1} T_IK R_KJ) T_JJ on the fp64 matrix
        // cores, the block rows I dealt to the waves.  The products are formed transposed,
        // U^T = sum_K R_KJ^T T_IK^T and T_IJ^T = -T_JJ^T U^T, so that the accumulator of the first is the
        // B operand of the second without a move.  R_KJ is read from a copy of the block column, T in place.
        for (int J = 1; J < nbk; ++J) {
            for (int e = t; e < 16 * J * 16; e += nt) {
                const int row = e >> 4, col = 16 * J + (e & 15);
                panel[e] = col < w ? a[tri_idx(row, col, w)] : 0.0;
            }
            __syncthreads();
            for (int I = wv; I < J; I += nw) {
                doublex4 acc = {0.0, 0.0, 0.0, 0.0};
                const int trow = 16 * I + li;
                const int tbase = tri_idx(trow, trow, w) - trow;               // a[tbase + c] = T[trow][c], c > trow
                for (int K = I; K < J; ++K)
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const int kk = 16 * K + 4 * c + lk;                     // < 16 J <= w
                        const double av = panel[kk * 16 + li];                  // R[kk][16 J + li]
                        const double bv = trow < kk ? a[tbase + kk] : (trow == kk ? rdiag[trow] : 0.0);   // T[trow][kk]
                        acc = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bv, acc, 0, 0, 0);
                    }
                doublex4 d2 = {0.0, 0.0, 0.0, 0.0};
                const int jcol = 16 * J + li;
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const int jrow = 16 * J + 4 * c + lk;
                    double av = 0.0;                                            // T_JJ[jrow][jcol]
                    if (jcol < w) av = jrow < jcol ? a[tri_idx(jrow, jcol, w)] : (jrow == jcol ? rdiag[jrow] : 0.0);
                    d2 = __builtin_amdgcn_mfma_f64_16x16x4f64(av, acc[c], d2, 0, 0, 0);
                }
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int col = 16 * J + 4 * v + lk;
                    if (col < w) a[tbase + col] = -d2[v];                       // T[trow][col]
                }
            }
            __syncthreads();
        }
    }
    for (int i = ty; i < w; i += nty) {
        const int base = tri_idx(i, i, w) - i;
        for (int j = tx; j < w; j += 16) {
            double v = 0.0;
            if (!bad[j]) v = (i < j) ? a[base + j] : (i == j ? rdiag[i] : 0.0);
            tm[(int64_t)i * w + j] = v * dsc[i];
        }
    }
    if (t == 0) {
        int nbad = 0;
        for (int i = 0; i < w; ++i) nbad += bad[i];
        const int need2 = (allow2 && min_piv < kSecondPassPivot) ? 1 : 0;
        if (need2_out) *need2_out = need2;
        if (write_status) {
            if (pass == 1) {
                L.status[0] = nbad;
                L.status[1] = need2;
            } else {
                L.status[0] = max(L.status[0], nbad);
            }
        }
    }
}

// True in exactly one workgroup of the `n_wg` that call it for a layer: the one that arrives last, after
// which everything the others wrote before their call is visible to it.  `counter` starts at zero and is
// zero again afterwards.  All threads of the workgroup must call it; flag points to an int in LDS.
__device__ inline bool last_to_arrive(int* counter, int n_wg, int* flag) {
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) {
        const int old = atomicAdd(counter, 1);
        *flag = (old == n_wg - 1) ? 1 : 0;
    }
    __syncthreads();
    const bool last = *flag != 0;
    if (last) {
        __threadfence();
        if (threadIdx.x == 0) *counter = 0;
    }
    return last;
}

// Partial Gram matrices added up in two levels, so that no workgroup has to read all of them: the slots form
// groups of kSlotGroup; the workgroup that completes a group adds the group's slots into the first one (fixed
// order), and the one that completes the last group goes on with one matrix per group.  Used where one
// workgroup per slot runs anyway and the matrices are large (width above the register path, many slots).
constexpr int kSlotGroup = 8;
constexpr int kMaxSlotGroups = 16;      // arrival counters per layer
__device__ inline bool grouped_slot_sum(int w, int n_slots) {
    return w > kCholRegWidth && n_slots >= 2 * kSlotGroup && n_slots <= kSlotGroup * kMaxSlotGroups;
}
// Called by all threads of the workgroup that completed group `grp`: slot first <- sum of the group's slots.
__device__ inline void sum_slot_group(double* gram, int w, int n_slots, int grp) {
    typedef double doublex2 __attribute__((ext_vector_type(2)));
    const int ntri = (w * (w + 1)) / 2;
    const int first = grp * kSlotGroup;
    const int cnt = min(kSlotGroup, n_slots - first);
    PSGD_GLOBAL double* g0 = as_global(gram) + (int64_t)first * ntri;
    const int t = threadIdx.x, nt = blockDim.x;
    if ((ntri & 1) == 0 && cnt == kSlotGroup) {
        // two 16-byte entries x 8 slots in flight per thread
        for (int e = 2 * t; e < ntri; e += 4 * nt) {
            const bool two = e + 2 * nt < ntri;
            const int e2 = two ? e + 2 * nt : e;
            doublex2 x[kSlotGroup], y[kSlotGroup];
#pragma unroll
            for (int d = 0; d < kSlotGroup; ++d) {
                x[d] = *reinterpret_cast<const PSGD_GLOBAL doublex2*>(g0 + (int64_t)d * ntri + e);
                y[d] = *reinterpret_cast<const PSGD_GLOBAL doublex2*>(g0 + (int64_t)d * ntri + e2);
            }
            doublex2 sx = x[0], sy = y[0];
#pragma unroll
            for (int d = 1; d < kSlotGroup; ++d) { sx += x[d]; sy += y[d]; }
            *reinterpret_cast<PSGD_GLOBAL doublex2*>(g0 + e) = sx;
            if (two) *reinterpret_cast<PSGD_GLOBAL doublex2*>(g0 + e2) = sy;
        }
    } else {
        for (int e = t; e < ntri; e += nt) {
            double sacc = g0[e];
            for (int d = 1; d < cnt; ++d) sacc += g0[(int64_t)d * ntri + e];
            g0[e] = sacc;
        }
    }
}

}  // namespace psgd
