// Device-side data structures shared by the kernels of the PowerSGD+ compressor library.
//
// Vocabulary.  A layer is stored as S (rows x cols, row-major, leading dimension ld).  Thin
// matrices attached to the row dimension are "L-side" (rows x w), those attached to the column
// dimension are "W-side" (cols x w).  With the paper's convention m >= n (Section 1), P~ (m x r) is
// L-side and Q (n x r) is W-side when rows >= cols, and the other way round when the stored buffer
// is the transpose of the logical matrix.  Kernels work on sides; the host maps the paper's P and Q
// onto them through "roles".
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace psgd {

typedef __bf16 bf16_t;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));
typedef unsigned int uintx2 __attribute__((ext_vector_type(2)));

// Pointers read from a layer descriptor are generic to the compiler, which then emits flat memory
// instructions (tied to the LDS counter as well); the kernels cast them to the global address space.
#define PSGD_GLOBAL __attribute__((address_space(1)))
template <class T> __device__ inline PSGD_GLOBAL T* as_global(T* p) { return (PSGD_GLOBAL T*)p; }

// Streaming accesses.  An m x n buffer that a pass touches once and the next kernel does not read again
// (the gradients, E_t coming in, M read for the last time by the residual, E_{t+1} and the reconstruction
// going out, the optimizer state) carries the non-temporal hint: measured on this machine a read-only stream
// goes from 6.3 to 7.1 TB/s with it and a copy from 5.5 to 6.0.  M written by the first pass and read by the
// second does not: for a matrix that fits the memory-side cache the plain accesses are the faster ones there.
// One bit per stream; the mask is a compile-time constant so that a variant can be built for measurement.
#ifndef PSGD_NT_MASK
#define PSGD_NT_MASK 0x1f3
#endif
enum Stream { NT_G = 1, NT_E_IN = 2, NT_M_OUT = 4, NT_S_PROD = 8, NT_M_RES = 16, NT_E_OUT = 32, NT_DEC = 64,
              NT_OPT_IN = 128, NT_OPT_OUT = 256 };
template <int BIT, class V> __device__ inline V ld_stream(const PSGD_GLOBAL V* p) {
    if constexpr ((PSGD_NT_MASK & BIT) != 0) return __builtin_nontemporal_load(p); else return *p;
}
template <int BIT, class V> __device__ inline void st_stream(PSGD_GLOBAL V* p, V v) {
    if constexpr ((PSGD_NT_MASK & BIT) != 0) __builtin_nontemporal_store(v, p); else *p = v;
}

constexpr int kStatusWords = 8 + 16 + 8; // per layer: 8 diagnostics and counters, one counter per Gram slot group,
                                         // then: [24] refreshes this layer has run in this workspace, [25] iterations
                                         // its next refresh runs if its cut has no gap (see refresh_iterations)
constexpr int kThreads = 256;      // 4 wavefronts of 64 lanes
constexpr int kLenPad = 128;       // packed operand rows are padded (with zeros) to this multiple
constexpr int kGramRows1 = 128;    // rows per partial Gram matrix written by a product's epilogue
constexpr int kGramRows2 = 64;     // rows per partial Gram matrix written by the apply kernel

enum Side { SIDE_L = 0, SIDE_W = 1 };
// Roles: the paper's P~ and Q (user buffers, leading dimension r) and the two wide internal
// blocks of the subspace iteration (leading dimension wz).
// what a product's epilogue does besides storing the thin result
enum Epilogue { EPI_NONE = 0, EPI_GRAM = 1, EPI_PACK = 2, EPI_KIND_MASK = 3,
                EPI_KEEP_E = 16,     // flag: a FORM pass uses M but leaves E in place (M is formed again later)
                EPI_KEPT = 32 };     // flag: EPI_PACK writes the kept copies (fragment order) in place of the row-major ones
enum Role { ROLE_P = 0, ROLE_Q = 1, ROLE_ZP = 2, ROLE_ZQ = 3, ROLE_COUNT = 4 };

struct ThinRef {
    float* ptr;   // len x width, row-major
    int ld;
    int width;
};

// Split-bf16 operand copies of one thin matrix X (len x width), zero padded to lenP x cp.
// X is written as a sum of `planes` bf16 numbers, plane 0 the rounded value and each further plane
// the rounded remainder: two planes carry 16 mantissa bits (|error| <= 2^-17 |x|), three carry 24.
//   n[k] : [lenP][cp]   row-major      (A/B operand of the rank-r outer product)
//   t[k] : the B operand of the tall-skinny products (reduction over len) in the register layout of
//          v_mfma_f32_32x32x16_bf16: [lenP / 16][cp / 32][64 lanes][8], lane li + 32 lg of block (k16, nb) holding
//          X[16 k16 + 8 lg .. + 7][32 nb + li].  One MFMA B fragment of a wavefront is 1 KB of consecutive memory,
//          so a kernel can load it straight into registers, and a 64-row chunk of all columns is one run of 4 cp bytes.
constexpr int kMaxPlanes = 3;
// Fragment order of a row-major thin matrix X (len x cp) as the A or B operand of an outer product (reduction over
// the cp columns): [len / 32][cp / 16][64 lanes][8], lane li + 32 lg of fragment (row block, k-step) holding
// X[32 block + li][16 kstep + 8 lg .. + 7].  Offset of the 16-byte piece (row, 8-column group g8):
__host__ __device__ inline int64_t frag_piece(int row, int g8, int cp) {
    return ((int64_t)(row >> 5) * (cp >> 4) + (g8 >> 1)) * 64 + (row & 31) + 32 * (g8 & 1);
}
__host__ __device__ inline int64_t pack_t_offset(int k, int c, int cp) {
    return ((((int64_t)(k >> 4) * (cp >> 5) + (c >> 5)) * 64 + (c & 31) + 32 * ((k >> 3) & 1)) << 3) + (k & 7);
}
struct PackRef {
    bf16_t* n[kMaxPlanes];
    bf16_t* t[kMaxPlanes];
};

struct LayerDev {
    int rows, cols;
    int64_t ld;
    int r;             // rank of the compressor
    int wz;            // block width of the subspace iteration (multiple of 32, >= r)
    int gdt;           // PSGD_F32 / PSGD_BF16
    int n_workers;
    int transposed;    // rows < cols: P~ is W-side
    int planes;        // 2 or 3 bf16 planes per fp32 operand (3 or 6 MFMA products per term)
    int rowsP, colsP;  // rows / cols rounded up to kLenPad
    int split_row;     // k-splits of the row-mode product  (reduction over cols)
    int split_col;     // k-splits of the column-mode product (reduction over rows)
    int split_row_f;   // the same for the forming passes, which want about twice as many workgroups
    int split_col_f;
    int split_row_v2;  // k-splits of the row-mode forming pass on 32 x 256 tiles (form_row_kernel)
    int split_col_v2;  // k-splits of the column-mode product on 32 x 256 tiles (col_prod_kernel)
    int pad_[2];
    const void* const* G;   // n_workers device pointers
    float* S;               // E on entry, M between the sweeps, E_{t+1} on exit
    ThinRef thin[ROLE_COUNT];
    float* part[2];         // per side: [split][width][lenP] fp32 partial products of a split reduction
    PackRef pack[2];        // per side
    bf16_t* lzf[2][kMaxPlanes];  // per side: copies of the compress step's P~ and Q operands in MFMA fragment order
                                 // (frag_piece), kept while the residual of that step is still owed (deferred residual)
    double* gram;           // [slots][w(w+1)/2] partial Gram matrices (packed upper triangles), one slot per
                            // row block of the producer
    double* tmat;           // [wmax*wmax] small factor applied from the right
    double* eval;           // [wmax]
    int* status;            // [kStatusWords] : rank_deficient, second-pass-needed flag, sigma_max bits, sigma_r bits,
                            //       iterations the next refresh needs (0 = not known yet), Jacobi sweeps of the last
                            //       refresh, arrival counters of the two kernels that hand over to the
                            //       factorisation, then the arrival counters of the Gram slot groups
};

__host__ __device__ inline int side_of_role(int transposed, int role) {
    // P-like roles live on the long side (m): L-side unless the storage is transposed.
    const int p_like = (role == ROLE_P || role == ROLE_ZP);
    return (p_like != (transposed != 0)) ? SIDE_L : SIDE_W;
}

// x = p[0] + p[1] (+ p[2]) with every p a bf16; the remainder after the last plane is dropped.
template <int PL>
__device__ inline void split_planes(float x, bf16_t (&p)[PL]) {
    float rem = x;
#pragma unroll
    for (int k = 0; k < PL; ++k) {
        p[k] = (bf16_t)rem;
        rem -= (float)p[k];
    }
}

// v / d and v % d for the small divisors that occur as cp/32, cp/8 or nrows/8 (1..6; 4..24 in steps of 4): constant
// divisors compile to a multiply and a shift instead of the long generic division sequence.
__device__ inline void divmod_small(int v, int d, int& q, int& r) {
    switch (d) {
        case 1: q = v; break;
        case 2: q = v / 2; break;
        case 3: q = v / 3; break;
        case 5: q = v / 5; break;
        case 6: q = v / 6; break;
        case 4: q = v / 4; break;
        case 8: q = v / 8; break;
        case 12: q = v / 12; break;
        case 16: q = v / 16; break;
        case 20: q = v / 20; break;
        case 24: q = v / 24; break;
        default: q = v / d; break;
    }
    r = v - q * d;
}

// Operand copies of `nrows` finished rows held as an fp32 LDS tile [nrows][tw] (columns >= cp unused,
// nrows and row0 multiples of 16); global rows row0 .. row0 + nrows - 1.  All threads of the workgroup take part.
// which: 1 = the row-major copies only, 2 = the transposed ones only, 3 = both.
// kept: the layer's lzf[side] where the result is a factor of a compress step whose residual is deferred: the pieces of
// the row-major copies then go there instead, in fragment order (frag_piece), for the layers that have such copies.
// PLT: the plane count as a compile-time constant where the caller has it (0: from `planes`, all kMaxPlanes are formed)
template <int PLT = 0>
__device__ inline void write_packs(const PackRef& K, int planes, const float* tile, int tw, int cp, int row0,
                                   int nrows, int lenP, int which = 3, bf16_t* const* kept = nullptr) {
    constexpr int NPL = PLT > 0 ? PLT : kMaxPlanes;
    const int t = threadIdx.x;
    const bool to_kept = kept && kept[0];
    // (the destinations are read before the first store: after one, the compiler would read them again)
    PSGD_GLOBAL bf16_t* dn[NPL];
    PSGD_GLOBAL bf16_t* dt[NPL];
#pragma unroll
    for (int k = 0; k < NPL; ++k) {
        dn[k] = k < planes ? as_global(to_kept ? kept[k] : K.n[k]) : nullptr;
        dt[k] = k < planes ? as_global(K.t[k]) : nullptr;
    }
    for (int v = t; (which & 1) && v < nrows * (cp / 8); v += kThreads) {
        int row, g8;
        if (to_kept) {
            // along the destination: piece v of the tile's run of whole fragments (row0, nrows: multiples of 32)
            int blk, ks;
            divmod_small(v >> 6, cp >> 4, blk, ks);
            row = 32 * blk + (v & 31);
            g8 = 2 * ks + ((v >> 5) & 1);
        } else {
            divmod_small(v, cp / 8, row, g8);
        }
        const int c0 = 8 * g8;
        bf16x8 o[NPL];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            bf16_t q[NPL];
            split_planes<NPL>(tile[row * tw + c0 + u], q);
#pragma unroll
            for (int k = 0; k < NPL; ++k) o[k][u] = q[k];
        }
        const int64_t off = to_kept ? frag_piece(row0 + row, g8, cp) * 8 : (int64_t)(row0 + row) * cp + c0;
#pragma unroll
        for (int k = 0; k < NPL; ++k)
            if (k < planes) *reinterpret_cast<PSGD_GLOBAL bf16x8*>(dn[k] + off) = o[k];
    }
    // fragment-order copy: the tile's rows are (nrows / 16) * (cp / 32) whole fragments, one run of consecutive memory
    // per plane; thread v writes the v-th 16-byte piece of that run (row0 and nrows are multiples of 16)
    for (int v = t; (which & 2) && v < cp * (nrows / 8); v += kThreads) {
        const int ln = v & 63, frag = v >> 6;
        int k16, nb;
        divmod_small(frag, cp >> 5, k16, nb);
        const int c = 32 * nb + (ln & 31), ib = 16 * k16 + 8 * (ln >> 5);
        bf16x8 o[NPL];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            bf16_t q[NPL];
            split_planes<NPL>(tile[(ib + u) * tw + c], q);
#pragma unroll
            for (int k = 0; k < NPL; ++k) o[k][u] = q[k];
        }
        const int64_t off = pack_t_offset(row0 + ib, c, cp);      // (= 8 * (first piece of the tile + v))
#pragma unroll
        for (int k = 0; k < NPL; ++k)
            if (k < planes) *reinterpret_cast<PSGD_GLOBAL bf16x8*>(dt[k] + off) = o[k];
    }
}

// Launches inside the subspace iteration carry a gate (-1 outside it), see make_gate: the iteration the launch
// belongs to, its kind, the iteration budget and the number of iterations the host launches this time.
// A layer runs k iterations: the whole budget in its first two refreshes (the first knows nothing; the second is the
// first to meet the error-feedback state, whose spectrum is flatter at the cut than that of the first step's plain
// gradient: on a 4096 x 4096 run sigma_{b+1}/sigma_r went from 0.13 at t = 0 to 0.43 at t = 10, and the count taken
// from t = 0 left sin(theta) = 2e-4); after that status[4] (what
// its spectrum needs to converge, from the Ritz values of its last refresh) when that is within the budget; and
// otherwise -- the cut is then too close to a cluster of singular values to converge across in the budget, and the
// members of such a cluster compress almost equally well -- the count that keeps the compression error within a
// tenth of 1e-4 ||M||^2 of the optimum (status[25]), at least 2, at most the budget.  k never exceeds the number of launched iterations (the host may launch fewer than the budget when
// it knows an upper bound of the counts; should that bound be out of date, a layer's last iteration is still one
// that was launched).  kind 1 marks the orthonormalisation of Y, which the last executed iteration skips because
// the Rayleigh-Ritz step wants Y = M^T Z itself; kind 2 is open in the last executed iteration only (the second
// CholeskyQR pass on Z, which the Rayleigh-Ritz step needs exact).
constexpr int kMaxRefreshIterations = 255;
__host__ __device__ inline int make_gate(int iteration, int kind, int budget, int launched) {
    return iteration | kind << 8 | budget << 10 | launched << 18;
}
__host__ __device__ inline int gate_with_kind(int gate, int kind) { return (gate & ~(3 << 8)) | kind << 8; }
// iterations the layer's next refresh runs when the budget is mx
__device__ inline int refresh_iterations(const LayerDev& L, int mx) {
    int k = L.status[4];
    if (k <= 0 || L.status[24] < 2) k = mx;
    else if (k > mx) {
        // no gap to converge across within the budget: as many iterations as the error bound of Lemma 2 needs
        // (status[25], see jacobi_kernel), at least 2, at most the budget
        const int ke = L.status[25] < 2 ? 2 : L.status[25];
        k = mx < ke ? mx : ke;
    }
    return k;
}
__device__ inline bool gate_open(const LayerDev& L, int gate) {
    if (gate < 0) return true;
    const int it = gate & 0xff, kind = (gate >> 8) & 3, mx = (gate >> 10) & 0xff, launched = (gate >> 18) & 0xff;
    int k = refresh_iterations(L, mx);
    k = k < launched ? k : launched;
    if (kind == 2) return it == k - 1;
    return it < k - kind;
}

typedef __attribute__((__vector_size__(4 * sizeof(double)))) double doublex4;

// index of (i, j), i <= j, in a packed upper triangle of order w stored row by row
__host__ __device__ inline int tri_idx(int i, int j, int w) { return i * w - (i * (i - 1)) / 2 + (j - i); }

// Partial Gram matrix of a tile of finished rows on the fp64 matrix cores:
//   g[tri_idx(i, j, w)] = sum_rows tile[row][i] * tile[row][j]   for i <= j < w   (packed upper triangle)
// tile is fp32 in LDS, [nrows][tw], nrows a multiple of 4, columns up to the next multiple of 16 of w
// readable (zero padded).  The 16 x 16 blocks (bi <= bj) are dealt to the four waves of the workgroup;
// v_mfma_f64_16x16x4_f64 takes A = tile^T (lane: column, k: row) and B = tile.
__device__ inline void gram_tile_f64(const float* tile, int tw, int nrows, int w, double* __restrict__ g_generic) {
    PSGD_GLOBAL double* __restrict__ g = as_global(g_generic);
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int li = lane & 15, lk = lane >> 4;
    const int nt = (w + 15) / 16;
    int p = 0;
    for (int bi = 0; bi < nt; ++bi)
        for (int bj = bi; bj < nt; ++bj, ++p) {
            if ((p & 3) != wv) continue;
            doublex4 acc = {0.0, 0.0, 0.0, 0.0};
            const float* __restrict__ pa = tile + lk * tw + 16 * bi + li;
            const float* __restrict__ pb = tile + lk * tw + 16 * bj + li;
            for (int k0 = 0; k0 < nrows; k0 += 4)
                acc = __builtin_amdgcn_mfma_f64_16x16x4f64((double)pa[k0 * tw], (double)pb[k0 * tw], acc, 0, 0, 0);
            const int j = 16 * bj + li;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int i = 16 * bi + 4 * v + lk;
                if (i <= j && j < w) g[tri_idx(i, j, w)] = acc[v];
            }
        }
}

static_assert(sizeof(LayerDev) % 16 == 0, "descriptor tables are written in 16-byte words");

__device__ inline int side_len(const LayerDev& L, int side) { return side == SIDE_L ? L.rows : L.cols; }
__device__ inline int side_lenP(const LayerDev& L, int side) { return side == SIDE_L ? L.rowsP : L.colsP; }

}  // namespace psgd
