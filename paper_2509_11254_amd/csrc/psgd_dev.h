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

constexpr int kThreads = 256;      // 4 wavefronts of 64 lanes
constexpr int kLenPad = 128;       // packed operand rows are padded (with zeros) to this multiple
constexpr int kMaxGramSplit = 8;   // row blocks of the partial Gram matrices

enum Side { SIDE_L = 0, SIDE_W = 1 };
// Roles: the paper's P~ and Q (user buffers, leading dimension r) and the two wide internal
// blocks of the subspace iteration (leading dimension wz).
enum Role { ROLE_P = 0, ROLE_Q = 1, ROLE_ZP = 2, ROLE_ZQ = 3, ROLE_COUNT = 4 };

struct ThinRef {
    float* ptr;   // len x width, row-major
    int ld;
    int width;
};

// Split-bf16 operand copies of one thin matrix X (len x width), zero padded to lenP x cp:
//   n_hi/n_lo : [lenP][cp]   row-major      (A/B operand of the rank-r outer product)
//   t_hi/t_lo : [cp][lenP]   transposed     (B operand of the tall-skinny products)
// X = hi + lo up to 2^-17 relative, each half a bf16.
struct PackRef {
    bf16_t* n_hi;
    bf16_t* n_lo;
    bf16_t* t_hi;
    bf16_t* t_lo;
};

struct LayerDev {
    int rows, cols;
    int64_t ld;
    int r;             // rank of the compressor
    int wz;            // block width of the subspace iteration (multiple of 32, >= r)
    int gdt;           // PSGD_F32 / PSGD_BF16
    int n_workers;
    int transposed;    // rows < cols: P~ is W-side
    int rowsP, colsP;  // rows / cols rounded up to kLenPad
    int split_row;     // k-splits of the row-mode product  (reduction over cols)
    int split_col;     // k-splits of the column-mode product (reduction over rows)
    const void* const* G;   // n_workers device pointers
    float* S;               // E on entry, M between the sweeps, E_{t+1} on exit
    ThinRef thin[ROLE_COUNT];
    float* part[2];         // per side: [split][lenP][cpmax] fp32 partial products
    PackRef pack[2];        // per side
    double* gram;           // [kMaxGramSplit][wmax*wmax] partial Gram matrices
    double* tmat;           // [wmax*wmax] small factor applied from the right
    double* evec;           // [wmax*wmax] accumulated Jacobi rotations
    double* jwork;          // [wmax*wmax] Jacobi working copy of the projected Gram matrix
    double* eval;           // [wmax]
    int* status;            // [4] : rank_deficient, -, sigma_max bits, sigma_r bits
};

__host__ __device__ inline int side_of_role(int transposed, int role) {
    // P-like roles live on the long side (m): L-side unless the storage is transposed.
    const int p_like = (role == ROLE_P || role == ROLE_ZP);
    return (p_like != (transposed != 0)) ? SIDE_L : SIDE_W;
}

__device__ inline int side_len(const LayerDev& L, int side) { return side == SIDE_L ? L.rows : L.cols; }
__device__ inline int side_lenP(const LayerDev& L, int side) { return side == SIDE_L ? L.rowsP : L.colsP; }

}  // namespace psgd
