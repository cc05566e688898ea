// Plain streaming kernels with the access patterns of the compressor's passes and no arithmetic to speak of:
// what HBM on this machine gives such patterns.  Not part of the library (built into its own shared
// object); `bench.py --ceilings` runs them so that the roofline fractions of the real kernels can be read
// against measured ceilings as well as against the nominal peak.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {
typedef float floatx4 __attribute__((ext_vector_type(4)));
#define GLOBAL_AS __attribute__((address_space(1)))
constexpr int kT = 256;

struct Ptrs { const float* g[8]; };

// contiguous read of n4 16-byte words
__global__ __launch_bounds__(kT) void flat_read(const float* src, size_t n4, float* sink) {
    const GLOBAL_AS floatx4* s = (const GLOBAL_AS floatx4*)src;
    floatx4 a = {0, 0, 0, 0};
    for (size_t i = (size_t)blockIdx.x * kT + threadIdx.x; i < n4; i += (size_t)gridDim.x * kT) a += s[i];
    if (a.x + a.y + a.z + a.w == 12345.678f) sink[0] = a.x;
}

__global__ __launch_bounds__(kT) void flat_copy(const float* src, float* dst, size_t n4) {
    const GLOBAL_AS floatx4* s = (const GLOBAL_AS floatx4*)src;
    GLOBAL_AS floatx4* d = (GLOBAL_AS floatx4*)dst;
    for (size_t i = (size_t)blockIdx.x * kT + threadIdx.x; i < n4; i += (size_t)gridDim.x * kT) d[i] = s[i];
}

// write-only stream (decompress)
__global__ __launch_bounds__(kT) void flat_write(float* dst, size_t n4) {
    GLOBAL_AS floatx4* d = (GLOBAL_AS floatx4*)dst;
    const floatx4 v = {1.0f, 2.0f, 3.0f, (float)blockIdx.x};
    for (size_t i = (size_t)blockIdx.x * kT + threadIdx.x; i < n4; i += (size_t)gridDim.x * kT) d[i] = v;
}

// in place x <- x + 1 (the residual's read-modify-write)
__global__ __launch_bounds__(kT) void flat_rmw(float* buf, size_t n4) {
    GLOBAL_AS floatx4* d = (GLOBAL_AS floatx4*)buf;
    for (size_t i = (size_t)blockIdx.x * kT + threadIdx.x; i < n4; i += (size_t)gridDim.x * kT) d[i] = d[i] + 1.0f;
}

// out = mean of nw arrays + e, elementwise (pass 1 without the product); 4 x 16 bytes per thread and array,
// two arrays in flight
__global__ __launch_bounds__(kT) void form_elementwise(Ptrs p, int nw, const float* e, float* out, size_t n4) {
    constexpr int U = 4;
    const size_t stride = (size_t)gridDim.x * kT;
    const float inv = 1.0f / (float)nw;
    for (size_t base = (size_t)blockIdx.x * kT * U + threadIdx.x; base < n4; base += stride * U) {
        floatx4 acc[U];
#pragma unroll
        for (int u = 0; u < U; ++u) acc[u] = floatx4{0, 0, 0, 0};
        for (int w = 0; w < nw; w += 2) {
            floatx4 x[2][U];
#pragma unroll
            for (int d = 0; d < 2; ++d)
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const size_t i = base + (size_t)u * kT;
                    x[d][u] = (i < n4 && w + d < nw) ? ((const GLOBAL_AS floatx4*)p.g[w + d])[i] : floatx4{0, 0, 0, 0};
                }
#pragma unroll
            for (int d = 0; d < 2; ++d)
#pragma unroll
                for (int u = 0; u < U; ++u) acc[u] += x[d][u];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t i = base + (size_t)u * kT;
            if (i < n4) ((GLOBAL_AS floatx4*)out)[i] = acc[u] * inv + ((const GLOBAL_AS floatx4*)e)[i];
        }
    }
}

// Tile-pattern read of nmat matrices (rows x cols fp32, ld = cols, both multiples of 128), next tile requested
// before the current one is consumed, two workgroups per compute unit like the product kernels.
// COLMODE 0: a workgroup owns 128 rows and walks 64-column chunks along them (256 bytes per row and chunk);
// COLMODE 1: it owns 128 columns and walks 64-row chunks down them (512 bytes per row).
template <int COLMODE>
__global__ __launch_bounds__(kT, 2) void tile_read(const float* const* mats, int rows, int cols, float* sink) {
    const GLOBAL_AS float* m = (const GLOBAL_AS float*)mats[blockIdx.y];
    const int t = threadIdx.x;
    floatx4 acc = {0, 0, 0, 0};
    floatx4 cur[8], nxt[8];
    if (!COLMODE) {
        const int ob = blockIdx.x, nch = cols / 64;
        if (ob >= rows / 128) return;
        const GLOBAL_AS float* base = m + (size_t)(ob * 128 + (t >> 4)) * cols + 4 * (t & 15);
#pragma unroll
        for (int u = 0; u < 8; ++u) cur[u] = *(const GLOBAL_AS floatx4*)(base + (size_t)u * 16 * cols);
        for (int ch = 0; ch < nch; ++ch) {
            if (ch + 1 < nch) {
#pragma unroll
                for (int u = 0; u < 8; ++u) nxt[u] = *(const GLOBAL_AS floatx4*)(base + (size_t)u * 16 * cols + (ch + 1) * 64);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) { acc += cur[u]; cur[u] = nxt[u]; }
        }
    } else {
        const int ob = blockIdx.x, nch = rows / 64;
        if (ob >= cols / 128) return;
        const GLOBAL_AS float* base = m + (size_t)(8 * (t >> 5)) * cols + ob * 128 + 4 * (t & 31);
#pragma unroll
        for (int u = 0; u < 8; ++u) cur[u] = *(const GLOBAL_AS floatx4*)(base + (size_t)u * cols);
        for (int ch = 0; ch < nch; ++ch) {
            if (ch + 1 < nch) {
#pragma unroll
                for (int u = 0; u < 8; ++u) nxt[u] = *(const GLOBAL_AS floatx4*)(base + (size_t)((ch + 1) * 64 + u) * cols);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) { acc += cur[u]; cur[u] = nxt[u]; }
        }
    }
    if (acc.x + acc.y + acc.z + acc.w == 12345.678f) sink[0] = acc.x;
}

// ---- the same streams with the non-temporal hint (what the library's kernels use on data touched once)
__global__ __launch_bounds__(kT) void flat_read_nt(const float* src, size_t n4, float* sink) {
    const GLOBAL_AS floatx4* s = (const GLOBAL_AS floatx4*)src;
    floatx4 a = {0, 0, 0, 0};
    for (size_t i = (size_t)blockIdx.x * kT + threadIdx.x; i < n4; i += (size_t)gridDim.x * kT) a += __builtin_nontemporal_load(s + i);
    if (a.x + a.y + a.z + a.w == 12345.678f) sink[0] = a.x;
}

// in place x <- x + 1, four 16-byte pieces per thread in flight, non-temporal loads and stores
__global__ __launch_bounds__(kT) void flat_rmw_nt(float* buf, size_t n4) {
    GLOBAL_AS floatx4* d = (GLOBAL_AS floatx4*)buf;
    constexpr int U = 4;
    const size_t stride = (size_t)gridDim.x * kT * U;
    for (size_t b = (size_t)blockIdx.x * kT * U + threadIdx.x; b < n4; b += stride) {
        floatx4 x[U];
#pragma unroll
        for (int u = 0; u < U; ++u) { const size_t i = b + (size_t)u * kT; x[u] = i < n4 ? __builtin_nontemporal_load(d + i) : floatx4{0, 0, 0, 0}; }
#pragma unroll
        for (int u = 0; u < U; ++u) { const size_t i = b + (size_t)u * kT; if (i < n4) __builtin_nontemporal_store(x[u] + 1.0f, d + i); }
    }
}

// Write-only in tiles (decompress): a workgroup writes a 128 x 128 tile, consecutive workgroups consecutive column
// blocks.  PAT 0: per store instruction a wave writes 2 rows x 512 B, rows 4 apart (the MFMA accumulator layout of the
// outer-product kernels); PAT 1: tile 64 rows x 256 columns, per store a wave writes 1 row x 1 KB; PAT 2: tile 128 rows x
// 256 columns in the accumulator layout of eight column blocks, a lane owning 8 consecutive columns: two stores per
// row pair, each 32 pieces of 16 bytes 32 bytes apart, together 2 rows x 1 KB.
template <int PAT>
__global__ __launch_bounds__(kT) void tile_write(float* const* mats, int rows, int cols) {
    GLOBAL_AS float* m = (GLOBAL_AS float*)mats[blockIdx.y];
    const int t = threadIdx.x, lane = t & 63, wv = t >> 6, li = lane & 31, lg = lane >> 5;
    const floatx4 val = {1.f, 2.f, 3.f, (float)blockIdx.x};
    if (PAT == 2) {
        const int n_cb = cols / 256, cb = blockIdx.x % n_cb, rb = blockIdx.x / n_cb;
        if (rb >= rows / 128) return;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            GLOBAL_AS float* p = m + (size_t)(rb * 128 + 32 * wv + 8 * (v >> 2) + (v & 3) + 4 * lg) * cols + cb * 256 + 8 * li;
            *(GLOBAL_AS floatx4*)p = val;
            *(GLOBAL_AS floatx4*)(p + 4) = val;
        }
    } else if (PAT == 1) {
        const int n_cb = cols / 256, cb = blockIdx.x % n_cb, rb = blockIdx.x / n_cb;
        if (rb >= rows / 64) return;
#pragma unroll
        for (int v = 0; v < 16; ++v)
            *(GLOBAL_AS floatx4*)(m + (size_t)(rb * 64 + 16 * wv + v) * cols + cb * 256 + 4 * lane) = val;
    } else {
        const int n_cb = cols / 128, cb = blockIdx.x % n_cb, rb = blockIdx.x / n_cb;
        if (rb >= rows / 128) return;
#pragma unroll
        for (int v = 0; v < 16; ++v)
            *(GLOBAL_AS floatx4*)(m + (size_t)(rb * 128 + 32 * wv + 8 * (v >> 2) + (v & 3) + 4 * lg) * cols + cb * 128 + 4 * li) = val;
    }
}

// Pass 1 of the one-worker bf16 case without the product: S <- widen(G) + S in place, a workgroup owns 128 rows and
// walks 64-column chunks along them, next chunk requested before the current one is consumed.  ROT 1: every row
// block starts its walk at a chunk of its own (ob + ob / 8) and wraps around, as the library's kernel does; ROT 0:
// all row blocks walk in step from column 0 and meet on the same memory channels.
typedef unsigned int uintx2 __attribute__((ext_vector_type(2)));
template <int ROT>
__global__ __launch_bounds__(kT, 2) void form_tile(const uint16_t* const* gs, float* const* ss, int rows, int cols) {
    const GLOBAL_AS uint16_t* g = (const GLOBAL_AS uint16_t*)gs[blockIdx.y];
    GLOBAL_AS float* s = (GLOBAL_AS float*)ss[blockIdx.y];
    const int t = threadIdx.x, ob = blockIdx.x;
    if (ob >= rows / 128) return;
    const int nch = cols / 64, rot = ROT ? (ob + (ob >> 3)) % nch : 0;
    const size_t base = (size_t)(ob * 128 + (t >> 4)) * cols + 4 * (t & 15);
    floatx4 sv[8], sn[8];
    uintx2 gv[8], gn[8];
    auto off_of = [&](int it, int u) { int c = it + rot; if (c >= nch) c -= nch; return base + (size_t)u * 16 * cols + (size_t)c * 64; };
#pragma unroll
    for (int u = 0; u < 8; ++u) { sv[u] = __builtin_nontemporal_load((const GLOBAL_AS floatx4*)(s + off_of(0, u))); gv[u] = __builtin_nontemporal_load((const GLOBAL_AS uintx2*)(g + off_of(0, u))); }
    for (int it = 0; it < nch; ++it) {
        if (it + 1 < nch) {
#pragma unroll
            for (int u = 0; u < 8; ++u) { sn[u] = __builtin_nontemporal_load((const GLOBAL_AS floatx4*)(s + off_of(it + 1, u))); gn[u] = __builtin_nontemporal_load((const GLOBAL_AS uintx2*)(g + off_of(it + 1, u))); }
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const floatx4 w = {__uint_as_float(gv[u].x << 16), __uint_as_float(gv[u].x & 0xffff0000u), __uint_as_float(gv[u].y << 16), __uint_as_float(gv[u].y & 0xffff0000u)};
            *(GLOBAL_AS floatx4*)(s + off_of(it, u)) = w + sv[u];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) { sv[u] = sn[u]; gv[u] = gn[u]; }
    }
}
// The walks of the kernels built on 32 x 256 tiles, without the products: every load and store instruction of a
// wavefront covers 1 KB of one row.
//   MODE 0 (form_row_kernel, one bf16 worker): a workgroup owns 32 rows and walks them 256 columns at a time,
//          S <- widen(G) + S in place, next step requested before the current one is consumed; every row block starts
//          at a step of its own.  NTS: non-temporal stores.
//   MODE 1 (col_prod_kernel): a workgroup owns 256 columns and walks down the rows 32 at a time, read only, DEPTH
//          steps in flight.
template <int MODE, int NTS, int DEPTH>
__global__ __launch_bounds__(kT, 2) void walk_32x256(const uint16_t* const* gs, float* const* ss, int rows, int cols, float* sink) {
    const GLOBAL_AS uint16_t* g = MODE == 0 ? (const GLOBAL_AS uint16_t*)gs[blockIdx.y] : nullptr;
    GLOBAL_AS float* s = (GLOBAL_AS float*)ss[blockIdx.y];
    const int t = threadIdx.x, lane = t & 63, wv = t >> 6, ob = blockIdx.x;
    const int nstrip = MODE == 0 ? rows / 32 : cols / 256;
    if (ob >= nstrip) return;
    const int nch = MODE == 0 ? cols / 256 : rows / 32;
    const int rot = MODE == 0 ? ((ob & 7) * (nch >> 3) + 2 * (ob >> 3) + (int)blockIdx.y) % nch : 0;
    auto off_of = [&](int it, int u) -> size_t {
        int ch = it + rot; if (ch >= nch) ch -= nch;
        const int row = (MODE == 0 ? ob * 32 + 4 * u + wv : ch * 32 + 8 * wv + u);
        const int col = (MODE == 0 ? ch * 256 : ob * 256) + 4 * lane;
        return (size_t)row * cols + col;
    };
    floatx4 sv[DEPTH + 1][8];
    uintx2 gv[DEPTH + 1][8];
    auto ld = [&](int it, int slot) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            sv[slot][u] = __builtin_nontemporal_load((const GLOBAL_AS floatx4*)(s + off_of(it, u)));
            if (MODE == 0) gv[slot][u] = __builtin_nontemporal_load((const GLOBAL_AS uintx2*)(g + off_of(it, u)));
        }
    };
    floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) if (d < nch) ld(d, d);
    for (int it0 = 0; it0 < nch; it0 += DEPTH + 1) {
#pragma unroll
        for (int k = 0; k <= DEPTH; ++k) {
            const int it = it0 + k;
            if (it >= nch) break;
            if (it + DEPTH < nch) ld(it + DEPTH, (k + DEPTH) % (DEPTH + 1));
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                if (MODE == 1) { acc += sv[k][u]; continue; }
                const uintx2 b = gv[k][u];
                const floatx4 w = {__uint_as_float(b.x << 16), __uint_as_float(b.x & 0xffff0000u), __uint_as_float(b.y << 16), __uint_as_float(b.y & 0xffff0000u)};
                const floatx4 o = w + sv[k][u];
                if (NTS) __builtin_nontemporal_store(o, (GLOBAL_AS floatx4*)(s + off_of(it, u)));
                else *(GLOBAL_AS floatx4*)(s + off_of(it, u)) = o;
            }
        }
    }
    if (MODE == 1 && acc.x + acc.y + acc.z + acc.w == 12345.678f) sink[0] = acc.x;
}
}  // namespace

// All pointers are device pointers; n = number of floats (multiple of 4); returns the HIP error code.
extern "C" int ceil_flat_read(void* stream, int grid, const void* src, size_t n, void* sink) {
    hipLaunchKernelGGL(flat_read, dim3(grid), dim3(kT), 0, (hipStream_t)stream, (const float*)src, n / 4, (float*)sink);
    return (int)hipGetLastError();
}
extern "C" int ceil_flat_copy(void* stream, int grid, const void* src, void* dst, size_t n) {
    hipLaunchKernelGGL(flat_copy, dim3(grid), dim3(kT), 0, (hipStream_t)stream, (const float*)src, (float*)dst, n / 4);
    return (int)hipGetLastError();
}
extern "C" int ceil_flat_write(void* stream, int grid, void* dst, size_t n) {
    hipLaunchKernelGGL(flat_write, dim3(grid), dim3(kT), 0, (hipStream_t)stream, (float*)dst, n / 4);
    return (int)hipGetLastError();
}
extern "C" int ceil_flat_rmw(void* stream, int grid, void* buf, size_t n) {
    hipLaunchKernelGGL(flat_rmw, dim3(grid), dim3(kT), 0, (hipStream_t)stream, (float*)buf, n / 4);
    return (int)hipGetLastError();
}
// g: host array of nw (<= 8) device pointers
extern "C" int ceil_form(void* stream, int grid, const void* const* g, int nw, const void* e, void* out, size_t n) {
    if (nw < 1 || nw > 8) return (int)hipErrorInvalidValue;
    Ptrs p;
    for (int i = 0; i < 8; ++i) p.g[i] = (const float*)g[i < nw ? i : 0];
    hipLaunchKernelGGL(form_elementwise, dim3(grid), dim3(kT), 0, (hipStream_t)stream, p, nw, (const float*)e, (float*)out, n / 4);
    return (int)hipGetLastError();
}
// mats: device array of nmat device pointers; rows, cols multiples of 128
extern "C" int ceil_tile_read(void* stream, int colmode, const void* const* mats, int nmat, int rows, int cols, void* sink) {
    if (rows % 128 || cols % 128 || nmat < 1) return (int)hipErrorInvalidValue;
    const float* const* m = (const float* const*)mats;
    if (colmode) hipLaunchKernelGGL(tile_read<1>, dim3(cols / 128, nmat), dim3(kT), 0, (hipStream_t)stream, m, rows, cols, (float*)sink);
    else hipLaunchKernelGGL(tile_read<0>, dim3(rows / 128, nmat), dim3(kT), 0, (hipStream_t)stream, m, rows, cols, (float*)sink);
    return (int)hipGetLastError();
}
extern "C" int ceil_flat_read_nt(void* stream, int grid, const void* src, size_t n, void* sink) {
    hipLaunchKernelGGL(flat_read_nt, dim3(grid), dim3(kT), 0, (hipStream_t)stream, (const float*)src, n / 4, (float*)sink);
    return (int)hipGetLastError();
}
extern "C" int ceil_flat_rmw_nt(void* stream, int grid, void* buf, size_t n) {
    hipLaunchKernelGGL(flat_rmw_nt, dim3(grid), dim3(kT), 0, (hipStream_t)stream, (float*)buf, n / 4);
    return (int)hipGetLastError();
}
// mats: device array of nmat device pointers to rows x cols fp32 (rows multiple of 128, cols of 256)
extern "C" int ceil_tile_write(void* stream, int pat, const void* const* mats, int nmat, int rows, int cols) {
    if (rows % 128 || cols % 256 || nmat < 1) return (int)hipErrorInvalidValue;
    dim3 grid((rows / 128) * (cols / 128), nmat);
    float* const* m = (float* const*)mats;
    if (pat == 2) hipLaunchKernelGGL(tile_write<2>, dim3((rows / 128) * (cols / 256), nmat), dim3(kT), 0, (hipStream_t)stream, m, rows, cols);
    else if (pat) hipLaunchKernelGGL(tile_write<1>, grid, dim3(kT), 0, (hipStream_t)stream, m, rows, cols);
    else hipLaunchKernelGGL(tile_write<0>, grid, dim3(kT), 0, (hipStream_t)stream, m, rows, cols);
    return (int)hipGetLastError();
}
// gs, ss: device arrays of nmat device pointers (bf16 and fp32 matrices rows x cols, rows multiple of 128, cols of 64)
extern "C" int ceil_form_tile(void* stream, int rot, const void* const* gs, const void* const* ss, int nmat, int rows, int cols) {
    if (rows % 128 || cols % 64 || nmat < 1) return (int)hipErrorInvalidValue;
    dim3 grid(rows / 128, nmat);
    if (rot) hipLaunchKernelGGL(form_tile<1>, grid, dim3(kT), 0, (hipStream_t)stream, (const uint16_t* const*)gs, (float* const*)ss, rows, cols);
    else hipLaunchKernelGGL(form_tile<0>, grid, dim3(kT), 0, (hipStream_t)stream, (const uint16_t* const*)gs, (float* const*)ss, rows, cols);
    return (int)hipGetLastError();
}
// which: 0 = form walk, plain stores; 1 = form walk, non-temporal stores; 2 = read-only walk down the rows, one step in
// flight; 3 = two steps in flight.  gs (which < 2), ss: device arrays of nmat device pointers to bf16 / fp32 matrices
// rows x cols (rows multiple of 32, cols of 256)
extern "C" int ceil_walk_32x256(void* stream, int which, const void* const* gs, const void* const* ss, int nmat, int rows,
                                int cols, void* sink) {
    if (rows % 32 || cols % 256 || nmat < 1 || which < 0 || which > 3) return (int)hipErrorInvalidValue;
    const uint16_t* const* g = (const uint16_t* const*)gs;
    float* const* s = (float* const*)ss;
    hipStream_t st = (hipStream_t)stream;
    if (which == 0) hipLaunchKernelGGL((walk_32x256<0, 0, 1>), dim3(rows / 32, nmat), dim3(kT), 0, st, g, s, rows, cols, (float*)sink);
    else if (which == 1) hipLaunchKernelGGL((walk_32x256<0, 1, 1>), dim3(rows / 32, nmat), dim3(kT), 0, st, g, s, rows, cols, (float*)sink);
    else if (which == 2) hipLaunchKernelGGL((walk_32x256<1, 0, 1>), dim3(cols / 256, nmat), dim3(kT), 0, st, g, s, rows, cols, (float*)sink);
    else hipLaunchKernelGGL((walk_32x256<1, 0, 2>), dim3(cols / 256, nmat), dim3(kT), 0, st, g, s, rows, cols, (float*)sink);
    return (int)hipGetLastError();
}
