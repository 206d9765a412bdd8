// Offline calibration: from the Hessian H = X^T X of the layer-wise objective (Eq. 5, App. A.2) to the matrix U that
// carries the updates of Eq. 12 -- dampening and Cholesky factorization (Sec. 3.3).
//
// U is the upper-triangular factor of the inverse dampened Hessian, H_d^-1 = U^T U.  It is reached without forming
// H_d^-1: with J the index reversal, the lower Cholesky factor L of J H_d J gives H_d = R R^T with R = J L J upper
// triangular, hence H_d^-1 = (R^-1)^T R^-1 and U = R^-1 = J L^-1 J (the factor with positive diagonal is unique).
// So the work is one blocked Cholesky factorization and one blocked triangular inversion, both in float64 on 64 x 64
// tiles (the Hessian arrives as float32, and U leaves as float32):
//   factorization, for each diagonal tile k:  factor the tile and invert its factor (one workgroup);  scale the tiles
//     below it by that inverse;  subtract the panel's outer product from every tile to the right (right-looking);
//   inversion X = L^-1, for each tile row k:  X[k, j] = L_kk^-1 (delta_kj - S[k, j]) for j <= k;  then
//     S[i, j] += L[i, k] X[k, j] for every i > k, j <= k (S lives in the tiles of X that are not final yet).
// Every step is one launch over independent tiles, so no kernel waits on another workgroup.
#include "w4a8_device.hpp"
#include "w4a8_internal.hpp"

namespace w4a8 {
namespace {

constexpr int TB = 64;              // tile edge
constexpr int KS = 16;              // depth of one staged slice

// scalars[0] = damp * mean(diag(H)); *info = 0.  One workgroup; a fixed summation order.
__global__ void __launch_bounds__(256) damp_term_kernel(const float* __restrict__ h, int n, double damp, double* __restrict__ scalars,
                                                        int32_t* __restrict__ info) {
    __shared__ double part[256];
    double s = 0.0;
    for (int i = threadIdx.x; i < n; i += 256) s += (double)h[(int64_t)i * n + i];
    part[threadIdx.x] = s;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        scalars[0] = damp * part[0] / (double)n;
        *info = 0;
    }
}

// a[i, j] = H_d[p(n-1-i), p(n-1-j)] for j <= i (the lower triangle of the reversed, reordered, dampened Hessian)
__global__ void __launch_bounds__(256) gather_reversed_kernel(const float* __restrict__ h, const int32_t* __restrict__ perm, int n,
                                                              const double* __restrict__ scalars, double* __restrict__ a) {
    const int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (u >= (int64_t)n * n) return;
    const int i = (int)(u / n), j = (int)(u - (int64_t)i * n);
    if (j > i) return;
    const int oi = perm ? perm[n - 1 - i] : n - 1 - i, oj = perm ? perm[n - 1 - j] : n - 1 - j;
    double v = (double)h[(int64_t)oi * n + oj];
    if (i == j) v += scalars[0];
    a[u] = v;
}

// Diagonal tile kb: a[kb, kb] <- its lower Cholesky factor L (zeros above the diagonal); dinv[kb] <- V = L^-1, row-major
// 64 x 64 (zeros above the diagonal).  A pivot that is not positive is reported through *info (1 + its index in the
// reversed order, first failure only); the results are then not finite.
// The tile lives in registers, 4 x 4 per thread (thread (ty, tx) = (t / 16, t % 16) owns rows 4 ty.., columns 4 tx..),
// and so does S, which starts as the identity and ends as V.  Step j: the owners of column j scale it by the pivot's
// root (column j of L), the owners of row j of S divide it by the same (row j of V); both go through LDS to everyone,
// who then take L[r, j] L[c, j] off their part of the tile and L[r, j] V[j, c] off their part of S.
__global__ void __launch_bounds__(256) factor_diagonal_kernel(double* __restrict__ a, int n, int kb, double* __restrict__ dinv,
                                                              int32_t* __restrict__ info) {
    __shared__ __attribute__((aligned(16))) double lcol[TB], vrow[TB];
    __shared__ double pivot;
    const int t = threadIdx.x, ty = t >> 4, tx = t & 15;
    double* tile = a + ((int64_t)kb * TB) * n + (int64_t)kb * TB;
    double A[4][4], S[4][4];
#pragma unroll
    for (int rr = 0; rr < 4; ++rr)
#pragma unroll
        for (int cc = 0; cc < 4; ++cc) {
            const int r = 4 * ty + rr, c = 4 * tx + cc;
            A[rr][cc] = (c <= r) ? tile[(int64_t)r * n + c] : 0.0;
            S[rr][cc] = (r == c) ? 1.0 : 0.0;
        }
    if (t == 0) pivot = A[0][0];
    __syncthreads();
    for (int jb = 0; jb < TB / 4; ++jb) {
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            const int j = 4 * jb + jj;
            const double d = pivot;
            if (t == 0 && !(d > 0.0) && *info == 0) *info = kb * TB + j + 1;
            const double s = sqrt(d), rs = 1.0 / s;              // one division per step; the scalings below multiply
            if (tx == jb) {                                      // owners of column j
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) {
                    const int r = 4 * ty + rr;
                    if (r >= j) {
                        A[rr][jj] = (r == j) ? s : A[rr][jj] * rs;
                        lcol[r] = A[rr][jj];
                    }
                }
            }
            if (ty == jb) {                                      // owners of row j of S
#pragma unroll
                for (int cc = 0; cc < 4; ++cc) {
                    const int c = 4 * tx + cc;
                    if (c <= j) {
                        S[jj][cc] *= rs;
                        vrow[c] = S[jj][cc];
                    }
                }
            }
            __syncthreads();
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const int r = 4 * ty + rr;
                if (r > j) {
                    const double lr = lcol[r];
#pragma unroll
                    for (int cc = 0; cc < 4; ++cc) {
                        const int c = 4 * tx + cc;
                        if (c > j && c <= r) A[rr][cc] -= lr * lcol[c];
                        if (c <= j) S[rr][cc] -= lr * vrow[c];
                    }
                }
            }
            // the owner of the next pivot hands it on
            if (jj < 3) {
                if (ty == jb && tx == jb) pivot = A[(jj + 1) & 3][(jj + 1) & 3];
            } else {
                if (ty == jb + 1 && tx == jb + 1) pivot = A[0][0];
            }
            __syncthreads();
        }
    }
    double* dv = dinv + (int64_t)kb * TB * TB;
#pragma unroll
    for (int rr = 0; rr < 4; ++rr)
#pragma unroll
        for (int cc = 0; cc < 4; ++cc) {
            const int r = 4 * ty + rr, c = 4 * tx + cc;
            tile[(int64_t)r * n + c] = (c <= r) ? A[rr][cc] : 0.0;
            dv[r * TB + c] = (c <= r) ? S[rr][cc] : 0.0;
        }
}

// acc[i][j] += sum over k < depth of A(4 ty + i, k) * B(k, 4 tx + j) for a 64 x 64 tile, thread (ty, tx) = (t / 16,
// t % 16).  A(r, k) = ap[r * ars + k] (k contiguous); B(k, c) = bp[k * bks + c * bcs], with k contiguous in memory when
// B_KFAST and c contiguous otherwise (that only chooses which threads load which element).  Ends with a barrier after
// the last slice has been read from global memory AND consumed, so a caller may overwrite an operand tile afterwards.
template <bool B_KFAST>
__device__ __forceinline__ void tile_mac(double (&acc)[4][4], const double* ap, int64_t ars, const double* bp, int64_t bks,
                                         int64_t bcs, int depth, double* as, double* bs) {
    const int t = threadIdx.x, ty = t >> 4, tx = t & 15;
    for (int k0 = 0; k0 < depth; k0 += KS) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int ra = t >> 2, ka = (t & 3) * 4 + e;
            as[ka * TB + ra] = ap[(int64_t)ra * ars + k0 + ka];
            const int cb = B_KFAST ? (t >> 2) : (t & 15) * 4 + e, kb = B_KFAST ? (t & 3) * 4 + e : (t >> 4);
            bs[kb * TB + cb] = bp[(int64_t)(k0 + kb) * bks + (int64_t)cb * bcs];
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < KS; ++k) {
            double av[4], bv[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                av[e] = as[k * TB + ty * 4 + e];
                bv[e] = bs[k * TB + tx * 4 + e];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fma(av[i], bv[j], acc[i][j]);
        }
        __syncthreads();
    }
}

// a[i, kb] <- a[i, kb] * (L_kk^-1)^T for the tiles i = kb + 1 + blockIdx.x below the diagonal tile
__global__ void __launch_bounds__(256) scale_panel_kernel(double* a, int n, int kb, const double* dinv) {
    __shared__ double as[KS * TB], bs[KS * TB];
    const int i = kb + 1 + blockIdx.x;
    double* tile = a + ((int64_t)i * TB) * n + (int64_t)kb * TB;
    double acc[4][4] = {};
    // B(k, c) = V(c, k) = dinv[c * 64 + k]
    tile_mac<true>(acc, tile, n, dinv + (int64_t)kb * TB * TB, 1, TB, TB, as, bs);
    const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c) tile[(int64_t)(ty * 4 + r) * n + tx * 4 + c] = acc[r][c];
}

// a[i, j] -= a[i, kb] a[j, kb]^T for kb < j <= i; blockIdx = (j - kb - 1, i - kb - 1)
__global__ void __launch_bounds__(256) trailing_update_kernel(double* a, int n, int kb) {
    __shared__ double as[KS * TB], bs[KS * TB];
    const int j = kb + 1 + blockIdx.x, i = kb + 1 + blockIdx.y;
    if (j > i) return;
    double acc[4][4] = {};
    // B(k, c) = a[j, kb](c, k)
    tile_mac<true>(acc, a + ((int64_t)i * TB) * n + (int64_t)kb * TB, n, a + ((int64_t)j * TB) * n + (int64_t)kb * TB, 1, n,
                   TB, as, bs);
    double* tile = a + ((int64_t)i * TB) * n + (int64_t)j * TB;
    const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c) tile[(int64_t)(ty * 4 + r) * n + tx * 4 + c] -= acc[r][c];
}

// x[kb, j] <- L_kk^-1 (delta_kj - S[kb, j]) for j = blockIdx.x <= kb, S being what x[kb, j] holds
__global__ void __launch_bounds__(256) finish_row_kernel(double* x, int n, int kb, const double* dinv) {
    __shared__ double as[KS * TB], bs[KS * TB];
    const int j = blockIdx.x;
    const double* dv = dinv + (int64_t)kb * TB * TB;
    double* tile = x + ((int64_t)kb * TB) * n + (int64_t)j * TB;
    const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
    double acc[4][4] = {};
    if (j < kb) tile_mac<false>(acc, dv, TB, tile, n, 1, TB, as, bs);
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c)
            tile[(int64_t)(ty * 4 + r) * n + tx * 4 + c] = (j < kb) ? -acc[r][c] : dv[(ty * 4 + r) * TB + tx * 4 + c];
}

// S[i, j] (+)= L[i, kb] x[kb, j] for i > kb, j <= kb (j == kb: the tile's first term); blockIdx = (j, i - kb - 1)
__global__ void __launch_bounds__(256) push_row_kernel(const double* a, double* x, int n, int kb) {
    __shared__ double as[KS * TB], bs[KS * TB];
    const int j = blockIdx.x, i = kb + 1 + blockIdx.y;
    double acc[4][4] = {};
    tile_mac<false>(acc, a + ((int64_t)i * TB) * n + (int64_t)kb * TB, n, x + ((int64_t)kb * TB) * n + (int64_t)j * TB, n, 1, TB,
                    as, bs);
    double* tile = x + ((int64_t)i * TB) * n + (int64_t)j * TB;
    const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            double* p = tile + (int64_t)(ty * 4 + r) * n + tx * 4 + c;
            *p = (j < kb) ? *p + acc[r][c] : acc[r][c];
        }
}

// u[r, c] = X[n-1-r, n-1-c] for c >= r, 0 below the diagonal
__global__ void __launch_bounds__(256) write_factor_kernel(const double* __restrict__ x, int n, float* __restrict__ u) {
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (int64_t)n * n) return;
    const int r = (int)(idx / n), c = (int)(idx - (int64_t)r * n);
    u[idx] = (c >= r) ? (float)x[(int64_t)(n - 1 - r) * n + (n - 1 - c)] : 0.0f;
}

}  // namespace

size_t hessian_factor_workspace_bytes(int64_t K) {
    return (size_t)(2 * K * K + K * TB + 2) * sizeof(double);
}

int launch_hessian_inverse_factor(const float* h, int64_t K, double damp, const int32_t* perm, void* workspace, float* u,
                                  int32_t* info, hipStream_t st) {
    const int n = (int)K, nb = n / TB;
    double* a = static_cast<double*>(workspace);
    double* x = a + K * K;
    double* dinv = x + K * K;
    double* scalars = dinv + K * TB;
    const unsigned flat = (unsigned)((K * K + 255) / 256);
    hipLaunchKernelGGL(damp_term_kernel, dim3(1), dim3(256), 0, st, h, n, damp, scalars, info);
    hipLaunchKernelGGL(gather_reversed_kernel, dim3(flat), dim3(256), 0, st, h, perm, n, scalars, a);
    if (int e = launch_status()) return e;
    for (int kb = 0; kb < nb; ++kb) {
        hipLaunchKernelGGL(factor_diagonal_kernel, dim3(1), dim3(256), 0, st, a, n, kb, dinv, info);
        const int below = nb - kb - 1;
        if (below > 0) {
            hipLaunchKernelGGL(scale_panel_kernel, dim3(below), dim3(256), 0, st, a, n, kb, dinv);
            hipLaunchKernelGGL(trailing_update_kernel, dim3(below, below), dim3(256), 0, st, a, n, kb);
        }
        if (int e = launch_status()) return e;
    }
    for (int kb = 0; kb < nb; ++kb) {
        hipLaunchKernelGGL(finish_row_kernel, dim3(kb + 1), dim3(256), 0, st, x, n, kb, dinv);
        if (kb + 1 < nb) hipLaunchKernelGGL(push_row_kernel, dim3(kb + 1, nb - kb - 1), dim3(256), 0, st, a, x, n, kb);
        if (int e = launch_status()) return e;
    }
    hipLaunchKernelGGL(write_factor_kernel, dim3(flat), dim3(256), 0, st, x, n, u);
    return launch_status();
}

}  // namespace w4a8
