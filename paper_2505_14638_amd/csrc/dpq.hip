// Offline calibration: Dual Precision Quantization (Alg. 1, Eq. 5-12) and the Group-Aware Reordering permutation
// (Sec. 3.2, App. A.3).
//
// Alg. 1 walks along a row: quantize one weight (FP8, then INT4, Eq. 7-9), dequantize it the way inference will
// (Eq. 10-11), and push the error onto every later weight of the row through the Hessian factor U (Eq. 12; U is the
// upper Cholesky factor of the inverse Hessian, Sec. 3.3).  Rows are independent, columns strictly sequential.  The
// work is arranged in blocks of 128 columns: inside a block 32 lanes of one wavefront own one row (each takes
// the quantization step itself and applies the error to its share of the rest of the block); the columns right of
// the block receive the block's 128 errors afterwards, in one tiled pass over the matrix.  Every weight still sees the same float32 operations in the same order as in the plain
// column-by-column statement (w <- w - err_q * U[q, v] for q ascending, product and difference rounded separately),
// so the integer decisions are reproducible bit for bit; only the time at which an update is applied moves.
#include "w4a8_device.hpp"
#include "w4a8_internal.hpp"

namespace w4a8 {
namespace {

constexpr int DPQ_BLOCK = 128;      // columns per block

// val(nearest_Z(t)): the E4M3 value nearest to t (ties to even, saturating), as a float32
__device__ __forceinline__ float fp8_value(float t) {
    const int b = __builtin_amdgcn_cvt_pk_fp8_f32(sat448(t), 0.0f, 0, false);
    return __builtin_amdgcn_cvt_f32_fp8(b, 0);
}

__device__ __forceinline__ float load_as_float(const float* p) { return *p; }
__device__ __forceinline__ float load_as_float(const uint16_t* p) { return bf16_bits_to_f32(*p); }

// position i of the reordered tensor holds original column perm[i]: inside a group by descending diagonal, groups
// by descending maximum; ties keep the lower original index first.  One thread per column.
__global__ void __launch_bounds__(256) gar_permutation_kernel(const float* __restrict__ d, int K, int G, int32_t* __restrict__ perm) {
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= K) return;
    const int g = c / G, NG = K / G;
    const float mine = d[c];
    int inside = 0;
    float gmax = d[g * G];
    for (int j = 0; j < G; ++j) {
        const float v = d[g * G + j];
        inside += (v > mine) || (v == mine && g * G + j < c);
        gmax = fmaxf(gmax, v);
    }
    int rank = 0;
    for (int h = 0; h < NG; ++h) {
        float m = d[h * G];
        for (int j = 1; j < G; ++j) m = fmaxf(m, d[h * G + j]);
        rank += (m > gmax) || (m == gmax && h < g);
    }
    perm[rank * G + inside] = c;
}

// work[n, i] = w[n, perm[i]] (perm == nullptr: a copy)
__global__ void __launch_bounds__(256) dpq_gather_kernel(const float* __restrict__ w, const int32_t* __restrict__ perm,
                                                         int64_t N, int64_t K, float* __restrict__ work) {
    const int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (u >= N * K) return;
    const int64_t n = u / K, i = u - n * K;
    work[u] = w[n * K + (perm ? perm[i] : i)];
}

struct DpqArgs {
    float* work;                  // [N, K] current weights, reordered columns
    const float* u;               // [K, K] upper factor, reordered columns
    const float* s_w;
    int per_channel;
    const int32_t* perm;          // or nullptr
    int N, K, G;
    uint8_t* codes;               // [N, K], original column order
    float* scales;                // [N, K / G], original group order
    uint8_t* zeros;               // [N, K / G]
    float* err;                   // [N, 128] errors of the current block
    int mse_grid;                 // candidates of the scale search (Sec. 3.3); <= 1: none
    float shrink_step;            // max_shrink / mse_grid
};

// Eq. 8 for a range [lo, hi] that contains zero: s = (hi - lo) / 15 (1 for an empty range), z = round(-lo / s)
__device__ __forceinline__ void group_params(float lo, float hi, float& s, float& z) {
    const float span = __fsub_rn(hi, lo);
    s = (span == 0.0f) ? 1.0f : __fdiv_rn(span, 15.0f);
    z = fminf(fmaxf(rintf(__fdiv_rn(-lo, s)), 0.0f), 15.0f);
}

// One block of 128 columns starting at c0.  The DPQ_LPR lanes of a row sit next to each other in one wavefront and
// share the row's 128 weights through LDS; a wavefront executes its LDS accesses in program order, so a lane's update
// of a column is in place before every lane of the row reads that column in a later step -- no barrier is needed.
// All lanes of a row take the (identical) quantization step; lane p updates the columns v with v % DPQ_LPR == p.
// DPQ_LPR lanes per row: more lanes shorten a step (fewer columns to update per lane) but repeat the quantization
// arithmetic on every one of them, so many lanes suit few rows and few lanes many rows.
// The 128 steps are strictly sequential.  STAGE_U: the block's corner of U is staged in LDS once (64 KiB), so that no
// step waits for a global load -- right when there are few rows and nothing else to run meanwhile; with many rows
// the loads stay global and many small workgroups per compute unit hide them instead (64 KiB of LDS would leave two).
template <int DPQ_LPR, bool STAGE_U, int DPQ_THREADS>
__global__ void __launch_bounds__(DPQ_THREADS) dpq_block_kernel(DpqArgs a, int c0) {
    constexpr int DPQ_ROWS = DPQ_THREADS / DPQ_LPR;              // rows per workgroup
    __shared__ float wl[DPQ_BLOCK * DPQ_ROWS];                   // wl[v * DPQ_ROWS + r]: column c0 + v of row r of the workgroup
    __shared__ float ul[STAGE_U ? DPQ_BLOCK * DPQ_BLOCK : 1];    // ul[q * 128 + v] = U[c0 + q, c0 + v]
    if (STAGE_U) {
        for (int idx = threadIdx.x; idx < DPQ_BLOCK * DPQ_BLOCK; idx += DPQ_THREADS)
            ul[idx] = a.u[(int64_t)(c0 + idx / DPQ_BLOCK) * a.K + c0 + idx % DPQ_BLOCK];
        __syncthreads();
    }
    const int lane = threadIdx.x / DPQ_LPR, part = threadIdx.x % DPQ_LPR;
    const int n = blockIdx.x * DPQ_ROWS + lane;
    if (n >= a.N) return;                                        // whole rows leave together
    float* row = a.work + (int64_t)n * a.K;
    const float sw = a.s_w[a.per_channel ? n : 0];
    const int NG = a.K / a.G;
    for (int v = part; v < DPQ_BLOCK; v += DPQ_LPR) wl[v * DPQ_ROWS + lane] = row[c0 + v];
    __builtin_amdgcn_wave_barrier();                             // keeps the compiler from moving LDS accesses across
    // group parameters (Eq. 8 on the group's current weights): computed where the group starts, kept in the outputs
    const int g = c0 / a.G;
    const int og = a.perm ? a.perm[g * a.G] / a.G : g;           // the original group these columns belong to
    float s, z;
    if (c0 % a.G == 0) {
        float lo = 0.0f, hi = 0.0f;                              // minimum and maximum: any order gives the same result
        for (int j = part; j < a.G; j += DPQ_LPR) {
            const float w8 = fp8_value(__fdiv_rn(row[c0 + j], sw));
            lo = fminf(lo, w8);
            hi = fmaxf(hi, w8);
        }
#pragma unroll
        for (int m = 1; m < DPQ_LPR; m <<= 1) {
            lo = fminf(lo, __shfl_xor(lo, m));
            hi = fmaxf(hi, __shfl_xor(hi, m));
        }
        group_params(lo, hi, s, z);
        if (a.mse_grid > 1) {
            // The scale search of Sec. 3.3: candidate i shrinks the range by p_i = 1 - i * shrink_step and is scored by
            // the squared error, on the FP8 values, of what inference will reconstruct (Eq. 9 with clipping, Eq. 10);
            // float32 sums over the group in visiting order.  The row's lanes share the candidates (i % DPQ_LPR) and
            // then agree on the smallest score, the lowest index among equals -- the first minimum of a sequential scan.
            float best = __builtin_inff(), bs = s, bz = z;
            int best_i = a.mse_grid;
            for (int i = part; i < a.mse_grid; i += DPQ_LPR) {
                const float p = __fsub_rn(1.0f, __fmul_rn((float)i, a.shrink_step));
                float si, zi;
                group_params(__fmul_rn(p, lo), __fmul_rn(p, hi), si, zi);
                float score = 0.0f;
                for (int j = 0; j < a.G; ++j) {
                    const float w8 = fp8_value(__fdiv_rn(row[c0 + j], sw));
                    const float uq = fminf(fmaxf(rintf(__fadd_rn(__fdiv_rn(w8, si), zi)), 0.0f), 15.0f);
                    const float d = __fsub_rn(w8, fp8_value(__fmul_rn(__fsub_rn(uq, zi), si)));
                    score = __fadd_rn(score, __fmul_rn(d, d));
                }
                if (score < best) { best = score; best_i = i; bs = si; bz = zi; }
            }
#pragma unroll
            for (int m = 1; m < DPQ_LPR; m <<= 1) {
                const float ob = __shfl_xor(best, m), os = __shfl_xor(bs, m), oz = __shfl_xor(bz, m);
                const int oi = __shfl_xor(best_i, m);
                if (ob < best || (ob == best && oi < best_i)) { best = ob; best_i = oi; bs = os; bz = oz; }
            }
            s = bs;
            z = bz;
        }
        if (part == 0) {
            a.scales[(int64_t)n * NG + og] = s;
            a.zeros[(int64_t)n * NG + og] = (uint8_t)z;
        }
    } else {
        s = a.scales[(int64_t)n * NG + og];
        z = (float)a.zeros[(int64_t)n * NG + og];
    }
    for (int q = 0; q < DPQ_BLOCK; ++q) {
        const float w = wl[q * DPQ_ROWS + lane];
        const float w8 = fp8_value(__fdiv_rn(w, sw));                                     // Eq. 7
        const float t = __fadd_rn(__fdiv_rn(w8, s), z);
        const float uq = fminf(fmaxf(rintf(t), 0.0f), 15.0f);                             // Eq. 9
        const float w8_hat = fp8_value(__fmul_rn(__fsub_rn(uq, z), s));                   // Eq. 10
        const float w_hat = __fmul_rn(w8_hat, sw);                                        // Eq. 11
        const float* urow = STAGE_U ? ul + q * DPQ_BLOCK : a.u + (int64_t)(c0 + q) * a.K + c0;   // U[c0 + q, c0 + v]
        const float e = __fdiv_rn(__fsub_rn(w, w_hat), urow[q]);
        if (part == 0) {
            a.err[(int64_t)n * DPQ_BLOCK + q] = e;
            a.codes[(int64_t)n * a.K + (a.perm ? a.perm[c0 + q] : c0 + q)] = (uint8_t)uq;
        }
        for (int v = q + 1 + (part + DPQ_LPR - (q + 1) % DPQ_LPR) % DPQ_LPR; v < DPQ_BLOCK; v += DPQ_LPR)   // Eq. 12 inside the block
            wl[v * DPQ_ROWS + lane] = __fsub_rn(wl[v * DPQ_ROWS + lane], __fmul_rn(e, urow[v]));
        __builtin_amdgcn_wave_barrier();
    }
}

// Eq. 12 for the columns right of the block [c0, c0 + 128): work[n, v] <- work[n, v] - err[n, q] * U[c0 + q, v], q = 0..127
// in ascending order.  A workgroup of 256 threads owns a 64 x 64 tile of (rows, columns), a thread 4 x 4 of it.
__global__ void __launch_bounds__(256) dpq_lazy_update_kernel(DpqArgs a, int c0) {
    __shared__ float el[DPQ_BLOCK * 64];                         // el[q * 64 + r]: error q of row r of the tile
    __shared__ float ul[DPQ_BLOCK * 64];                         // ul[q * 64 + c]: U[c0 + q, column c of the tile]
    const int tid = threadIdx.x;
    const int r0 = blockIdx.y * 64, v0 = c0 + DPQ_BLOCK + blockIdx.x * 64;
    for (int idx = tid; idx < DPQ_BLOCK * 64; idx += 256) {
        const int q = idx & (DPQ_BLOCK - 1), r = idx >> 7;       // consecutive threads, consecutive q: coalesced reads of err
        el[q * 64 + r] = (r0 + r < a.N) ? a.err[(int64_t)(r0 + r) * DPQ_BLOCK + q] : 0.0f;
    }
    for (int idx = tid; idx < DPQ_BLOCK * 64; idx += 256) {
        const int c = idx & 63, q = idx >> 6;
        ul[q * 64 + c] = (v0 + c < a.K) ? a.u[(int64_t)(c0 + q) * a.K + v0 + c] : 0.0f;
    }
    __syncthreads();
    const int tr = (tid >> 4) * 4, tc = (tid & 15) * 4;
    float w[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            w[i][j] = (r0 + tr + i < a.N && v0 + tc + j < a.K) ? a.work[(int64_t)(r0 + tr + i) * a.K + v0 + tc + j] : 0.0f;
    for (int q = 0; q < DPQ_BLOCK; ++q) {
        const float4 e = *reinterpret_cast<const float4*>(&el[q * 64 + tr]);
        const float4 u = *reinterpret_cast<const float4*>(&ul[q * 64 + tc]);
        const float ev[4] = {e.x, e.y, e.z, e.w}, uv[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) w[i][j] = __fsub_rn(w[i][j], __fmul_rn(ev[i], uv[j]));
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (r0 + tr + i < a.N && v0 + tc + j < a.K) a.work[(int64_t)(r0 + tr + i) * a.K + v0 + tc + j] = w[i][j];
}

// H += X^T X for one batch of calibration activations X [T, K] (the Hessian of the layer-wise objective, Eq. 5 and
// App. A.2).  A workgroup of 256 threads owns a 64 x 64 tile of H, a thread 4 x 4 of it; 32 tokens at a time are staged
// in LDS for the tile's rows and columns.  float32 accumulation.
template <typename InT>
__global__ void __launch_bounds__(256) hessian_accumulate_kernel(const InT* __restrict__ x, int64_t T, int64_t K, int64_t ldx,
                                                                 float* __restrict__ h) {
    __shared__ float xi[32 * 64], xj[32 * 64];                   // xi[t * 64 + r]: token t, feature i0 + r
    const int tid = threadIdx.x;
    const int64_t i0 = (int64_t)blockIdx.y * 64, j0 = (int64_t)blockIdx.x * 64;
    const int tr = (tid >> 4) * 4, tc = (tid & 15) * 4;
    float acc[4][4] = {};
    for (int64_t t0 = 0; t0 < T; t0 += 32) {
        for (int idx = tid; idx < 32 * 64; idx += 256) {
            const int c = idx & 63, t = idx >> 6;                // consecutive threads, consecutive features: coalesced
            const bool row_ok = t0 + t < T;
            float a = 0.0f, b = 0.0f;
            if (row_ok && i0 + c < K) a = load_as_float(x + (t0 + t) * ldx + i0 + c);
            if (row_ok && j0 + c < K) b = load_as_float(x + (t0 + t) * ldx + j0 + c);
            xi[idx] = a;
            xj[idx] = b;
        }
        __syncthreads();
#pragma unroll 8
        for (int t = 0; t < 32; ++t) {
            const float4 a = *reinterpret_cast<const float4*>(&xi[t * 64 + tr]);
            const float4 b = *reinterpret_cast<const float4*>(&xj[t * 64 + tc]);
            const float av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (i0 + tr + i < K && j0 + tc + j < K) h[(i0 + tr + i) * K + j0 + tc + j] += acc[i][j];
}

}  // namespace

int launch_hessian_accumulate(const void* x, w4a8_dtype dt, int64_t T, int64_t K, int64_t ldx, float* h, hipStream_t st) {
    const dim3 grid((unsigned)((K + 63) / 64), (unsigned)((K + 63) / 64));
    if (dt == W4A8_F32)
        hipLaunchKernelGGL(hessian_accumulate_kernel<float>, grid, dim3(256), 0, st, static_cast<const float*>(x), T, K, ldx, h);
    else
        hipLaunchKernelGGL(hessian_accumulate_kernel<uint16_t>, grid, dim3(256), 0, st, static_cast<const uint16_t*>(x), T, K,
                           ldx, h);
    return launch_status();
}

int launch_gar_permutation(const float* hdiag, int64_t K, int32_t G, int32_t* perm, hipStream_t st) {
    hipLaunchKernelGGL(gar_permutation_kernel, dim3((unsigned)((K + 255) / 256)), dim3(256), 0, st, hdiag, (int)K, (int)G, perm);
    return launch_status();
}

int launch_dpq_calibrate(const float* w, const float* u, const float* s_w, int per_channel, const int32_t* perm,
                         int64_t N, int64_t K, int32_t G, uint8_t* codes, float* scales, uint8_t* zeros, void* workspace,
                         int mse_grid, float mse_max_shrink, hipStream_t st) {
    DpqArgs a;
    a.mse_grid = mse_grid;
    a.shrink_step = mse_grid > 1 ? mse_max_shrink / (float)mse_grid : 0.0f;
    a.work = static_cast<float*>(workspace);
    a.err = a.work + N * K;
    a.u = u; a.s_w = s_w; a.per_channel = per_channel; a.perm = perm;
    a.N = (int)N; a.K = (int)K; a.G = (int)G;
    a.codes = codes; a.scales = scales; a.zeros = zeros;
    hipLaunchKernelGGL(dpq_gather_kernel, dim3((unsigned)((N * K + 255) / 256)), dim3(256), 0, st, w, perm, N, K, a.work);
    if (int e = launch_status()) return e;
    const int lpr = N <= 8192 ? 32 : N <= 16384 ? 16 : 8;        // lanes per row: about a quarter to half of the chip's lanes
    const int threads = lpr == 8 ? 128 : 256;
    const int rows_per_wg = threads / lpr;
    const unsigned row_groups = (unsigned)((N + rows_per_wg - 1) / rows_per_wg);
    for (int c0 = 0; c0 < K; c0 += DPQ_BLOCK) {
        if (lpr == 32)
            hipLaunchKernelGGL((dpq_block_kernel<32, true, 256>), dim3(row_groups), dim3(256), 0, st, a, c0);
        else if (lpr == 16)
            hipLaunchKernelGGL((dpq_block_kernel<16, true, 256>), dim3(row_groups), dim3(256), 0, st, a, c0);
        else
            hipLaunchKernelGGL((dpq_block_kernel<8, false, 128>), dim3(row_groups), dim3(128), 0, st, a, c0);
        if (int e = launch_status()) return e;
        const int64_t rest = K - c0 - DPQ_BLOCK;
        if (rest > 0) {
            hipLaunchKernelGGL(dpq_lazy_update_kernel, dim3((unsigned)((rest + 63) / 64), (unsigned)((N + 63) / 64)), dim3(256),
                               0, st, a, c0);
            if (int e = launch_status()) return e;
        }
    }
    return W4A8_OK;
}

}  // namespace w4a8
