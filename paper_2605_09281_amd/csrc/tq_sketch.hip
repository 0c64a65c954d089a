// Offline helper: rank-r approximation of a dense fp32 matrix by r Gaussian-sketch rank-1 deflations (Section 3.1,
// "Plug-in", Eq. 13), the replacement for the SVD of the tiled matrix W_big of Eq. 11.  Per rank, with sketch vector s:
//   Q = (W W^T)^it W s,   U = Q / |Q|,   Sigma = |Q^T W| / |Q|,   V = Q^T W / |Q^T W|,   W <- W - U Sigma V.
// Everything is a matrix-vector product or a rank-1 update over a matrix that does not fit any cache, so every kernel
// is a coalesced stream over W (HBM-bound): products along the rows by one wave per row, products along the columns
// by column strips with the rows cut into slabs (partial sums added in a fixed order), and the deflation fused into the
// first product of the next rank, so that a rank costs 2 it + 2 reads and one write of W.
// Q is renormalised after every power iteration (U, Sigma and V do not depend on the length of Q; the raw powers leave
// the fp32 range after a few iterations).  All sums have a fixed order: results are run-to-run identical.
#include "tq_common.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
// the matrix is read once per pass and fits no cache: the non-temporal hint on those loads is worth 8 % (measured)

__device__ inline float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

// y[i] = sum_j W'[i][j] x[j] with W' = W - u p^T written back when UPDATE.  One wave per row, four rows per workgroup
// and grid step.
template <bool UPDATE>
__global__ void __launch_bounds__(256) sk_rows_kernel(float* __restrict__ W, int64_t rows, int64_t cols,
                                                      const float* __restrict__ x, const float* __restrict__ u,
                                                      const float* __restrict__ p, float* __restrict__ y)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int64_t row = (int64_t)blockIdx.x * 4 + wave; row < rows; row += (int64_t)gridDim.x * 4) {
        float* wr = W + row * cols;
        const float ui = UPDATE ? u[row] : 0.f;
        float acc = 0.f;
        for (int64_t j = (int64_t)lane * 4; j < cols; j += 256) {
            // the update pass writes the row back in place, so it loads normally
            f32x4 w4 = UPDATE ? *reinterpret_cast<const f32x4*>(wr + j)
                              : __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(wr + j));
            if (UPDATE) {
                const f32x4 p4 = *reinterpret_cast<const f32x4*>(p + j);
                w4 -= ui * p4;
                *reinterpret_cast<f32x4*>(wr + j) = w4;
            }
            if (x) {
                const f32x4 x4 = *reinterpret_cast<const f32x4*>(x + j);
                acc = fmaf(w4[0], x4[0], acc); acc = fmaf(w4[1], x4[1], acc);
                acc = fmaf(w4[2], x4[2], acc); acc = fmaf(w4[3], x4[3], acc);
            }
        }
        acc = wave_sum(acc);
        if (lane == 0 && y) y[row] = acc;
    }
}

// partial[slab][j] = sum over the rows of the slab of W[i][j] q[i] * inv, inv = 1 / *norm (0 if the norm is 0) when a
// norm is given.  One thread per four columns; a row of a strip is one contiguous 4 KB read.
__global__ void __launch_bounds__(256) sk_cols_kernel(const float* __restrict__ W, int64_t rows, int64_t cols,
                                                      const float* __restrict__ q, const float* __restrict__ norm,
                                                      int64_t rows_per_slab, float* __restrict__ partial)
{
    const int64_t j = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    const int64_t r0 = (int64_t)blockIdx.y * rows_per_slab;
    const int64_t r1 = r0 + rows_per_slab < rows ? r0 + rows_per_slab : rows;
    float inv = 1.f;
    if (norm) { const float n = *norm; inv = n > 0.f ? 1.f / n : 0.f; }
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    if (j < cols) {
        for (int64_t i = r0; i < r1; ++i) {
            const f32x4 w4 = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(W + i * cols + j));
            const float qi = q[i] * inv;
            acc += qi * w4;
        }
        *reinterpret_cast<f32x4*>(partial + (int64_t)blockIdx.y * cols + j) = acc;
    }
}

__global__ void __launch_bounds__(256) sk_colsum_kernel(const float* __restrict__ partial, int slabs, int64_t cols,
                                                        float* __restrict__ z)
{
    const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= cols) return;
    float acc = 0.f;
    int s = 0;
    for (; s + 8 <= slabs; s += 8) {       // eight loads in flight, added in slab order
        float v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = partial[(int64_t)(s + i) * cols + j];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc += v[i];
    }
    for (; s < slabs; ++s) acc += partial[(int64_t)s * cols + j];
    z[j] = acc;
}

// *out = |v| (one workgroup: per-thread strided sums in fp32, then a tree in LDS; fixed order)
__global__ void __launch_bounds__(1024) sk_norm_kernel(const float* __restrict__ v, int64_t n, float* __restrict__ out)
{
    __shared__ float red[1024];
    float acc = 0.f;
    for (int64_t i = threadIdx.x; i < n; i += 1024) acc = fmaf(v[i], v[i], acc);
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int s = 512; s >= 1; s >>= 1) {
        if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) *out = sqrtf(red[0]);
}

// out[i] = v[i] / *norm (zeros if the norm is zero: the matrix has run out of rank); sigma_out = *norm * sigma_scale
__global__ void __launch_bounds__(256) sk_scale_kernel(const float* __restrict__ v, int64_t n, const float* __restrict__ norm,
                                                       float* __restrict__ out, float* __restrict__ sigma_out)
{
    const float nv = *norm;
    const float inv = nv > 0.f ? 1.f / nv : 0.f;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) out[i] = v[i] * inv;
    if (sigma_out && i == 0) *sigma_out = nv;
}

struct SketchPlan {
    int slabs;
    int64_t rows_per_slab;
    size_t q, z, p, partial, norms, total;
};

bool make_plan(int64_t rows, int64_t cols, SketchPlan* P)
{
    if (rows < 1 || cols < 4 || (cols & 3) || rows > (int64_t)1 << 24 || cols > (int64_t)1 << 24) return false;
    const int64_t strips = (cols / 4 + 255) / 256;
    int64_t slabs = (1024 + strips - 1) / strips;          // about 1024 workgroups per product along the columns
    if (slabs > rows) slabs = rows;
    if (slabs > 1024) slabs = 1024;
    if (slabs < 1) slabs = 1;
    P->rows_per_slab = (rows + slabs - 1) / slabs;
    P->slabs = (int)((rows + P->rows_per_slab - 1) / P->rows_per_slab);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += tq_align256(bytes); return o; };
    P->q = take((size_t)rows * 4);
    P->z = take((size_t)cols * 4);
    P->p = take((size_t)cols * 4);
    P->partial = take((size_t)P->slabs * cols * 4);
    P->norms = take(256);
    P->total = off;
    return true;
}

}  // namespace

extern "C" size_t tq_sketch_workspace_size(int64_t rows, int64_t cols)
{
    SketchPlan P;
    return make_plan(rows, cols, &P) ? P.total : 0;
}

extern "C" tq_status tq_sketch_lowrank(float* W, int64_t rows, int64_t cols, int32_t r, int32_t it, const float* sketch,
                                       float* U, float* sigma, float* V, void* workspace, size_t workspace_bytes,
                                       void* stream)
{
    if (!W || !sketch || !U || !sigma || !V || !workspace) return TQ_ERR_NULL;
    SketchPlan P;
    if (!make_plan(rows, cols, &P) || r < 1 || r > 4096 || it < 0 || it > 64) return TQ_ERR_SHAPE;
    if (((uintptr_t)W | (uintptr_t)sketch | (uintptr_t)V | (uintptr_t)workspace) & 15) return TQ_ERR_ALIGN;
    if (((uintptr_t)U | (uintptr_t)sigma) & 3) return TQ_ERR_ALIGN;
    if (workspace_bytes < P.total) return TQ_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    uint8_t* ws = (uint8_t*)workspace;
    float* q = (float*)(ws + P.q);
    float* z = (float*)(ws + P.z);
    float* p = (float*)(ws + P.p);
    float* partial = (float*)(ws + P.partial);
    float* norms = (float*)(ws + P.norms);        // [0] |q|, [1] |p|
    const unsigned row_blocks = (unsigned)((rows + 3) / 4 < 8192 ? (rows + 3) / 4 : 8192);
    const dim3 col_grid((unsigned)((cols / 4 + 255) / 256), (unsigned)P.slabs);
    const unsigned col_blocks = (unsigned)((cols + 255) / 256), rowv_blocks = (unsigned)((rows + 255) / 256);
    auto cols_product = [&](const float* vec, const float* norm, float* out) {      // out = W^T (vec / norm)
        hipLaunchKernelGGL(sk_cols_kernel, col_grid, dim3(256), 0, st, (const float*)W, rows, cols, vec, norm, P.rows_per_slab,
                           partial);
        hipLaunchKernelGGL(sk_colsum_kernel, dim3(col_blocks), dim3(256), 0, st, (const float*)partial, P.slabs, cols, out);
    };
    for (int rho = 0; rho < r; ++rho) {
        const float* s = sketch + (size_t)rho * cols;
        // Q = W s, with the previous rank's deflation W -= u p^T applied on the way
        if (rho == 0)
            hipLaunchKernelGGL(sk_rows_kernel<false>, dim3(row_blocks), dim3(256), 0, st, W, rows, cols, s, (const float*)nullptr,
                               (const float*)nullptr, q);
        else
            hipLaunchKernelGGL(sk_rows_kernel<true>, dim3(row_blocks), dim3(256), 0, st, W, rows, cols, s,
                               (const float*)(U + (size_t)(rho - 1) * rows), (const float*)p, q);
        for (int i = 0; i < it; ++i) {       // Q <- W W^T Q / |Q|
            hipLaunchKernelGGL(sk_norm_kernel, dim3(1), dim3(1024), 0, st, (const float*)q, rows, norms);
            cols_product(q, norms, z);
            hipLaunchKernelGGL(sk_rows_kernel<false>, dim3(row_blocks), dim3(256), 0, st, W, rows, cols, (const float*)z,
                               (const float*)nullptr, (const float*)nullptr, q);
        }
        float* u = U + (size_t)rho * rows;
        hipLaunchKernelGGL(sk_norm_kernel, dim3(1), dim3(1024), 0, st, (const float*)q, rows, norms);
        hipLaunchKernelGGL(sk_scale_kernel, dim3(rowv_blocks), dim3(256), 0, st, (const float*)q, rows, (const float*)norms, u,
                           (float*)nullptr);
        // p = W^T U = Sigma V
        cols_product(u, nullptr, p);
        hipLaunchKernelGGL(sk_norm_kernel, dim3(1), dim3(1024), 0, st, (const float*)p, cols, norms + 1);
        hipLaunchKernelGGL(sk_scale_kernel, dim3(col_blocks), dim3(256), 0, st, (const float*)p, cols, (const float*)(norms + 1),
                           V + (size_t)rho * cols, sigma + rho);
        TQ_CHECK_LAUNCH();
    }
    // the last deflation: W holds the residual on return
    hipLaunchKernelGGL(sk_rows_kernel<true>, dim3(row_blocks), dim3(256), 0, st, W, rows, cols, (const float*)nullptr,
                       (const float*)(U + (size_t)(r - 1) * rows), (const float*)p, (float*)nullptr);
    TQ_CHECK_LAUNCH();
    return TQ_OK;
}
