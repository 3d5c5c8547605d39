// Iterative reconstruction on top of the matched projector pair: SIRT and steepest descent on the least-squares
// cost ("CT Projection Models and Geometries": the cost 1/2 ||A x - y||^2 and its gradient A^T (A x - y); the matched
// pair is what keeps such iterations stable over a thousand or more steps).  Everything between the projector calls
// is a streaming elementwise kernel or a reduction on the caller's stream; nothing synchronises with the host and
// nothing is allocated: the caller passes the workspace.
#include <hip/hip_runtime.h>

#include "leap_internal.h"

namespace {

constexpr int RB = 256;            // threads per block of the streaming kernels
constexpr int RED_BLOCKS = 1024;   // partial sums of a reduction

inline unsigned blocks_for(size_t n)
{
    const size_t b = (n + (size_t)RB * 4 - 1) / ((size_t)RB * 4);
    return (unsigned)(b < 1 ? 1 : (b > 65535u * 16u ? 65535u * 16u : b));
}

__global__ __launch_bounds__(RB) void k_fill(float *__restrict__ p, float v, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * RB + threadIdx.x; i < n; i += (size_t)gridDim.x * RB) p[i] = v;
}

// p <- 1/p where p > 0, else 0 (rays that miss the volume, voxels no ray sees)
__global__ __launch_bounds__(RB) void k_safe_reciprocal(float *__restrict__ p, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * RB + threadIdx.x; i < n; i += (size_t)gridDim.x * RB) {
        const float v = p[i];
        p[i] = v > 0.0f ? 1.0f / v : 0.0f;
    }
}

// out <- w * (y - ax)   (w may be null: out <- ax - y, the least-squares residual); out may be ax itself
__global__ __launch_bounds__(RB) void k_residual(const float *__restrict__ y, const float *ax, const float *__restrict__ w,
                                                 float *out, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * RB + threadIdx.x; i < n; i += (size_t)gridDim.x * RB)
        out[i] = w ? w[i] * (y[i] - ax[i]) : ax[i] - y[i];
}

// x <- x + scale * c * g  (c may be null), clipped at zero from below when nonneg; scale = relax, or -(*alpha) when alpha
// is given (a step length computed on the device)
__global__ __launch_bounds__(RB) void k_update(float *__restrict__ x, const float *__restrict__ g, const float *__restrict__ c,
                                               float relax, const float *__restrict__ alpha, int nonneg, size_t n)
{
    const float s = alpha ? -alpha[0] : relax;
    for (size_t i = (size_t)blockIdx.x * RB + threadIdx.x; i < n; i += (size_t)gridDim.x * RB) {
        float v = fmaf(s * (c ? c[i] : 1.0f), g[i], x[i]);
        x[i] = (nonneg && v < 0.0f) ? 0.0f : v;
    }
}

// partial[b] <- sum over block b's share of p[i]^2, in double
__global__ __launch_bounds__(RB) void k_sumsq_partial(const float *__restrict__ p, size_t n, double *__restrict__ partial)
{
    __shared__ double sh[RB];
    double acc = 0.0;
    for (size_t i = (size_t)blockIdx.x * RB + threadIdx.x; i < n; i += (size_t)gridDim.x * RB) acc += (double)p[i] * (double)p[i];
    sh[threadIdx.x] = acc;
    __syncthreads();
    for (int s = RB / 2; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) sh[threadIdx.x] += sh[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) partial[blockIdx.x] = sh[0];
}

// alpha <- (sum of num partials) / (sum of den partials), 0 when the denominator vanishes; one block
__global__ __launch_bounds__(RB) void k_step_length(const double *__restrict__ num, const double *__restrict__ den, int nb,
                                                    float *__restrict__ alpha)
{
    __shared__ double a[RB], b[RB];
    double sa = 0.0, sb = 0.0;
    for (int i = threadIdx.x; i < nb; i += RB) { sa += num[i]; sb += den[i]; }
    a[threadIdx.x] = sa; b[threadIdx.x] = sb;
    __syncthreads();
    for (int s = RB / 2; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) { a[threadIdx.x] += a[threadIdx.x + s]; b[threadIdx.x] += b[threadIdx.x + s]; }
        __syncthreads();
    }
    if (threadIdx.x == 0) alpha[0] = b[0] > 0.0 ? (float)(a[0] / b[0]) : 0.0f;
}

int check(const leap_geometry *G, const void *y, const void *x, const void *work, int iterations)
{
    if (!G || !y || !x || !work) {
        leap_set_error("null handle, data or workspace pointer");
        return LEAP_INVALID_ARG;
    }
    if (iterations < 0) {
        leap_set_error("iterations must not be negative");
        return LEAP_INVALID_ARG;
    }
    return LEAP_OK;
}

}  // namespace

extern "C" int leap_recon_workspace_floats(const leap_geometry *G, int64_t *n_floats)
{
    if (!G || !n_floats) {
        leap_set_error("null handle or output pointer");
        return LEAP_INVALID_ARG;
    }
    const int64_t nvol = (int64_t)G->g.nx * G->g.ny * G->g.nz, nsino = (int64_t)G->g.nviews * G->g.nrows * G->g.ncols;
    *n_floats = 2 * nsino + 2 * nvol + 4 * RED_BLOCKS + 64;      // two sinograms, two volumes, 2 x 1024 doubles, alpha
    return LEAP_OK;
}

extern "C" int leap_sirt(const leap_geometry *G, const float *d_sino, float *d_vol, float *d_work, int32_t iterations,
                         float relaxation, int32_t nonneg, void *hip_stream)
{
    int rc = check(G, d_sino, d_vol, d_work, iterations);
    if (rc != LEAP_OK) return rc;
    hipStream_t st = (hipStream_t)hip_stream;
    const size_t nvol = (size_t)G->g.nx * G->g.ny * G->g.nz, nsino = (size_t)G->g.nviews * G->g.nrows * G->g.ncols;
    float *row_w = d_work, *resid = d_work + nsino, *col_w = d_work + 2 * nsino, *grad = col_w + nvol;
    // R = 1 / (A 1), C = 1 / (A^T 1)
    hipLaunchKernelGGL(k_fill, dim3(blocks_for(nvol)), dim3(RB), 0, st, grad, 1.0f, nvol);
    if ((rc = leap_project(G, grad, row_w, 1, hip_stream)) != LEAP_OK) return rc;
    hipLaunchKernelGGL(k_fill, dim3(blocks_for(nsino)), dim3(RB), 0, st, resid, 1.0f, nsino);
    if ((rc = leap_backproject(G, resid, col_w, 1, hip_stream)) != LEAP_OK) return rc;
    hipLaunchKernelGGL(k_safe_reciprocal, dim3(blocks_for(nsino)), dim3(RB), 0, st, row_w, nsino);
    hipLaunchKernelGGL(k_safe_reciprocal, dim3(blocks_for(nvol)), dim3(RB), 0, st, col_w, nvol);
    for (int it = 0; it < iterations; ++it) {
        if ((rc = leap_project(G, d_vol, resid, 1, hip_stream)) != LEAP_OK) return rc;                 // resid <- A x
        hipLaunchKernelGGL(k_residual, dim3(blocks_for(nsino)), dim3(RB), 0, st, d_sino, resid, row_w, resid, nsino);
        if ((rc = leap_backproject(G, resid, grad, 1, hip_stream)) != LEAP_OK) return rc;              // grad <- A^T R (y - A x)
        hipLaunchKernelGGL(k_update, dim3(blocks_for(nvol)), dim3(RB), 0, st, d_vol, grad, col_w, relaxation,
                           (const float *)nullptr, nonneg, nvol);
    }
    LEAP_HIP_CHECK(hipGetLastError());
    return LEAP_OK;
}

extern "C" int leap_least_squares_descent(const leap_geometry *G, const float *d_sino, float *d_vol, float *d_work,
                                          int32_t iterations, void *hip_stream)
{
    int rc = check(G, d_sino, d_vol, d_work, iterations);
    if (rc != LEAP_OK) return rc;
    hipStream_t st = (hipStream_t)hip_stream;
    const size_t nvol = (size_t)G->g.nx * G->g.ny * G->g.nz, nsino = (size_t)G->g.nviews * G->g.nrows * G->g.ncols;
    float *resid = d_work, *q = d_work + nsino, *grad = d_work + 2 * nsino;
    // the reduction scratch sits behind the two sinograms and two volumes, 8-byte aligned
    uintptr_t tail = (uintptr_t)(d_work + 2 * nsino + 2 * nvol);
    tail = (tail + 7u) & ~(uintptr_t)7u;
    double *num = (double *)tail, *den = num + RED_BLOCKS;
    float *alpha = (float *)(den + RED_BLOCKS);
    for (int it = 0; it < iterations; ++it) {
        if ((rc = leap_project(G, d_vol, resid, 1, hip_stream)) != LEAP_OK) return rc;                 // A x
        hipLaunchKernelGGL(k_residual, dim3(blocks_for(nsino)), dim3(RB), 0, st, d_sino, resid, (const float *)nullptr, resid,
                           nsino);                                                                  // r = A x - y
        if ((rc = leap_backproject(G, resid, grad, 1, hip_stream)) != LEAP_OK) return rc;              // g = A^T r
        if ((rc = leap_project(G, grad, q, 1, hip_stream)) != LEAP_OK) return rc;                      // q = A g
        hipLaunchKernelGGL(k_sumsq_partial, dim3(RED_BLOCKS), dim3(RB), 0, st, grad, nvol, num);
        hipLaunchKernelGGL(k_sumsq_partial, dim3(RED_BLOCKS), dim3(RB), 0, st, q, nsino, den);
        hipLaunchKernelGGL(k_step_length, dim3(1), dim3(RB), 0, st, num, den, RED_BLOCKS, alpha);      // alpha = |g|^2 / |A g|^2
        hipLaunchKernelGGL(k_update, dim3(blocks_for(nvol)), dim3(RB), 0, st, d_vol, grad, (const float *)nullptr, 0.0f, alpha,
                           0, nvol);                                                                // x <- x - alpha g
    }
    LEAP_HIP_CHECK(hipGetLastError());
    return LEAP_OK;
}
