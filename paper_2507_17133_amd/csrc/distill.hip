// United-expert distillation (the paper's section "United Expert Model"): the student FFN of one group is
// fitted to the group's teacher FFNs on calibration tokens by minimising the section's MSE equation
//   L = (1/k) sum_i || H_u - H_o^i ||^2   (summed over features, averaged over tokens)
// with full-batch Adam.  The paper gives no optimiser, settings or data; this is the reading documented in
// the header.  Off the serving path: plain GEMMs through the 64-row kernel (fp32 results), explicit
// transposes for the contractions over tokens, element-wise kernels for SwiGLU and the update.
//   forward   G = X W1^T, U = X W3^T, A = silu(G) U, Y = A W2^T
//   backward  dY = Y - mean_i Y_i  (the factor 2/n goes into the update), dW2 = dY^T A, dA = dY W2,
//             dG = dA U silu'(G), dU = dA silu(G), dW1 = dG^T X, dW3 = dU^T X
#include "internal.h"

#include <algorithm>

namespace bmoe {

__device__ __forceinline__ float bf_to_f(unsigned short b) { return __uint_as_float(((unsigned)b) << 16); }
__device__ __forceinline__ unsigned short f_to_bf(float f)
{
    unsigned u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (unsigned short)(u >> 16);
}

// out[c][r] = in[r][c] (16-bit elements), R and C multiples of 64
__global__ void __launch_bounds__(256) transpose16_kernel(const unsigned short* __restrict__ in,
                                                          unsigned short* __restrict__ out, int R, int C)
{
    __shared__ unsigned short tile[64][66];
    const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int i = ty; i < 64; i += 4) tile[i][tx] = in[(size_t)(r0 + i) * C + c0 + tx];
    __syncthreads();
    for (int i = ty; i < 64; i += 4) out[(size_t)(c0 + i) * R + r0 + tx] = tile[tx][i];
}

__global__ void __launch_bounds__(256) bf16_to_f32_kernel(const unsigned short* __restrict__ in, float* __restrict__ out,
                                                          size_t n)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) out[i] = bf_to_f(in[i]);
}

__global__ void __launch_bounds__(256) fill_f32_kernel(float* __restrict__ p, size_t n, float v)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = v;
}

// tbar += y / k  (y: FFN output rows in half precision)
__global__ void __launch_bounds__(256) teacher_mean_kernel(const unsigned short* __restrict__ y, float* __restrict__ tbar,
                                                           size_t n, float inv_k)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) tbar[i] += (float)__builtin_bit_cast(_Float16, y[i]) * inv_k;
}

// A = silu(G) * U
__global__ void __launch_bounds__(256) swiglu_fwd_kernel(const float* __restrict__ G, const float* __restrict__ U,
                                                         unsigned short* __restrict__ A, size_t n)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const float g = G[i];
    A[i] = f_to_bf(g / (1.0f + __expf(-g)) * U[i]);
}

// dG = dA U sig(G) (1 + G (1 - sig(G))), dU = dA silu(G)
__global__ void __launch_bounds__(256) swiglu_bwd_kernel(const float* __restrict__ G, const float* __restrict__ U,
                                                         const float* __restrict__ dA, unsigned short* __restrict__ dG,
                                                         unsigned short* __restrict__ dU, size_t n)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const float g = G[i], u = U[i], da = dA[i];
    const float sg = 1.0f / (1.0f + __expf(-g));
    dG[i] = f_to_bf(da * u * sg * (1.0f + g * (1.0f - sg)));
    dU[i] = f_to_bf(da * g * sg);
}

// dY = Y - tbar (bf16), and hist[0] = offset + scale * sum (Y - tbar)^2: one block, fixed summation order
__global__ void __launch_bounds__(1024) diff_loss_kernel(const float* __restrict__ Y, const float* __restrict__ tbar,
                                                         unsigned short* __restrict__ dY, size_t n, float scale,
                                                         const float* __restrict__ offset, float* __restrict__ hist)
{
    __shared__ double red[16];
    double s = 0.0;
    for (size_t e = threadIdx.x; e < n; e += 1024) {
        const float df = Y[e] - tbar[e];
        if (dY) dY[e] = f_to_bf(df);
        s += (double)df * (double)df;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0 && hist) {
        double t = 0.0;
        for (int w = 0; w < 16; ++w) t += red[w];
        hist[0] = (offset ? offset[0] : 0.0f) + (float)(t * (double)scale);
    }
}

// floor[0] += scale * sum (y - tbar)^2 for one teacher (y in half precision): one block
__global__ void __launch_bounds__(1024) teacher_spread_kernel(const unsigned short* __restrict__ y,
                                                              const float* __restrict__ tbar, size_t n, float scale,
                                                              float* __restrict__ floor_)
{
    __shared__ double red[16];
    double s = 0.0;
    for (size_t e = threadIdx.x; e < n; e += 1024) {
        const float df = (float)__builtin_bit_cast(_Float16, y[e]) - tbar[e];
        s += (double)df * (double)df;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        for (int w = 0; w < 16; ++w) t += red[w];
        floor_[0] += (float)(t * (double)scale);
    }
}

// Adam with bias correction on fp32 master weights; writes the bf16 copy the GEMMs use.
__global__ void __launch_bounds__(256) adam_kernel(float* __restrict__ w, float* __restrict__ m, float* __restrict__ v,
                                                   const float* __restrict__ grad, unsigned short* __restrict__ w_bf16,
                                                   size_t n, float gscale, float lr, float beta1, float beta2, float eps,
                                                   float c1, float c2)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const float g = grad[i] * gscale;
    const float mi = beta1 * m[i] + (1.0f - beta1) * g;
    const float vi = beta2 * v[i] + (1.0f - beta2) * g * g;
    m[i] = mi;
    v[i] = vi;
    const float wi = w[i] - lr * (mi * c1) / (sqrtf(vi * c2) + eps);
    w[i] = wi;
    w_bf16[i] = f_to_bf(wi);
}

static inline int nblk(size_t n) { return (int)((n + 255) / 256); }

struct DistillBufs {
    float *W[3], *M[3], *V[3], *Gd[3];                    // masters, Adam moments, gradients of W1, W3, W2
    bf16_t* w2t;                                          // W2^T
    float *Gf, *Uf, *dAf;                                 // [n][F]
    bf16_t *A, *dG, *dU, *At, *dGt, *dUt;                 // [n][F] and [F][n]
    float *Y, *tbar;                                      // [n][d]
    bf16_t *dY, *dYt, *xt;                                // [n][d], [d][n], [d][n]
    float* floor_;
    int32_t* table;
    size_t total;
};

static DistillBufs carve_distill(void* buf, int n, int d, int F)
{
    const size_t dF = (size_t)d * F, nF = (size_t)n * F, nd = (size_t)n * d;
    char* base = static_cast<char*>(buf);
    size_t o = 0;
    auto take = [&](size_t bytes) { char* p = base + o; o = align_up(o + bytes, 256); return p; };
    DistillBufs B;
    for (int q = 0; q < 3; ++q) B.W[q] = reinterpret_cast<float*>(take(dF * 4));
    for (int q = 0; q < 3; ++q) B.M[q] = reinterpret_cast<float*>(take(dF * 4));
    for (int q = 0; q < 3; ++q) B.V[q] = reinterpret_cast<float*>(take(dF * 4));
    for (int q = 0; q < 3; ++q) B.Gd[q] = reinterpret_cast<float*>(take(dF * 4));
    B.w2t = reinterpret_cast<bf16_t*>(take(dF * 2));
    B.Gf = reinterpret_cast<float*>(take(nF * 4));
    B.Uf = reinterpret_cast<float*>(take(nF * 4));
    B.dAf = reinterpret_cast<float*>(take(nF * 4));
    B.A = reinterpret_cast<bf16_t*>(take(nF * 2));
    B.dG = reinterpret_cast<bf16_t*>(take(nF * 2));
    B.dU = reinterpret_cast<bf16_t*>(take(nF * 2));
    B.At = reinterpret_cast<bf16_t*>(take(nF * 2));
    B.dGt = reinterpret_cast<bf16_t*>(take(nF * 2));
    B.dUt = reinterpret_cast<bf16_t*>(take(nF * 2));
    B.Y = reinterpret_cast<float*>(take(nd * 4));
    B.tbar = reinterpret_cast<float*>(take(nd * 4));
    B.dY = reinterpret_cast<bf16_t*>(take(nd * 2));
    B.dYt = reinterpret_cast<bf16_t*>(take(nd * 2));
    B.xt = reinterpret_cast<bf16_t*>(take(nd * 2));
    B.floor_ = reinterpret_cast<float*>(take(256));
    B.table = reinterpret_cast<int32_t*>(take(16 + 16 * (size_t)(std::max(std::max(n, d), F) / 64 + 1)));
    B.total = o;
    return B;
}

size_t distill_buffer_bytes(int n, int d, int F) { return carve_distill(nullptr, n, d, F).total; }
float* distill_tbar(void* buf, int n, int d, int F) { return carve_distill(buf, n, d, F).tbar; }
float* distill_floor(void* buf, int n, int d, int F) { return carve_distill(buf, n, d, F).floor_; }

// Trains the student (w1u, w3u [F][d], w2u [d][F], bf16, updated in place) of ONE group.  The mean teacher
// output (distill_tbar) and the loss at it (distill_floor) have been prepared by the caller in buf.
hipError_t distill_group(const bf16_t* x, int n, int d, int F, bf16_t* w1u, bf16_t* w3u, bf16_t* w2u, int steps,
                         float lr, float* hist, void* buf, hipStream_t s)
{
    const size_t dF = (size_t)d * F, nF = (size_t)n * F, nd = (size_t)n * d;
    const DistillBufs B = carve_distill(buf, n, d, F);
    float* const* W = B.W; float* const* M = B.M; float* const* V = B.V; float* const* Gd = B.Gd;
    bf16_t* w2t = B.w2t;
    float *Gf = B.Gf, *Uf = B.Uf, *dAf = B.dAf;
    bf16_t *A = B.A, *dG = B.dG, *dU = B.dU, *At = B.At, *dGt = B.dGt, *dUt = B.dUt;
    float* Y = B.Y;
    const float* tbar = B.tbar;
    const float* floor_ = B.floor_;
    bf16_t *dY = B.dY, *dYt = B.dYt, *xt = B.xt;
    int32_t* table = B.table;

    auto us = [](bf16_t* p) { return reinterpret_cast<unsigned short*>(p); };
    auto cus = [](const bf16_t* p) { return reinterpret_cast<const unsigned short*>(p); };
    auto transpose = [&](const bf16_t* in, bf16_t* out, int R, int C) {
        transpose16_kernel<<<dim3(C / 64, R / 64), 256, 0, s>>>(cus(in), us(out), R, C);
    };
    bf16_t* wb[3] = {w1u, w3u, w2u};
    for (int q = 0; q < 3; ++q) {
        bf16_to_f32_kernel<<<nblk(dF), 256, 0, s>>>(cus(wb[q]), W[q], dF);
        fill_f32_kernel<<<nblk(dF), 256, 0, s>>>(M[q], dF, 0.0f);
        fill_f32_kernel<<<nblk(dF), 256, 0, s>>>(V[q], dF, 0.0f);
    }
    transpose(x, xt, n, d);                               // X^T [d][n]
    const float beta1 = 0.9f, beta2 = 0.999f, eps = 1e-8f;
    double b1t = 1.0, b2t = 1.0;
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    for (int t = 0; t <= steps; ++t) {
        // forward
        if ((e = launch_plain_gemm(x, w1u, n, F, d, Gf, table, s)) != hipSuccess) return e;
        if ((e = launch_plain_gemm(x, w3u, n, F, d, Uf, table, s)) != hipSuccess) return e;
        swiglu_fwd_kernel<<<nblk(nF), 256, 0, s>>>(Gf, Uf, us(A), nF);
        if ((e = launch_plain_gemm(A, w2u, n, d, F, Y, table, s)) != hipSuccess) return e;
        diff_loss_kernel<<<1, 1024, 0, s>>>(Y, tbar, t < steps ? us(dY) : nullptr, nd, 1.0f / (float)n, floor_,
                                            hist ? hist + t : nullptr);
        if (t == steps) break;
        // backward
        transpose(dY, dYt, n, d);                         // [d][n]
        transpose(A, At, n, F);                           // [F][n]
        if ((e = launch_plain_gemm(dYt, At, d, F, n, Gd[2], table, s)) != hipSuccess) return e;      // dW2 [d][F]
        transpose(w2u, w2t, d, F);                        // W2^T [F][d]
        if ((e = launch_plain_gemm(dY, w2t, n, F, d, dAf, table, s)) != hipSuccess) return e;        // dA [n][F]
        swiglu_bwd_kernel<<<nblk(nF), 256, 0, s>>>(Gf, Uf, dAf, us(dG), us(dU), nF);
        transpose(dG, dGt, n, F);
        transpose(dU, dUt, n, F);
        if ((e = launch_plain_gemm(dGt, xt, F, d, n, Gd[0], table, s)) != hipSuccess) return e;      // dW1 [F][d]
        if ((e = launch_plain_gemm(dUt, xt, F, d, n, Gd[1], table, s)) != hipSuccess) return e;      // dW3 [F][d]
        // update
        b1t *= beta1;
        b2t *= beta2;
        const float c1 = (float)(1.0 / (1.0 - b1t)), c2 = (float)(1.0 / (1.0 - b2t));
        for (int q = 0; q < 3; ++q)
            adam_kernel<<<nblk(dF), 256, 0, s>>>(W[q], M[q], V[q], Gd[q], us(wb[q]), dF, 2.0f / (float)n, lr, beta1, beta2,
                                                 eps, c1, c2);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    return hipGetLastError();
}

hipError_t launch_teacher_mean(const bf16_t* y_half, float* tbar, size_t n, float inv_k, hipStream_t s)
{
    teacher_mean_kernel<<<nblk(n), 256, 0, s>>>(reinterpret_cast<const unsigned short*>(y_half), tbar, n, inv_k);
    return hipGetLastError();
}

hipError_t launch_teacher_spread(const bf16_t* y_half, const float* tbar, size_t n, float scale, float* floor_,
                                 hipStream_t s)
{
    teacher_spread_kernel<<<1, 1024, 0, s>>>(reinterpret_cast<const unsigned short*>(y_half), tbar, n, scale, floor_);
    return hipGetLastError();
}

hipError_t launch_fill_f32(float* p, size_t n, float v, hipStream_t s)
{
    fill_f32_kernel<<<nblk(n), 256, 0, s>>>(p, n, v);
    return hipGetLastError();
}

}  // namespace bmoe
