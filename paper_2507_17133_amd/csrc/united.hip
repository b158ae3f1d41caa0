// United experts (United Expert Model): parameter mean of each group of `way` consecutive experts,
// and helpers to evaluate the distillation loss of that section on calibration tokens.
#include "internal.h"

#include <algorithm>

namespace bmoe {

// Round a double to bf16 (8 significant bits), to nearest, ties to even, in one step.
__device__ __forceinline__ unsigned short f64_to_bf16_bits(double v)
{
    const float f = (float)v;                       // nearest float
    unsigned int u = __float_as_uint(f);
    const unsigned int low = u & 0xFFFFu;
    unsigned int up = 0;
    if (low > 0x8000u) up = 1;
    else if (low == 0x8000u) {
        // f sits on a bf16 midpoint; the double may lie to either side of it
        const double rest = fabs(v) - fabs((double)f);
        if (rest > 0.0) up = 1;
        else if (rest < 0.0) up = 0;
        else up = (u >> 16) & 1u;
    }
    return (unsigned short)((u >> 16) + up);
}

__global__ void __launch_bounds__(256) united_mean_kernel(const unsigned short* __restrict__ w, int m, int way,
                                                          size_t n_elem, unsigned short* __restrict__ u)
{
    const int g = blockIdx.y;
    const int lo = g * way, hi = min(m, lo + way);
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < n_elem; e += (size_t)gridDim.x * 256) {
        double s = 0.0;
        for (int i = lo; i < hi; ++i) s += (double)__uint_as_float(((unsigned int)w[(size_t)i * n_elem + e]) << 16);
        u[(size_t)g * n_elem + e] = f64_to_bf16_bits(s / (double)(hi - lo));
    }
}

hipError_t launch_united_mean(const bf16_t* w, int m, int way, size_t n_elem, bf16_t* u, hipStream_t s)
{
    const int G = ceil_div(m, way);
    const int bx = (int)std::min<size_t>((n_elem + 255) / 256, 4096);
    united_mean_kernel<<<dim3(bx, G), 256, 0, s>>>(reinterpret_cast<const unsigned short*>(w), m, way, n_elem,
                                                   reinterpret_cast<unsigned short*>(u));
    return hipGetLastError();
}

// Row tables of a single unit u holding rows 0..n-1 (identity gather), weights 1.
__global__ void __launch_bounds__(256) single_unit_kernel(int32_t* unit_cnt, int32_t* unit_off, int U, int u, int n,
                                                          float* ones)
{
    const int gid = blockIdx.x * 256 + threadIdx.x;
    if (gid < U) unit_cnt[gid] = gid == u ? n : 0;
    if (gid <= U) unit_off[gid] = gid <= u ? 0 : n;
    if (ones && gid < n) ones[gid] = 1.0f;
}

hipError_t launch_single_unit(int32_t* unit_cnt, int32_t* unit_off, int U, int u, int n, float* ones, hipStream_t s)
{
    const int span = std::max(U + 1, n);
    single_unit_kernel<<<ceil_div(span, 256), 256, 0, s>>>(unit_cnt, unit_off, U, u, n, ones);
    return hipGetLastError();
}

__global__ void zero_f32_kernel(float* p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0.0f;
}
hipError_t launch_zero_f32(float* p, int n, hipStream_t s)
{
    zero_f32_kernel<<<ceil_div(n, 256), 256, 0, s>>>(p, n);
    return hipGetLastError();
}

__global__ void __launch_bounds__(1024) sqdiff_kernel(const unsigned short* __restrict__ a,
                                                      const unsigned short* __restrict__ b, size_t n, float scale,
                                                      float* loss_g)
{
    __shared__ double red[16];
    double s = 0.0;
    for (size_t e = threadIdx.x; e < n; e += 1024) {
        // FFN output rows are stored in half precision
        const float df = (float)__builtin_bit_cast(_Float16, a[e]) - (float)__builtin_bit_cast(_Float16, b[e]);
        s += (double)df * (double)df;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        for (int w = 0; w < 16; ++w) t += red[w];
        loss_g[0] += (float)(t * (double)scale);
    }
}

hipError_t launch_sqdiff_accumulate(const bf16_t* a, const bf16_t* b, size_t n, float scale, float* loss_g, hipStream_t s)
{
    sqdiff_kernel<<<1, 1024, 0, s>>>(reinterpret_cast<const unsigned short*>(a),
                                     reinterpret_cast<const unsigned short*>(b), n, scale, loss_g);
    return hipGetLastError();
}

}  // namespace bmoe
