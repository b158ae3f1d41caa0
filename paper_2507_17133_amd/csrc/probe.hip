// Measurement aids, not part of the layer: what this GPU sustains on the two resources the layer's kernels
// are priced against, measured the same way on the same box.
//   MFMA: a loop of independent v_mfma_f32_16x16x32_bf16 on register operands (no memory traffic at all),
//         eight waves per CU.  With realistic (random) operand bits the chip is power limited well below its
//         nominal peak; with constant operands it is not.  The operands come from the caller.
//   HBM:  every thread adds up 16-byte loads of a caller's buffer, grid-stride.
// Both time a batch of launches with HIP events on the caller's stream and wait for it (host synchronisation:
// these are probes, not hot-path calls).
#include "internal.h"

namespace bmoe {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kProbeBlocks = 256 * 4;           // four blocks of 512 threads per CU would fit; two run at a time
constexpr int kProbeThreads = 512;

__global__ void __launch_bounds__(kProbeThreads) probe_mfma_kernel(const bf16x8* __restrict__ in, float* __restrict__ out,
                                                                  int iters)
{
    bf16x8 a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i] = in[(threadIdx.x * 8 + i) & 4095];
        b[i] = in[(threadIdx.x * 8 + 4 + i) & 4095];
    }
    f32x4 acc[8][4];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b[j], a[i & 3], acc[i][j], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) s += acc[i][j][0] + acc[i][j][1] + acc[i][j][2] + acc[i][j][3];
    out[(size_t)blockIdx.x * kProbeThreads + threadIdx.x] = s;
}

__global__ void __launch_bounds__(256) probe_read_kernel(const uint4* __restrict__ p, size_t n, unsigned* __restrict__ out)
{
    unsigned acc = 0;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        const uint4 v = p[i];
        acc += v.x ^ v.y ^ v.z ^ v.w;
    }
    if (acc == 0x9E3779B9u) out[0] = acc;       // keeps the loads alive; practically never true
}

// Runs `launch` until about `warm_ms` have passed (clocks settle under load), then times `reps` launches.
template <class F>
static hipError_t time_launches(F launch, hipStream_t s, double warm_ms, int reps, double* ms_per_launch)
{
    hipEvent_t a = nullptr, b = nullptr;
    hipError_t e = hipEventCreate(&a);
    if (e != hipSuccess) return e;
    e = hipEventCreate(&b);
    if (e != hipSuccess) { (void)hipEventDestroy(a); return e; }
    auto done = [&](hipError_t r) { (void)hipEventDestroy(a); (void)hipEventDestroy(b); return r; };
    float ms = 0.f;
    // one launch, timed, tells how many make up the warm-up
    if ((e = hipEventRecord(a, s)) != hipSuccess) return done(e);
    launch();
    if ((e = hipEventRecord(b, s)) != hipSuccess) return done(e);
    if ((e = hipEventSynchronize(b)) != hipSuccess) return done(e);
    if ((e = hipEventElapsedTime(&ms, a, b)) != hipSuccess) return done(e);
    int n_warm = ms > 0.f ? (int)(warm_ms / ms) : 1;
    n_warm = n_warm < 1 ? 1 : (n_warm > 100000 ? 100000 : n_warm);
    for (int i = 0; i < n_warm; ++i) launch();
    if ((e = hipEventRecord(a, s)) != hipSuccess) return done(e);
    for (int i = 0; i < reps; ++i) launch();
    if ((e = hipEventRecord(b, s)) != hipSuccess) return done(e);
    if ((e = hipEventSynchronize(b)) != hipSuccess) return done(e);
    if ((e = hipEventElapsedTime(&ms, a, b)) != hipSuccess) return done(e);
    if ((e = hipGetLastError()) != hipSuccess) return done(e);
    *ms_per_launch = (double)ms / reps;
    return done(hipSuccess);
}

hipError_t probe_mfma(const void* operands, void* sink, hipStream_t s, double* tflops)
{
    const int iters = 2048;
    double ms = 0.0;
    hipError_t e = time_launches(
        [&]() {
            probe_mfma_kernel<<<kProbeBlocks, kProbeThreads, 0, s>>>(static_cast<const bf16x8*>(operands),
                                                                    static_cast<float*>(sink), iters);
        },
        s, 300.0, 20, &ms);
    if (e != hipSuccess) return e;
    const double flops = (double)kProbeBlocks * (kProbeThreads / 64) * 32.0 * 16384.0 * iters;   // 32 MFMAs of 16x16x32x2
    *tflops = flops / (ms * 1e-3) / 1e12;
    return hipSuccess;
}

hipError_t probe_hbm_read(const void* buf, size_t bytes, void* sink, hipStream_t s, double* gbs)
{
    const size_t n = bytes / 16;
    double ms = 0.0;
    hipError_t e = time_launches(
        [&]() { probe_read_kernel<<<2048, 256, 0, s>>>(static_cast<const uint4*>(buf), n, static_cast<unsigned*>(sink)); },
        s, 100.0, 10, &ms);
    if (e != hipSuccess) return e;
    *gbs = (double)(n * 16) / (ms * 1e-3) / 1e9;
    return hipSuccess;
}

}  // namespace bmoe
