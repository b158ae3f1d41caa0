// Expert FFNs of the BrownoutMoE layer as two grouped GEMMs on gfx950 MFMA, plus the weighted combine.
//
//   GEMM1  H[r][f] = silu(x_r . W1_u[f]) * (x_r . W3_u[f])      rows r of unit u, gathered from x
//   GEMM2  Y[r][c] = row_weight[r] * (H_r . W2_u[c])
//   combine out_t  = [x_t] + sum over the token's rows of Y      (layer equation, fixed order)
//
// Both operands of both GEMMs are K-contiguous (x [T][d], W1/W3 [F][d], H [R][F], W2 [d][F]), which is
// the natural operand order of v_mfma_f32_32x32x16_bf16: a lane supplies 8 consecutive k of one row.
// A block owns a BM x BN output tile; tiles of 64 k are staged global -> registers -> LDS (16-byte
// chunks, XOR-swizzled so that both the 16-byte stores and the ds_read_b128 fragment loads are
// conflict free), double buffered with one barrier per k tile.  In GEMM1 a block's BN columns are
// BN/2 columns of W1 and the same BN/2 columns of W3, interleaved 32 by 32, so that the gate and up
// values of one (row, f) land in the same lane and SwiGLU is applied in registers.
// Which (unit, rows) an M tile covers comes from a tile table built on the device from the unit
// counts, so skewed expert loads need no host round trip; the grid is an upper bound and surplus
// blocks exit.  Block ids are remapped so that each XCD (block id mod 8) works on a contiguous range
// of tiles and shares weight panels in its own L2.
#include "internal.h"

#include <algorithm>
#include <cstdlib>

namespace bmoe {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ unsigned short f2bf(float f)
{
    unsigned int u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (unsigned short)(u >> 16);
}
__device__ __forceinline__ float bf2f(unsigned short b) { return __uint_as_float(((unsigned int)b) << 16); }

// ------------------------------------------------------------------------------------------------
// Tile table: header {n_mtiles, 0, 0, 0} then one int4 {unit, first row, rows, 0} per M tile, units in
// ascending order, tiles of a unit consecutive.  One block.
// ------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) tile_table_kernel(const int32_t* __restrict__ unit_cnt,
                                                         const int32_t* __restrict__ unit_off, int u_lo, int u_hi,
                                                         int BM, int32_t* __restrict__ table, int cap)
{
    __shared__ int wsum[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n_units = u_hi - u_lo;
    const int per = (n_units + 255) / 256;
    int local = 0;
    for (int q = 0; q < per; ++q) {
        const int u = u_lo + tid * per + q;
        if (u < u_hi) local += (unit_cnt[u] + BM - 1) / BM;
    }
    int incl = local;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int o = __shfl_up(incl, off);
        if (lane >= off) incl += o;
    }
    if (lane == 63) wsum[wave] = incl;
    __syncthreads();
    int base = incl - local;
    for (int w = 0; w < wave; ++w) base += wsum[w];
    int4* entries = reinterpret_cast<int4*>(table + 4);
    for (int q = 0; q < per; ++q) {
        const int u = u_lo + tid * per + q;
        if (u >= u_hi) break;
        const int c = unit_cnt[u], o = unit_off[u];
        for (int r = 0; r < c; r += BM) {
            if (base < cap) entries[base] = make_int4(u, o + r, min(BM, c - r), 0);
            ++base;
        }
    }
    if (tid == 255) {
        table[0] = min(base, cap);
        table[1] = 0; table[2] = 0; table[3] = 0;
    }
}

// ------------------------------------------------------------------------------------------------
struct GemmArgs {
    const bf16_t* A; long lda; const int32_t* gather;
    const int32_t* table;
    const bf16_t *wa0, *wa1, *wa2;              // per weight source (experts, united, shared); GEMM1: W1, GEMM2: W2
    const bf16_t *wb0, *wb1, *wb2;              // GEMM1: W3; GEMM2: unused
    int m, G;
    int N, K;                                   // GEMM1: N = F (columns of W1 and of W3), GEMM2: N = d
    bf16_t* out; long ldo;
    const float* row_weight;
    int n_ntiles;
};

template <int BM, int BN, int WM, int WN, bool SWIGLU>
__global__ void __launch_bounds__(WM * WN * 64) ffn_gemm_kernel(GemmArgs p)
{
    constexpr int NTH = WM * WN * 64;
    constexpr int TM = BM / WM, TN = BN / WN;
    constexpr int FM = TM / 32, FN = TN / 32;
    constexpr int ROWS_PER_PASS = NTH / 8;
    constexpr int A_CH = BM / ROWS_PER_PASS, B_CH = BN / ROWS_PER_PASS;
    constexpr int STAGE = (BM + BN) * 128;
    static_assert(BM % ROWS_PER_PASS == 0 && BN % ROWS_PER_PASS == 0, "loader shape");
    static_assert(!SWIGLU || (FN % 2 == 0), "gate/up tiles must pair inside a wavefront");
    extern __shared__ __attribute__((aligned(16))) char smem[];

    // ---- which tile ----
    const int n_mt = p.table[0];
    const int total = n_mt * p.n_ntiles;
    const int chunk = (total + 7) >> 3;
    const int bi = blockIdx.x >> 3;
    if (bi >= chunk) return;
    const int L = (blockIdx.x & 7) * chunk + bi;
    if (L >= total) return;
    const int nt = L / n_mt, mt = L - nt * n_mt;
    const int4 te = reinterpret_cast<const int4*>(p.table + 4)[mt];
    const int unit = te.x, row0 = te.y, nrows = te.z;
    const int src = unit < p.m ? 0 : (unit < p.m + p.G ? 1 : 2);
    const int widx = unit - (src == 0 ? 0 : (src == 1 ? p.m : p.m + p.G));
    const size_t wsz = (size_t)p.N * p.K;
    const bf16_t* Wa = (src == 0 ? p.wa0 : (src == 1 ? p.wa1 : p.wa2)) + (size_t)widx * wsz;
    const bf16_t* Wb = SWIGLU ? (src == 0 ? p.wb0 : (src == 1 ? p.wb1 : p.wb2)) + (size_t)widx * wsz : nullptr;
    constexpr int BNC = SWIGLU ? BN / 2 : BN;    // output columns per block
    const int n0 = nt * BNC;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;

    // ---- loader: thread moves the 16-byte chunk (tid&7) of rows tid/8 + i*ROWS_PER_PASS ----
    const int lc = tid & 7, lr = tid >> 3;
    const bf16_t* aptr[A_CH];
    const bf16_t* bptr[B_CH];
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
        int r = lr + i * ROWS_PER_PASS;
        r = r < nrows ? r : 0;                                     // ragged tile: re-read row 0, never stored
        const long src_row = p.gather ? (long)p.gather[row0 + r] : (long)(row0 + r);
        aptr[i] = p.A + src_row * p.lda + lc * 8;
    }
#pragma unroll
    for (int i = 0; i < B_CH; ++i) {
        const int n = lr + i * ROWS_PER_PASS;
        int col;
        const bf16_t* W = Wa;
        if (SWIGLU) {
            const int w_n = n / TN, j = (n % TN) >> 5, c = n & 31;
            col = n0 + (w_n * (TN / 64) + (j >> 1)) * 32 + c;
            if (j & 1) W = Wb;
        } else {
            col = n0 + n;
        }
        col = col < p.N ? col : p.N - 1;                           // ragged N: clamp, never stored
        bptr[i] = W + (size_t)col * p.K + lc * 8;
    }
    u32x4 ra[A_CH], rb[B_CH];
    auto gload = [&](int kt) {
        const int ko = kt * 64;
#pragma unroll
        for (int i = 0; i < A_CH; ++i) ra[i] = *reinterpret_cast<const u32x4*>(aptr[i] + ko);
#pragma unroll
        for (int i = 0; i < B_CH; ++i) rb[i] = *reinterpret_cast<const u32x4*>(bptr[i] + ko);
    };
    auto sstore = [&](int buf) {
        char* As = smem + buf * STAGE;
        char* Bs = As + BM * 128;
#pragma unroll
        for (int i = 0; i < A_CH; ++i) {
            const int r = lr + i * ROWS_PER_PASS;
            *reinterpret_cast<u32x4*>(As + r * 128 + ((lc ^ (r & 7)) << 4)) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < B_CH; ++i) {
            const int r = lr + i * ROWS_PER_PASS;
            *reinterpret_cast<u32x4*>(Bs + r * 128 + ((lc ^ (r & 7)) << 4)) = rb[i];
        }
    };

    f32x16 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    const int nk = p.K >> 6;
    gload(0);
    sstore(0);
    __syncthreads();
    const int a_off = (wm * TM + (lane & 31)) * 128;
    const int b_off = BM * 128 + (wn * TN + (lane & 31)) * 128;
    for (int kt = 0; kt < nk; ++kt) {
        if (kt + 1 < nk) gload(kt + 1);
        const char* St = smem + (kt & 1) * STAGE;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const int sw = ((kk * 2 + (lane >> 5)) ^ (lane & 7)) << 4;
            bf16x8 af[FM], bfr[FN];
#pragma unroll
            for (int i = 0; i < FM; ++i) af[i] = *reinterpret_cast<const bf16x8*>(St + a_off + i * 32 * 128 + sw);
#pragma unroll
            for (int j = 0; j < FN; ++j) bfr[j] = *reinterpret_cast<const bf16x8*>(St + b_off + j * 32 * 128 + sw);
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) sstore((kt + 1) & 1);
        __syncthreads();
    }

    // ---- epilogue.  32x32 MFMA result: lane holds column lane&31, rows 8*(v/4) + 4*(lane>>5) + (v&3). ----
    unsigned short* out = reinterpret_cast<unsigned short*>(p.out);
#pragma unroll
    for (int i = 0; i < FM; ++i) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int rl = wm * TM + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
            if (rl >= nrows) continue;
            const long orow = (long)(row0 + rl) * p.ldo;
            if (SWIGLU) {
#pragma unroll
                for (int jp = 0; jp < FN / 2; ++jp) {
                    const int col = n0 + (wn * (TN / 64) + jp) * 32 + (lane & 31);
                    const float g = acc[i][2 * jp][v], u = acc[i][2 * jp + 1][v];
                    const float h = g / (1.0f + __expf(-g)) * u;
                    if (col < p.N) out[orow + col] = f2bf(h);
                }
            } else {
                const float w = p.row_weight[row0 + rl];
#pragma unroll
                for (int j = 0; j < FN; ++j) {
                    const int col = n0 + wn * TN + j * 32 + (lane & 31);
                    if (col < p.N) out[orow + col] = f2bf(acc[i][j][v] * w);
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// combine: one thread = 8 columns of one token; rows summed in slot order, shared experts first.
// ------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) combine_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ Y,
                                                      const int32_t* __restrict__ token_rows, bf16_t* __restrict__ out,
                                                      int T, int d, int K, int Ns, int add_residual)
{
    const int chunks = d >> 3;
    const long gid = (long)blockIdx.x * 256 + threadIdx.x;
    if (gid >= (long)T * chunks) return;
    const int t = (int)(gid / chunks), c8 = (int)(gid - (long)t * chunks) * 8;
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.0f;
    auto add_row = [&](const bf16_t* rowp) {
        const uint4 q = *reinterpret_cast<const uint4*>(rowp + c8);
        const unsigned int w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            acc[2 * e] += __uint_as_float(w[e] << 16);
            acc[2 * e + 1] += __uint_as_float(w[e] & 0xFFFF0000u);
        }
    };
    if (add_residual) add_row(x + (long)t * d);
    const int slots = K + Ns;
    const int32_t* tr = token_rows + (long)t * slots;
    for (int s = 0; s < Ns; ++s) add_row(Y + (long)tr[K + s] * d);
    for (int j = 0; j < K; ++j) {
        const int r = tr[j];
        if (r >= 0) add_row(Y + (long)r * d);
    }
    uint4 o;
    o.x = (unsigned)f2bf(acc[0]) | ((unsigned)f2bf(acc[1]) << 16);
    o.y = (unsigned)f2bf(acc[2]) | ((unsigned)f2bf(acc[3]) << 16);
    o.z = (unsigned)f2bf(acc[4]) | ((unsigned)f2bf(acc[5]) << 16);
    o.w = (unsigned)f2bf(acc[6]) | ((unsigned)f2bf(acc[7]) << 16);
    *reinterpret_cast<uint4*>(out + (long)t * d + c8) = o;
}

// ------------------------------------------------------------------------------------------------
template <int BM, int BN, int WM, int WN, bool SWIGLU>
static hipError_t launch_gemm(const GemmArgs& a, int max_mtiles, hipStream_t s)
{
    constexpr int NTH = WM * WN * 64;
    constexpr int LDS = 2 * (BM + BN) * 128;
    static bool attr_set = false;
    auto kern = ffn_gemm_kernel<BM, BN, WM, WN, SWIGLU>;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const long total = (long)max_mtiles * a.n_ntiles;
    const int grid = (int)((total + 7) / 8 * 8);
    kern<<<grid, NTH, LDS, s>>>(a);
    return hipGetLastError();
}

// Tile height from the expected rows per unit (the counts themselves stay on the device).
static int pick_bm(int64_t expected_rows_per_unit)
{
    if (const char* e = std::getenv("BROWNOUT_MOE_BM")) {
        const int v = std::atoi(e);
        if (v == 32 || v == 64 || v == 128 || v == 256) return v;
    }
    if (expected_rows_per_unit >= 384) return 256;
    if (expected_rows_per_unit >= 96) return 128;
    if (expected_rows_per_unit >= 40) return 64;
    return 32;
}

template <bool SWIGLU>
static hipError_t dispatch_gemm(int BM, const GemmArgs& a, int max_mtiles, hipStream_t s)
{
    switch (BM) {
        case 256: return launch_gemm<256, 256, 2, 4, SWIGLU>(a, max_mtiles, s);
        case 128: return launch_gemm<128, 256, 2, 4, SWIGLU>(a, max_mtiles, s);
        case 64: return launch_gemm<64, 256, 1, 4, SWIGLU>(a, max_mtiles, s);
        default: return launch_gemm<32, 256, 1, 4, SWIGLU>(a, max_mtiles, s);
    }
}

hipError_t launch_ffn(const Dims& D, int u_lo, int u_hi, int Fdim, int64_t expected_rows, const bf16_t* x,
                      const int32_t* gather, const int32_t* unit_cnt, const int32_t* unit_off,
                      const float* row_weight, const FfnWeights& experts, const FfnWeights& united,
                      const FfnWeights& shared, int32_t* tile_table, bf16_t* H, bf16_t* Y, hipStream_t s)
{
    const int n_units = u_hi - u_lo;
    const int BM = pick_bm(expected_rows);
    const int max_mtiles = (int)std::min<int64_t>(D.row_cap / BM + n_units, D.tile_cap);
    {
        ProfScope ps(MOE_STAGE_TILES, s);
        tile_table_kernel<<<1, 256, 0, s>>>(unit_cnt, unit_off, u_lo, u_hi, BM, tile_table, D.tile_cap);
    }
    GemmArgs g1;
    g1.A = x; g1.lda = D.d; g1.gather = gather; g1.table = tile_table;
    g1.wa0 = experts.w1; g1.wa1 = united.w1; g1.wa2 = shared.w1;
    g1.wb0 = experts.w3; g1.wb1 = united.w3; g1.wb2 = shared.w3;
    g1.m = D.m; g1.G = D.G; g1.N = Fdim; g1.K = D.d;
    g1.out = H; g1.ldo = D.Fmax; g1.row_weight = nullptr;
    g1.n_ntiles = ceil_div(Fdim, 128);
    {
        ProfScope ps(MOE_STAGE_GEMM1, s);
        hipError_t e = dispatch_gemm<true>(BM, g1, max_mtiles, s);
        if (e != hipSuccess) return e;
    }
    GemmArgs g2;
    g2.A = H; g2.lda = D.Fmax; g2.gather = nullptr; g2.table = tile_table;
    g2.wa0 = experts.w2; g2.wa1 = united.w2; g2.wa2 = shared.w2;
    g2.wb0 = g2.wb1 = g2.wb2 = nullptr;
    g2.m = D.m; g2.G = D.G; g2.N = D.d; g2.K = Fdim;
    g2.out = Y; g2.ldo = D.d; g2.row_weight = row_weight;
    g2.n_ntiles = ceil_div(D.d, 256);
    {
        ProfScope ps(MOE_STAGE_GEMM2, s);
        hipError_t e = dispatch_gemm<false>(BM, g2, max_mtiles, s);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_combine(const Dims& D, const bf16_t* x, const bf16_t* Y, const int32_t* token_rows, bf16_t* out,
                          hipStream_t s)
{
    ProfScope ps(MOE_STAGE_COMBINE, s);
    const long n = (long)D.T * (D.d / 8);
    combine_kernel<<<(int)((n + 255) / 256), 256, 0, s>>>(x, Y, token_rows, out, D.T, D.d, D.K, D.Ns, D.add_residual);
    return hipGetLastError();
}

}  // namespace bmoe
