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
    int group_m;                                // M tiles per L2 super-tile
};

// Workgroup barrier that orders LDS traffic for the compiler without the vmcnt(0) wait __syncthreads()
// implies: tiles still in flight to LDS (tracked by vmcnt) must stay in flight across it.  Every wave
// waits for the loads it needs (s_waitcnt vmcnt) itself before arriving.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// s_waitcnt immediate that waits for vmcnt <= n only (gfx9 encoding: vmcnt in bits 3:0 and 15:14).
__host__ __device__ constexpr int vmcnt_imm(int n) { return (n & 0xF) | ((n >> 4) << 14) | 0x0F70; }

template <int BM, int BN, int WM, int WN, int BK, int NSTAGE, bool PINGPONG, bool SWIGLU>
__global__ void __launch_bounds__(WM * WN * 64) ffn_gemm_kernel(GemmArgs p)
{
    constexpr int TM = BM / WM, TN = BN / WN;
    constexpr int FM = TM / 32, FN = TN / 32;
    constexpr int RB = BK * 2;                    // bytes of one LDS row (one tile row, BK bf16)
    constexpr int CPR = RB / 16;                  // 16-byte chunks per row
    constexpr int WR = 256 / RB;                  // rows per 256-byte bank window (the LDS has 64 banks)
    constexpr int RPG = 1024 / RB;                // rows one wave-wide 16-byte-per-lane load covers
    constexpr int STAGE = (BM + BN) * RB;
    static_assert(BK == 32 || BK == 64, "k tile");
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
    // Super-tiles of group_m M tiles x all N tiles, M fastest: the ~32 blocks an XCD runs at a time
    // cover group_m x (32/group_m) tiles and share their A and B panels in that XCD's L2.
    const int gspan = p.group_m * p.n_ntiles;
    const int gi = L / gspan, rem = L - gi * gspan;
    const int mt_first = gi * p.group_m;
    const int gsz = min(p.group_m, n_mt - mt_first);
    const int nt = rem / gsz, mt = mt_first + (rem - nt * gsz);
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

    // ---- loader: direct global -> LDS (global_load_lds_dwordx4).  One wave instruction fills 1 KiB of
    // LDS contiguously = RPG rows, lane l -> row l/CPR, slot l%CPR.  Slots are XOR-swizzled, on the global
    // side: slot s of row r receives chunk s ^ ((r/WR) & (CPR-1)).  The LDS serves a ds_read_b128 sixteen
    // lanes at a time across 64 banks (256 bytes = WR rows), so sixteen consecutive rows reading the
    // same chunk must fall on sixteen different 16-byte bank groups; the r/WR term does that.
    // Wave w moves row groups w, w+NW, ...
    constexpr int NW = WM * WN;
    constexpr int GROUPS = (BM + BN) / RPG;
    constexpr int LD_PER_WAVE = GROUPS / NW;
    static_assert(GROUPS % NW == 0, "loader shape");
    const bf16_t* gptr[LD_PER_WAVE];
#pragma unroll
    for (int i = 0; i < LD_PER_WAVE; ++i) {
        const int row = (wave + i * NW) * RPG + lane / CPR;      // row of the stage: A rows, then B rows
        const int l_chunk = (lane % CPR) ^ ((row / WR) & (CPR - 1));
        if (row < BM) {
            const int r = row < nrows ? row : 0;                   // ragged tile: re-read row 0, never stored
            const long src_row = p.gather ? (long)p.gather[row0 + r] : (long)(row0 + r);
            gptr[i] = p.A + src_row * p.lda + l_chunk * 8;
        } else {
            const int n = row - BM;
            int col;
            const bf16_t* W = Wa;
            if (SWIGLU) {
                const int w_n = n / TN, j = (n % TN) >> 5, c = n & 31;
                col = n0 + (w_n * (TN / 64) + (j >> 1)) * 32 + c;
                if (j & 1) W = Wb;
            } else {
                col = n0 + n;
            }
            col = col < p.N ? col : p.N - 1;                       // ragged N: clamp, never stored
            gptr[i] = W + (size_t)col * p.K + l_chunk * 8;
        }
    }
    auto issue_loads = [&](int kt) {
        char* dst = smem + (kt % NSTAGE) * STAGE + wave * 1024;
#pragma unroll
        for (int i = 0; i < LD_PER_WAVE; ++i)
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void*)(gptr[i] + kt * BK),
                (__attribute__((address_space(3))) void*)(dst + i * NW * 1024), 16, 0, 0);
    };

    f32x16 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    // ---- main loop: NSTAGE LDS buffers, tiles kt+1 .. kt+NSTAGE-1 in flight while tile kt is multiplied.
    const int nk = p.K / BK;
#pragma unroll
    for (int q = 0; q < NSTAGE - 1; ++q)
        if (q < nk) issue_loads(q);
    const int a_off = (wm * TM + (lane & 31)) * RB;
    const int b_off = BM * RB + (wn * TN + (lane & 31)) * RB;
    const int swz = ((lane & 31) / WR) & (CPR - 1);
    constexpr int KK = BK / 16;
    if constexpr (PINGPONG) {
        // Two groups of waves (one wave of each per SIMD) run half a step out of phase: while one group
        // issues its MFMAs for tile kt, the other reads its fragments of the next tile from LDS and
        // queues global->LDS loads, so the matrix pipe of every SIMD always has a wave feeding it.
        // Barriers separate the phases; group 1 starts one barrier late and group 0 ends one late.
        static_assert(NSTAGE >= 2 && WM == 2 && BK % 32 == 0, "ping-pong shape");
        constexpr int P = BK / 32;                            // steps (of 32 k) per tile
        const int grp = wm;
        if (NSTAGE - 2 < nk && NSTAGE > 2) __builtin_amdgcn_s_waitcnt(vmcnt_imm((NSTAGE - 2) * LD_PER_WAVE));
        else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
        lds_barrier();                                        // tile 0 is in LDS for everyone
        if (grp == 1) lds_barrier();
        for (int kt = 0; kt < nk; ++kt) {
            const char* St = smem + (kt % NSTAGE) * STAGE;
#pragma unroll
            for (int ph = 0; ph < P; ++ph) {
                // -- memory phase.  At the first step of tile kt the buffer of tile kt-1 is free (both
                // groups finished reading it two barriers ago): refill it with tile kt+NSTAGE-1.
                if (ph == 0 && kt + NSTAGE - 1 < nk) issue_loads(kt + NSTAGE - 1);
                bf16x8 af[2][FM], bfr[2][FN];
#pragma unroll
                for (int kk = 0; kk < 2; ++kk) {
                    const int sw = (((ph * 2 + kk) * 2 + (lane >> 5)) ^ swz) << 4;
#pragma unroll
                    for (int i = 0; i < FM; ++i)
                        af[kk][i] = *reinterpret_cast<const bf16x8*>(St + a_off + i * 32 * RB + sw);
#pragma unroll
                    for (int j = 0; j < FN; ++j)
                        bfr[kk][j] = *reinterpret_cast<const bf16x8*>(St + b_off + j * 32 * RB + sw);
                }
                // fragments are in registers (lgkmcnt 0); at the last step of tile kt, tile kt+1 must
                // have landed too: it is read right after the next barrier pair
                if (ph == P - 1) {
                    if (NSTAGE > 2 && kt + NSTAGE - 1 < nk)
                        __builtin_amdgcn_s_waitcnt(vmcnt_imm((NSTAGE - 2) * LD_PER_WAVE) & 0xF0FF);
                    else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0) & 0xF0FF);
                } else {
                    __builtin_amdgcn_s_waitcnt(0xC07F);       // lgkmcnt(0) only
                }
                __builtin_amdgcn_sched_barrier(0);
                lds_barrier();
                __builtin_amdgcn_sched_barrier(0);
                // -- compute phase
                __builtin_amdgcn_s_setprio(1);
#pragma unroll
                for (int kk = 0; kk < 2; ++kk)
#pragma unroll
                    for (int i = 0; i < FM; ++i)
#pragma unroll
                        for (int j = 0; j < FN; ++j)
                            acc[i][j] =
                                __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[kk][j], af[kk][i], acc[i][j], 0, 0, 0);
                __builtin_amdgcn_s_setprio(0);
                __builtin_amdgcn_sched_barrier(0);
                lds_barrier();
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if (grp == 0) lds_barrier();
    } else {
        for (int kt = 0; kt < nk; ++kt) {
            // this wave's loads of tile kt have landed once at most the NSTAGE-2 younger tiles are outstanding
            if (kt + NSTAGE - 2 < nk) __builtin_amdgcn_s_waitcnt(vmcnt_imm((NSTAGE - 2) * LD_PER_WAVE));
            else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
            lds_barrier();        // every wave's part of tile kt is in LDS; nobody still reads tile kt-1's buffer
            if (kt + NSTAGE - 1 < nk) issue_loads(kt + NSTAGE - 1);
            const char* St = smem + (kt % NSTAGE) * STAGE;
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                const int sw = ((kk * 2 + (lane >> 5)) ^ swz) << 4;
                bf16x8 af[FM], bfr[FN];
#pragma unroll
                for (int i = 0; i < FM; ++i) af[i] = *reinterpret_cast<const bf16x8*>(St + a_off + i * 32 * RB + sw);
#pragma unroll
                for (int j = 0; j < FN; ++j) bfr[j] = *reinterpret_cast<const bf16x8*>(St + b_off + j * 32 * RB + sw);
#pragma unroll
                for (int i = 0; i < FM; ++i)
#pragma unroll
                    for (int j = 0; j < FN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
            }
        }
    }

    // ---- epilogue.  The MFMAs were issued as (weights x rows), so a lane holds, for output row lane&31,
    // the four consecutive columns 8*(v>>2) + 4*(lane>>5) + 0..3 of each 32x32 tile: 8-byte bf16x4 stores.
    unsigned short* out = reinterpret_cast<unsigned short*>(p.out);
#pragma unroll
    for (int i = 0; i < FM; ++i) {
        const int rl = wm * TM + i * 32 + (lane & 31);
        if (rl >= nrows) continue;
        unsigned short* orow = out + (long)(row0 + rl) * p.ldo;
        if (SWIGLU) {
#pragma unroll
            for (int jp = 0; jp < FN / 2; ++jp) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int col = n0 + (wn * (TN / 64) + jp) * 32 + 8 * q + 4 * (lane >> 5);
                    unsigned short h[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float g = acc[i][2 * jp][4 * q + e], u = acc[i][2 * jp + 1][4 * q + e];
                        h[e] = f2bf(g * __frcp_rn(1.0f + __expf(-g)) * u);
                    }
                    if (col < p.N)
                        *reinterpret_cast<uint2*>(orow + col) =
                            make_uint2((unsigned)h[0] | ((unsigned)h[1] << 16), (unsigned)h[2] | ((unsigned)h[3] << 16));
                }
            }
        } else {
            const float w = p.row_weight[row0 + rl];
#pragma unroll
            for (int j = 0; j < FN; ++j) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int col = n0 + wn * TN + j * 32 + 8 * q + 4 * (lane >> 5);
                    unsigned short h[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) h[e] = f2bf(acc[i][j][4 * q + e] * w);
                    if (col < p.N)
                        *reinterpret_cast<uint2*>(orow + col) =
                            make_uint2((unsigned)h[0] | ((unsigned)h[1] << 16), (unsigned)h[2] | ((unsigned)h[3] << 16));
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
template <int BM, int BN, int WM, int WN, int BK, int NSTAGE, bool PINGPONG, bool SWIGLU>
static hipError_t launch_gemm(const GemmArgs& a, int max_mtiles, hipStream_t s)
{
    constexpr int NTH = WM * WN * 64;
    constexpr int LDS = NSTAGE * (BM + BN) * BK * 2;
    static_assert(LDS <= 160 * 1024, "LDS budget of one CU");
    static bool attr_set = false;
    auto kern = ffn_gemm_kernel<BM, BN, WM, WN, BK, NSTAGE, PINGPONG, SWIGLU>;
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
        case 256: return launch_gemm<256, 256, 2, 4, 64, 2, true, SWIGLU>(a, max_mtiles, s);
        case 128: return launch_gemm<128, 256, 2, 4, 64, 3, true, SWIGLU>(a, max_mtiles, s);
        case 64: return launch_gemm<64, 256, 1, 4, 64, 3, false, SWIGLU>(a, max_mtiles, s);
        default: return launch_gemm<32, 256, 1, 4, 64, 4, false, SWIGLU>(a, max_mtiles, s);
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
    int group_m = 4;
    if (const char* e = std::getenv("BROWNOUT_MOE_GM")) group_m = std::max(1, std::atoi(e));
    g1.group_m = group_m;
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
    g2.group_m = group_m;
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
