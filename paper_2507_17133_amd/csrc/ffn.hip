// Expert FFNs of the BrownoutMoE layer as two grouped GEMMs on gfx950 MFMA, plus the weighted combine.
//
//   GEMM1  H[r][f] = silu(x_r . W1_u[f]) * (x_r . W3_u[f])      rows r of unit u, gathered from x
//   GEMM2  Y[r][c] = H_r . W2_u[c]                              (stored in half precision)
//   combine out_t  = [x_t] + sum over the token's rows r of row_weight[r] * Y_r   (layer equation, fixed order)
//
// Both operands of both GEMMs are K-contiguous (x [T][d], W1/W3 [F][d], H [R][F], W2 [d][F]), which is
// the natural operand order of the bf16 MFMAs: a lane supplies 8 consecutive k of one row.  A block owns a
// BM x 256 output tile; k tiles of 64 (whole 128-byte lines per row) are staged in LDS in 16-byte chunks,
// XOR-swizzled so that the ds_read_b128 fragment loads are conflict free.  In GEMM1 a block's 256 B rows
// are 128 columns of W1 and the same 128 columns of W3, interleaved tile by tile, so that the gate and up
// values of one (row, f) land in the same lane and SwiGLU is applied in registers.
// Which (unit, rows) an M tile covers comes from a tile table built on the device from the unit counts,
// so skewed expert loads need no host round trip.  Each XCD (block id mod 8) works on a contiguous range
// of tiles, ordered so that the blocks it runs at a time share A and B panels in its own L2.
//
// Kernels, by tile height (chosen on the host from the expected rows per unit; all tiles of a unit, its ragged
// last one included, stay next to each other in the tile order, because they share the unit's weight panels
// in the L2 of the XCD that runs them):
//   256 rows  ffn_gemm_w4_kernel   four waves, one per SIMD, 128x128 wave tiles, 16x16x32 MFMA, persistent;
//                                  further blocks of the same launch take the tiles left over after the last
//                                  full round: cut along K (fp32 partial tiles, summed by
//                                  gemm_tail_sum_kernel) or in two along N
//   128 rows  ffn_gemm_pp_kernel   eight waves in two groups that alternate memory and MFMA phases
//   64, 32    ffn_gemm_kernel      four waves, plain multi-stage ring (decode: weight streaming bound)
#include "internal.h"
#include "tiles.h"

#include <algorithm>
#include <cstdlib>

namespace bmoe {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// two floats -> two bf16 (round to nearest even) in one 32-bit word, first value in the low half
__device__ __forceinline__ unsigned pack_bf16(float lo, float hi)
{
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    const f32x2 v = {lo, hi};
    const bf16x2 b = __builtin_convertvector(v, bf16x2);
    return __builtin_bit_cast(unsigned, b);
}
// Two floats -> two IEEE half values in one 32-bit word (round toward zero, so an overflow saturates at
// the largest finite half instead of becoming infinite).  Y, the FFN output rows between GEMM2 and the
// combine, is stored this way: the combine adds up rows of different experts that partly cancel, and with
// bf16's 8-bit mantissa the rounding of the large terms would dominate the error of the small sum.
__device__ __forceinline__ unsigned pack_f16(float lo, float hi)
{
    return __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pkrtz(lo, hi));
}
// silu(g) * u with the hardware exp2 and reciprocal (the result is rounded to bf16 right after)
__device__ __forceinline__ float swiglu(float g, float u)
{
    return g * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.44269504f * g)) * u;
}

// ------------------------------------------------------------------------------------------------
// Tile tables from the unit counts, when the routing kernels have not already built them (row lists brought
// by the caller; single units of the united-expert build): one wavefront per job.
// ------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(64) tile_table_kernel(const int32_t* __restrict__ unit_cnt,
                                                        const int32_t* __restrict__ unit_off, TileJobs jobs)
{
    if ((int)blockIdx.x < jobs.n)
        build_tile_table(unit_cnt, unit_off, jobs.job[blockIdx.x], jobs.cap, threadIdx.x);
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
    int n_ntiles;
    int group_m;                                // M tiles per L2 super-tile
    int ksplit; long plane;                     // GEMM2 only: K split into ksplit slices, slice s writes out + s*plane
    float* out32;                               // plain GEMM only (32- and 64-row kernel): fp32 output instead of out
    float* partial;                             // four-wave kernel, ksplit 1: scratch of the K-split tail (or null)
    int partial_cap;                            // fp32 tiles it holds
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

// s_waitcnt immediates (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8).
__host__ __device__ constexpr int vmcnt_imm(int n) { return (n & 0xF) | ((n >> 4) << 14) | 0x0F70; }       // vmcnt <= n
__host__ __device__ constexpr int vmcnt_lgkm0_imm(int n) { return vmcnt_imm(n) & 0xF0FF; }                 // and lgkmcnt 0

// Which tile a block works on.
struct Tile {
    int unit, row0, nrows, nt, n0;
    int kslice, ks;                             // this block multiplies slice kslice of ks slices of K
    int part;                                   // slot in GemmArgs::partial the result goes to, or -1: to the output
    int half;                                   // column-half tail of the four-wave kernel: which half of the tile
    const bf16_t *Wa, *Wb;
};

template <int BNC, bool SWIGLU>
__device__ __forceinline__ bool decode_tile(const GemmArgs& p, Tile& t)
{
    const int n_mt = p.table[0];
    const int tiles = n_mt * p.n_ntiles;
    const int total = tiles * p.ksplit;
    const int chunk = (total + 7) >> 3;
    const int bi = blockIdx.x >> 3;
    if (bi >= chunk) return false;
    const int Lfull = (blockIdx.x & 7) * chunk + bi;           // block id mod 8 = XCD: contiguous range per XCD
    if (Lfull >= total) return false;
    t.kslice = Lfull / tiles;
    t.ks = p.ksplit;
    t.part = -1;
    t.half = 0;
    const int L = Lfull - t.kslice * tiles;
    // Super-tiles of group_m M tiles x all N tiles, M fastest: the ~32 blocks an XCD runs at a time
    // cover group_m x (32/group_m) tiles and share their A and B panels in that XCD's L2.
    const int gspan = p.group_m * p.n_ntiles;
    const int gi = L / gspan, rem = L - gi * gspan;
    const int mt_first = gi * p.group_m;
    const int gsz = min(p.group_m, n_mt - mt_first);
    t.nt = rem / gsz;
    const int mt = mt_first + (rem - t.nt * gsz);
    const int4 te = reinterpret_cast<const int4*>(p.table + 4)[mt];
    t.unit = te.x; t.row0 = te.y; t.nrows = te.z;
    const int src = t.unit < p.m ? 0 : (t.unit < p.m + p.G ? 1 : 2);
    const int widx = t.unit - (src == 0 ? 0 : (src == 1 ? p.m : p.m + p.G));
    const size_t wsz = (size_t)p.N * p.K;
    t.Wa = (src == 0 ? p.wa0 : (src == 1 ? p.wa1 : p.wa2)) + (size_t)widx * wsz;
    t.Wb = SWIGLU ? (src == 0 ? p.wb0 : (src == 1 ? p.wb1 : p.wb2)) + (size_t)widx * wsz : nullptr;
    t.n0 = t.nt * BNC;
    return true;
}

// Global row of A for tile row `row` (ragged tiles re-read row 0; such rows are never stored).
__device__ __forceinline__ const bf16_t* a_row_ptr(const GemmArgs& p, const Tile& t, int row)
{
    const int r = row < t.nrows ? row : 0;
    const long src_row = p.gather ? (long)p.gather[t.row0 + r] : (long)(t.row0 + r);
    return p.A + src_row * p.lda;
}

// Weight row behind row n of the block's B tile.  GEMM1: the wave tile's TW-column MFMA tiles alternate
// W1 / W3 of the same TW f columns.  Columns past N are clamped (never stored).
template <int TN, bool SWIGLU, int TW = 32>
__device__ __forceinline__ const bf16_t* b_row_ptr(const GemmArgs& p, const Tile& t, int n)
{
    int col;
    const bf16_t* W = t.Wa;
    if (SWIGLU) {
        const int w_n = n / TN, j = (n % TN) / TW, c = n % TW;
        col = t.n0 + (w_n * (TN / (2 * TW)) + (j >> 1)) * TW + c;
        if (j & 1) W = t.Wb;
    } else {
        col = t.n0 + n;
    }
    col = col < p.N ? col : p.N - 1;
    return W + (size_t)col * p.K;
}

// Epilogue.  The MFMAs are issued as (weights x rows), so a lane holds, for output row lane&31, the four
// consecutive columns 8*(v>>2) + 4*(lane>>5) + 0..3 of each 32x32 tile: SwiGLU in registers, 8-byte stores.
template <int FM, int FN, int TM, int TN, bool SWIGLU>
__device__ __forceinline__ void store_tile(const GemmArgs& p, const Tile& t, const f32x16 (&acc)[FM][FN], int wm,
                                           int wn, int lane)
{
    unsigned short* out = reinterpret_cast<unsigned short*>(p.out) + (size_t)t.kslice * p.plane;
#pragma unroll
    for (int i = 0; i < FM; ++i) {
        const int rl = wm * TM + i * 32 + (lane & 31);
        if (rl >= t.nrows) continue;
        unsigned short* orow = out + (long)(t.row0 + rl) * p.ldo;
        if (SWIGLU) {
#pragma unroll
            for (int jp = 0; jp < FN / 2; ++jp) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int col = t.n0 + (wn * (TN / 64) + jp) * 32 + 8 * q + 4 * (lane >> 5);
                    float h[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) h[e] = swiglu(acc[i][2 * jp][4 * q + e], acc[i][2 * jp + 1][4 * q + e]);
                    if (col < p.N)
                        *reinterpret_cast<uint2*>(orow + col) = make_uint2(pack_bf16(h[0], h[1]), pack_bf16(h[2], h[3]));
                }
            }
        } else {
#pragma unroll
            for (int j = 0; j < FN; ++j) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int col = t.n0 + wn * TN + j * 32 + 8 * q + 4 * (lane >> 5);
                    if (col >= p.N) continue;
                    if (p.out32)
                        *reinterpret_cast<float4*>(p.out32 + (long)(t.row0 + rl) * p.ldo + col) =
                            make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
                    else
                        *reinterpret_cast<uint2*>(orow + col) =
                            make_uint2(pack_f16(acc[i][j][4 * q], acc[i][j][4 * q + 1]),
                                       pack_f16(acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]));
                }
            }
        }
    }
}

// The same tile written as whole row segments.  In the accumulator layout neighbouring lanes hold different
// rows, so a store instruction of store_tile reaches memory as 64 separate 8-byte writes.  Here the wave tile
// (32 FM rows x 64 tile columns: 64 output columns of GEMM2 = one 128-byte line per row, 32 of GEMM1 = 64
// bytes) goes through 4 KiB (2 KiB) per 32 rows of LDS private to the wave and comes back row-contiguous,
// 16 bytes per lane.  `scratch`: 8 KiB of the stage buffers, which are free once every wave has left the k
// loop (the caller's barrier).  8-byte slot s of row r lives at slot s ^ 2((r/2)&7) (rows of 64 bytes:
// s ^ 2((r/4)&3)): writes and reads are free of bank conflicts.  fp32 output keeps the plain path.
template <int FM, int FN, int TM, int TN, bool SWIGLU>
__device__ __forceinline__ void store_tile_lines(const GemmArgs& p, const Tile& t, const f32x16 (&acc)[FM][FN], int wm,
                                                 int wn, int lane, char* scratch)
{
    static_assert(FN == 2 && FM <= 2, "wave tile of 64 tile columns, one scratch half per 32 rows");
    if (p.out32) { store_tile<FM, FN, TM, TN, SWIGLU>(p, t, acc, wm, wn, lane); return; }
    unsigned short* out = reinterpret_cast<unsigned short*>(p.out) + (size_t)t.kslice * p.plane;
    const int r = lane & 31, hb = lane >> 5;
    constexpr int ROWB = SWIGLU ? 64 : 128;                     // bytes of a row in the scratch
    const int fx = SWIGLU ? ((r >> 2) & 3) << 1 : ((r >> 1) & 7) << 1;
#pragma unroll
    for (int i = 0; i < FM; ++i) {
        char* sc = scratch + i * 4096 + r * ROWB;
        if (SWIGLU) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float h[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) h[e] = swiglu(acc[i][0][4 * q + e], acc[i][1][4 * q + e]);
                *reinterpret_cast<uint2*>(sc + (((q * 2 + hb) ^ fx) << 3)) =
                    make_uint2(pack_bf16(h[0], h[1]), pack_bf16(h[2], h[3]));
            }
        } else {
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    *reinterpret_cast<uint2*>(sc + (((j * 8 + q * 2 + hb) ^ fx) << 3)) =
                        make_uint2(pack_f16(acc[i][j][4 * q], acc[i][j][4 * q + 1]),
                                   pack_f16(acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]));
        }
    }
    constexpr int LPR = ROWB / 16;                              // lanes per row on the way out: 8 or 4
    constexpr int RPI = 64 / LPR;                               // rows per store instruction: 8 or 16
    const int k = lane % LPR, rr = lane / LPR;
    const int col = (SWIGLU ? t.n0 + wn * (TN / 2) : t.n0 + wn * TN) + k * 8;
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int rd = 0; rd < 32 / RPI; ++rd) {
            const int row = rd * RPI + rr;
            const int gx = SWIGLU ? ((row >> 2) & 3) << 1 : ((row >> 1) & 7) << 1;
            const uint4 v = *reinterpret_cast<const uint4*>(scratch + i * 4096 + row * ROWB + (((2 * k) ^ gx) << 3));
            const int rl = wm * TM + i * 32 + row;
            if (rl < t.nrows && col < p.N) *reinterpret_cast<uint4*>(out + (long)(t.row0 + rl) * p.ldo + col) = v;
        }
}

// Epilogue for 16x16 MFMA tiles (same transposed product): a lane holds, for output row lane&15, the four
// consecutive columns 4*(lane>>4) + 0..3 of each 16x16 tile.  All values are converted first, as one
// branch-free block the scheduler can interleave freely (a lone wave per SIMD has nothing else to hide
// the latency of exp and rcp behind), then stored row by row under the row mask.  N is a multiple of 64,
// so a 64-column group of a wave tile is either entirely inside the matrix or entirely outside.
// (Used by the column-half tiles of the tail; whole tiles take store_tile16_lines below.)
template <int FM, int FN, int TM, int TN, bool SWIGLU>
__device__ __forceinline__ void store_tile16(const GemmArgs& p, const Tile& t, const f32x4 (&acc)[FM][FN], int wm,
                                             int wn, int lane)
{
    unsigned short* out = reinterpret_cast<unsigned short*>(p.out) + (size_t)t.kslice * p.plane;
    constexpr int NG = SWIGLU ? FN / 2 : FN;             // 8-byte stores per output row and wave
    constexpr int HM = FM / 2;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        uint2 res[HM][NG];
#pragma unroll
        for (int ii = 0; ii < HM; ++ii) {
            const int i = half * HM + ii;
#pragma unroll
            for (int g = 0; g < NG; ++g) {
                if (SWIGLU) {
                    float h[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) h[e] = swiglu(acc[i][2 * g][e], acc[i][2 * g + 1][e]);
                    res[ii][g] = make_uint2(pack_bf16(h[0], h[1]), pack_bf16(h[2], h[3]));
                } else {
                    res[ii][g] = make_uint2(pack_f16(acc[i][g][0], acc[i][g][1]), pack_f16(acc[i][g][2], acc[i][g][3]));
                }
            }
        }
#pragma unroll
        for (int ii = 0; ii < HM; ++ii) {
            const int i = half * HM + ii;
            const int rl = wm * TM + i * 16 + (lane & 15);
            if (rl >= t.nrows) continue;
            unsigned short* orow = out + (long)(t.row0 + rl) * p.ldo;
#pragma unroll
            for (int g = 0; g < NG; ++g) {
                const int cbase = SWIGLU ? t.n0 + (wn * (TN / 32) + g) * 16 : t.n0 + wn * TN + g * 16;
                if (cbase < p.N) *reinterpret_cast<uint2*>(orow + cbase + 4 * (lane >> 4)) = res[ii][g];
            }
        }
    }
}

// The same tile written in whole 128-byte lines.  In the accumulator layout neighbouring lanes hold different
// rows, so a store instruction of store_tile16 reaches memory as 64 separate 8-byte writes; short K makes that
// the largest cost of a GEMM2 tile.  Here each group of 16 rows x 64 output columns goes through 2 KiB of LDS
// private to the wave (`scratch`: four 1 KiB pieces 4 KiB apart, free while the epilogue runs: the wave's own
// load targets in the third B buffer that the first loads of the next tile do not use) and comes back as
// rows: 8 lanes x 16 bytes per row, 8 rows per store instruction.  8-byte slot s of row r lives at slot
// s ^ 2(r/2): both the 8-byte writes (16 lanes, one per row) and the 16-byte reads (16 lanes, two rows) are
// free of bank conflicts.  LDS operations of a wave execute in order, so no barrier is needed.  The LDS
// accesses are written as instructions: left to the compiler they are preceded by a wait for every direct
// global->LDS load in flight (it cannot tell their targets from this scratch), i.e. for the next tile's first
// loads, which were issued a moment ago to land behind this epilogue.
template <int FM, int FN, int TM, int TN, bool SWIGLU>
__device__ __forceinline__ void store_tile16_lines(const GemmArgs& p, const Tile& t, const f32x4 (&acc)[FM][FN], int wm,
                                                   int wn, int lane, char* scratch)
{
    unsigned short* out = reinterpret_cast<unsigned short*>(p.out) + (size_t)t.kslice * p.plane;
    constexpr int NG = SWIGLU ? FN / 2 : FN;             // 16-column groups of output per wave
    static_assert(NG % 4 == 0, "units of 64 output columns");
    constexpr int NU = NG / 4;                           // units per group of 16 rows
    constexpr int NUT = FM * NU;                         // units of the wave tile
    const unsigned base = (unsigned)(unsigned long)((__attribute__((address_space(3))) char*)scratch);
    const int r = lane & 15, c = lane >> 4;
    const int x = (r >> 1) << 1;
    unsigned w_addr[4];
#pragma unroll
    for (int gl = 0; gl < 4; ++gl)
        w_addr[gl] = base + (r >> 3) * 4096 + (r & 7) * 128 + ((c ^ (x & 3)) << 3) + ((gl * 32) ^ ((x & 12) << 3));
    const int k = lane & 7, rr = lane >> 3;
    unsigned r_addr[2];
#pragma unroll
    for (int rd = 0; rd < 2; ++rd)
        r_addr[rd] = base + rd * 4096 + rr * 128 + (((2 * k) ^ (((rd * 8 + rr) >> 1) << 1)) << 3);
    const int col0 = (SWIGLU ? t.n0 + wn * (TN / 2) : t.n0 + wn * TN) + k * 8;
    // unit u = 16 rows x 64 output columns; units alternate between the two halves of the scratch, and the
    // next unit is converted and written while the reads of the current one are in flight
    auto convert_write = [&](int u) {
        const int i = u / NU, h = u % NU;
#pragma unroll
        for (int gl = 0; gl < 4; ++gl) {
            const int g = h * 4 + gl;
            typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
            u32x2 v;
            if (SWIGLU) {
                float hh[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) hh[e] = swiglu(acc[i][2 * g][e], acc[i][2 * g + 1][e]);
                v = u32x2{pack_bf16(hh[0], hh[1]), pack_bf16(hh[2], hh[3])};
            } else {
                v = u32x2{pack_f16(acc[i][g][0], acc[i][g][1]), pack_f16(acc[i][g][2], acc[i][g][3])};
            }
            if ((u & 1) == 0) asm volatile("ds_write_b64 %0, %1" ::"v"(w_addr[gl]), "v"(v) : "memory");
            else asm volatile("ds_write_b64 %0, %1 offset:8192" ::"v"(w_addr[gl]), "v"(v) : "memory");
        }
    };
    convert_write(0);
#pragma unroll
    for (int u = 0; u < NUT; ++u) {
        u32x4 l0, l1;
        if ((u & 1) == 0) {
            asm volatile("ds_read_b128 %0, %1" : "=v"(l0) : "v"(r_addr[0]) : "memory");
            asm volatile("ds_read_b128 %0, %1" : "=v"(l1) : "v"(r_addr[1]) : "memory");
        } else {
            asm volatile("ds_read_b128 %0, %1 offset:8192" : "=v"(l0) : "v"(r_addr[0]) : "memory");
            asm volatile("ds_read_b128 %0, %1 offset:8192" : "=v"(l1) : "v"(r_addr[1]) : "memory");
        }
        if (u + 1 < NUT) {
            convert_write(u + 1);
            // LDS operations complete in order: all but the four writes just issued are done
            asm volatile("s_waitcnt lgkmcnt(4)" : "+v"(l0), "+v"(l1)::"memory");
        } else {
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(l0), "+v"(l1)::"memory");
        }
        const int i = u / NU, h = u % NU;
        const int col = col0 + h * 64;
        const u32x4 line[2] = {l0, l1};
#pragma unroll
        for (int rd = 0; rd < 2; ++rd) {
            const int rl = wm * TM + i * 16 + rd * 8 + rr;
            if (rl < t.nrows && col < p.N)
                *reinterpret_cast<u32x4*>(out + (long)(t.row0 + rl) * p.ldo + col) = line[rd];
        }
    }
}

// K slice of a block (ksplit > 1 only in GEMM2: partial sums go to separate planes of Y, which the
// combine adds up in a fixed order).  Returns the first k tile and the number of k tiles.
template <int BK>
__device__ __forceinline__ void k_range(const GemmArgs& p, const Tile& t, int& k_first, int& nk)
{
    const int nk_all = p.K / BK;
    const int nk_per = (nk_all + t.ks - 1) / t.ks;
    k_first = t.kslice * nk_per;
    nk = max(0, min(nk_all, k_first + nk_per) - k_first);
}

// LDS tile layout shared by both kernels.  A tile row holds BK bf16 = RB bytes = CPR 16-byte chunks.  The
// LDS serves a ds_read_b128 sixteen lanes at a time across 64 banks (256 bytes = WR rows), so sixteen
// consecutive rows reading the same chunk must fall on sixteen different 16-byte bank groups: chunk c of
// row r is stored in slot c ^ ((r/WR) & (CPR-1)).  Tiles are filled by global_load_lds_dwordx4: one wave
// instruction writes 1 KiB contiguously = RPG rows, lane l -> row l/CPR, slot l%CPR, so the swizzle is
// applied to the global address each lane reads.
template <int BK>
struct Lds {
    static constexpr int RB = BK * 2, CPR = RB / 16, WR = 256 / RB, RPG = 1024 / RB;
    __device__ static __forceinline__ int lane_row(int lane) { return lane / CPR; }
    __device__ static __forceinline__ int lane_chunk(int lane, int row) { return (lane % CPR) ^ ((row / WR) & (CPR - 1)); }
    __device__ static __forceinline__ int read_swz(int lane) { return ((lane & 31) / WR) & (CPR - 1); }
};

// ------------------------------------------------------------------------------------------------
// Small-tile kernel (4 waves, 32 or 64 rows): one ring of NSTAGE (A+B) stages, tiles kt+1..kt+NSTAGE-1 in
// flight while tile kt is multiplied.  Used when experts hold few rows (decode): weight streaming bound.
// ------------------------------------------------------------------------------------------------
template <int BM, int BN, int WM, int WN, int BK, int NSTAGE, bool SWIGLU>
__global__ void __launch_bounds__(WM * WN * 64) ffn_gemm_kernel(GemmArgs p)
{
    using L = Lds<BK>;
    constexpr int TM = BM / WM, TN = BN / WN, FM = TM / 32, FN = TN / 32;
    constexpr int RB = L::RB, RPG = L::RPG;
    constexpr int STAGE = (BM + BN) * RB;
    constexpr int NW = WM * WN;
    constexpr int GROUPS = (BM + BN) / RPG;
    constexpr int LD_PER_WAVE = GROUPS / NW;
    static_assert(GROUPS % NW == 0, "loader shape");
    static_assert(!SWIGLU || (FN % 2 == 0), "gate/up tiles must pair inside a wavefront");
    extern __shared__ __attribute__((aligned(16))) char smem[];

    Tile t;
    if (!decode_tile<SWIGLU ? BN / 2 : BN, SWIGLU>(p, t)) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    int k_first, nk;
    k_range<BK>(p, t, k_first, nk);

    // wave w moves row groups w, w+NW, ... of every stage (A rows first, then B rows)
    const bf16_t* gptr[LD_PER_WAVE];
#pragma unroll
    for (int i = 0; i < LD_PER_WAVE; ++i) {
        const int row = (wave + i * NW) * RPG + L::lane_row(lane);
        const bf16_t* base = row < BM ? a_row_ptr(p, t, row) : b_row_ptr<TN, SWIGLU>(p, t, row - BM);
        gptr[i] = base + L::lane_chunk(lane, row) * 8 + (size_t)k_first * BK;
    }
    auto issue_loads = [&](int kt) {
        char* dst = smem + (kt % NSTAGE) * STAGE + wave * 1024;
#pragma unroll
        for (int i = 0; i < LD_PER_WAVE; ++i)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(gptr[i] + kt * BK),
                                             (__attribute__((address_space(3))) void*)(dst + i * NW * 1024), 16, 0, 0);
    };

    f32x16 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

#pragma unroll
    for (int q = 0; q < NSTAGE - 1; ++q)
        if (q < nk) issue_loads(q);
    const int a_off = (wm * TM + (lane & 31)) * RB;
    const int b_off = BM * RB + (wn * TN + (lane & 31)) * RB;
    const int swz = L::read_swz(lane);
    for (int kt = 0; kt < nk; ++kt) {
        // this wave's loads of tile kt have landed once at most the NSTAGE-2 younger tiles are outstanding
        if (kt + NSTAGE - 2 < nk) __builtin_amdgcn_s_waitcnt(vmcnt_imm((NSTAGE - 2) * LD_PER_WAVE));
        else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
        lds_barrier();            // every wave's part of tile kt is in LDS; nobody still reads tile kt-1's buffer
        if (kt + NSTAGE - 1 < nk) issue_loads(kt + NSTAGE - 1);
        const char* St = smem + (kt % NSTAGE) * STAGE;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
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
    lds_barrier();                                        // every wave has left the stage buffers
    store_tile_lines<FM, FN, TM, TN, SWIGLU>(p, t, acc, wm, wn, lane, smem + wave * 8192);
}

// ------------------------------------------------------------------------------------------------
// Large-tile kernel (BM x 256, 8 waves as 2 x 4), ping-pong: the two wave groups (wm = 0 / 1, one wave of
// each per SIMD) run half a step out of phase, separated by barriers: while one group issues its 16
// MFMAs for a 32-wide k step, the other reads its fragments of the next step from LDS and queues
// global->LDS loads, so every SIMD's matrix pipe always has a wave feeding it.  Group 1 starts one
// barrier late and group 0 ends one late.  k tiles of BK = 64 (full 128-byte lines per row), NSTAGE
// LDS buffers; a tile is P = BK/32 steps.
// ------------------------------------------------------------------------------------------------
template <int BM, int BK, int NSTAGE, bool SWIGLU>
__global__ void __launch_bounds__(512) ffn_gemm_pp_kernel(GemmArgs p)
{
    constexpr int BN = 256, WN = 4, NW = 8;
    using L = Lds<BK>;
    constexpr int TM = BM / 2, TN = BN / WN, FM = TM / 32, FN = TN / 32;
    constexpr int RB = L::RB, RPG = L::RPG;
    constexpr int STAGE = (BM + BN) * RB;
    constexpr int GROUPS = (BM + BN) / RPG;
    constexpr int LD_PER_WAVE = GROUPS / NW;
    constexpr int P = BK / 32;
    static_assert(GROUPS % NW == 0 && NSTAGE >= 2 && BK % 32 == 0, "loader shape");
    static_assert(NSTAGE * STAGE <= 160 * 1024, "LDS budget of one CU");
    extern __shared__ __attribute__((aligned(16))) char smem[];

    Tile t;
    if (!decode_tile<SWIGLU ? BN / 2 : BN, SWIGLU>(p, t)) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 2, wn = wave & 3;
    const int grp = wm;
    int k_first, nk;
    k_range<BK>(p, t, k_first, nk);

    const bf16_t* gptr[LD_PER_WAVE];
#pragma unroll
    for (int i = 0; i < LD_PER_WAVE; ++i) {
        const int row = (wave + i * NW) * RPG + L::lane_row(lane);
        const bf16_t* base = row < BM ? a_row_ptr(p, t, row) : b_row_ptr<TN, SWIGLU>(p, t, row - BM);
        gptr[i] = base + L::lane_chunk(lane, row) * 8 + (size_t)k_first * BK;
    }
    auto issue_loads = [&](int kt) {
        char* dst = smem + (kt % NSTAGE) * STAGE + wave * 1024;
#pragma unroll
        for (int i = 0; i < LD_PER_WAVE; ++i)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(gptr[i] + kt * BK),
                                             (__attribute__((address_space(3))) void*)(dst + i * NW * 1024), 16, 0, 0);
    };

    f32x16 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

#pragma unroll
    for (int q = 0; q < NSTAGE - 1; ++q)
        if (q < nk) issue_loads(q);
    const int a_off = (wm * TM + (lane & 31)) * RB;
    const int b_off = BM * RB + (wn * TN + (lane & 31)) * RB;
    const int swz = L::read_swz(lane);
    if (NSTAGE - 2 < nk && NSTAGE > 2) __builtin_amdgcn_s_waitcnt(vmcnt_imm((NSTAGE - 2) * LD_PER_WAVE));
    else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    lds_barrier();                                        // tile 0 is in LDS for everyone
    // Loads of a tile are issued between the MFMAs of a compute phase, one per EV MFMAs, so the texture
    // path sees a steady trickle instead of a burst that would hold the issuing wave (and with it the
    // barrier the other group waits at).  The buffer of tile kt-1 is free once both groups have read its
    // last fragments: group 1 (which runs one barrier late) refills it with tile kt+NSTAGE-1 during the last
    // compute phase of tile kt-1, group 0 during the first compute phase of tile kt.
    auto issue_one = [&](int kt, int i) {
        char* dst = smem + (kt % NSTAGE) * STAGE + wave * 1024;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(gptr[i] + kt * BK),
                                         (__attribute__((address_space(3))) void*)(dst + i * NW * 1024), 16, 0, 0);
    };
    auto main_loop = [&](auto grp_tag) {
        constexpr int GRP = decltype(grp_tag)::value;
        constexpr int NM = 2 * FM * FN;                                   // MFMAs of one compute phase
        constexpr int EV = NM / LD_PER_WAVE > 0 ? NM / LD_PER_WAVE : 1;
        static_assert(LD_PER_WAVE <= NM, "one load slot per MFMA at most");
        for (int kt = 0; kt < nk; ++kt) {
            const char* St = smem + (kt % NSTAGE) * STAGE;
            const int lt = GRP == 0 ? kt + NSTAGE - 1 : kt + NSTAGE;      // tile this wave loads during tile kt
            const bool ld = lt < nk;
#pragma unroll
            for (int ph = 0; ph < P; ++ph) {
                // -- memory phase: fragments of this step from LDS
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
                // fragments are in registers (lgkmcnt 0).  Group 1's last memory phase of tile kt is the last
                // thing before group 0 reads tile kt+1: its loads of that tile must have landed.
                if (GRP == 1 && ph == P - 1) {
                    if (NSTAGE > 2 && kt + NSTAGE - 1 < nk)
                        __builtin_amdgcn_s_waitcnt(vmcnt_lgkm0_imm((NSTAGE - 2) * LD_PER_WAVE));
                    else __builtin_amdgcn_s_waitcnt(vmcnt_lgkm0_imm(0));
                } else {
                    __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0) only
                }
                __builtin_amdgcn_sched_barrier(0);
                lds_barrier();
                __builtin_amdgcn_sched_barrier(0);
                // -- compute phase
                const bool load_phase = GRP == 0 ? ph == 0 : ph == P - 1;
                __builtin_amdgcn_s_setprio(1);
#pragma unroll
                for (int kk = 0; kk < 2; ++kk)
#pragma unroll
                    for (int i = 0; i < FM; ++i)
#pragma unroll
                        for (int j = 0; j < FN; ++j) {
                            acc[i][j] =
                                __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[kk][j], af[kk][i], acc[i][j], 0, 0, 0);
                            const int mi = (kk * FM + i) * FN + j;
                            if (load_phase && mi % EV == 0 && mi / EV < LD_PER_WAVE) {
                                __builtin_amdgcn_sched_barrier(0);
                                if (ld) issue_one(lt, mi / EV);
                                __builtin_amdgcn_sched_barrier(0);
                            }
                        }
                __builtin_amdgcn_s_setprio(0);
                // group 0's last compute phase of tile kt ends right before it reads tile kt+1
                if (GRP == 0 && ph == P - 1) {
                    if (NSTAGE > 2 && kt + NSTAGE - 1 < nk) __builtin_amdgcn_s_waitcnt(vmcnt_imm((NSTAGE - 2) * LD_PER_WAVE));
                    else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
                }
                __builtin_amdgcn_sched_barrier(0);
                lds_barrier();
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };
    if (grp == 0) {
        main_loop(std::integral_constant<int, 0>{});
        lds_barrier();
    } else {
        if (NSTAGE - 1 < nk) issue_loads(NSTAGE - 1);     // its "compute phase before tile 0"
        lds_barrier();
        main_loop(std::integral_constant<int, 1>{});
    }
    lds_barrier();                                        // every wave has left the stage buffers
    store_tile_lines<FM, FN, TM, TN, SWIGLU>(p, t, acc, wm, wn, lane, smem + wave * 8192);
}

// Tells the compiler that a pointer is the same in every lane (keeps it in scalar registers).
__device__ __forceinline__ const bf16_t* uniform_ptr(const bf16_t* ptr)
{
    const unsigned long long v = reinterpret_cast<unsigned long long>(ptr);
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v);
    const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
    return reinterpret_cast<const bf16_t*>(((unsigned long long)hi << 32) | lo);
}

// ------------------------------------------------------------------------------------------------
// Four-wave kernel (256 x 256 x 64 block tile, one wave per SIMD, wave tile 128 x 128, 16x16x32 MFMA,
// accumulators in the accumulation registers), persistent: one block per CU walks over its tiles.
// One instruction stream per SIMD feeds the matrix pipe without hand-offs: a k tile is two steps of 64
// MFMAs, and between the MFMAs of a step the wave reads the next step's fragments from LDS
// (double-buffered in registers) and issues direct global->LDS loads.  The 160 KiB of LDS hold two
// buffers for the A rows (activations, mostly L2 hits) and three for the B rows (weights, which stream
// from memory and need the longer lead).  One barrier per k tile, three quarters into its first step,
// when a wave has read its last fragments of tile kt and its loads of tile kt+1 have landed; from there
// on one load is issued every eight MFMAs: first the A rows of tile kt+2 into the buffer just left, then
// the B rows of tile kt+3.  Requests past the end of K are clamped to the last k tile (never read).
// Between output tiles: the gather indices of the next tile are fetched during the main loop, its first
// k tiles are requested before the epilogue of the current tile, so they land while that runs.
// Blocks b, b+8, ... share an XCD; block b takes the tiles xcd*chunk + slot, + slots, ... of its XCD's
// contiguous chunk, so the blocks of an XCD sweep its chunk together.
// ------------------------------------------------------------------------------------------------
// K-split tail of the persistent kernel (launches with one plane of output).  With G blocks, the first
// floor(tiles / G) * G output tiles are whole-tile work, G at a time; the `rem` tiles left over would keep
// rem of G CUs busy for a whole tile time, so each is cut along K into tail_split() slices, one block each,
// which write fp32 partial tiles that a small kernel afterwards sums in slice order.  Slices are whole k
// tiles, at least 8 of them, at most 16 per tile, and none is empty; no split when it would not pay.
__host__ __device__ inline int tail_split(int G, int rem, int nk_all)
{
    if (rem <= 0) return 1;
    int sl = G / rem;
    sl = sl < 16 ? sl : 16;
    sl = sl < nk_all / 8 ? sl : nk_all / 8;
    if (sl <= 1) return 1;
    const int nk_per = (nk_all + sl - 1) / sl;
    sl = (nk_all + nk_per - 1) / nk_per;
    // Worth it?  In units of one k tile's time (about 1.4 us): a whole tile costs nk_all + 5, the tail saves
    // (1 - 1/sl) of that, and costs about 7 for its launches plus 1/8 per partial tile written and read back.
    return (nk_all + 5) * (sl - 1) > sl * (rem * sl / 8 + 7) ? sl : 1;
}

// Tile L of the launch's tile order -> its row tile and column tile: super-tiles of group_m M tiles x all N
// tiles, M fastest.
__device__ __forceinline__ void tile_coords(const GemmArgs& p, int n_mt, int L, int& mt, int& nt)
{
    const int gspan = p.group_m * p.n_ntiles;
    const int gi = L / gspan, rem = L - gi * gspan;
    const int mt_first = gi * p.group_m;
    const int gsz = min(p.group_m, n_mt - mt_first);
    nt = rem / gsz;
    mt = mt_first + (rem - nt * gsz);
}

// Left-over tiles that are not cut along K: when there are at most G/2 of them, each is cut in two along N
// instead (two blocks, 256 rows x half the columns each: no partial sums, half a tile time).
__host__ __device__ inline bool tail_halves(int G, int rem, int nk_all)
{
    return rem > 0 && 2 * rem <= G && nk_all >= 8 && tail_split(G, rem, nk_all) == 1;
}

// What a block of the persistent kernel needs to know about the launch as a whole: computed once per block
// (the divisions in it would otherwise be repeated for every tile).
struct Sched {
    int n_mt, tiles;
    int chunk;                                  // whole tiles per XCD (MODE 0 without scratch: tiles x K slices per XCD)
    int t_full, rem;                            // tiles in full rounds, tiles left over
    int sl;                                     // K slices per left-over tile (1: not cut along K)
    int halves;                                 // left-over tiles are cut in two along N
};

template <int MODE>
__device__ __forceinline__ Sched make_sched(const GemmArgs& p, int slots)
{
    Sched sc;
    sc.n_mt = p.table[0];
    sc.tiles = sc.n_mt * p.n_ntiles;
    if (MODE == 0 && p.partial == nullptr) {
        sc.chunk = (sc.tiles * p.ksplit + 7) >> 3;
        sc.t_full = sc.tiles; sc.rem = 0; sc.sl = 1; sc.halves = 0;
    } else {
        const int G = slots * 8;
        sc.t_full = sc.tiles / G * G;
        sc.chunk = sc.t_full >> 3;
        sc.rem = sc.tiles - sc.t_full;
        sc.sl = tail_split(G, sc.rem, p.K / 64);
        sc.halves = tail_halves(G, sc.rem, p.K / 64) ? 1 : 0;
    }
    return sc;
}

// MODE 0: whole tiles (the main launch); 1: K slices of the left-over tiles; 2: column halves of them.
template <int BNC, int MODE>
__device__ __forceinline__ bool decode_tile_at(const GemmArgs& p, const Sched& sc, int xcd, int bi, int slots, Tile& t)
{
    const int n_mt = sc.n_mt;
    int L;
    t.ks = p.ksplit;
    t.part = -1;
    t.kslice = 0;
    t.half = 0;
    if (MODE == 0 && p.partial == nullptr) {
        const int total = sc.tiles * p.ksplit;
        if (bi >= sc.chunk) return false;
        const int Lfull = xcd * sc.chunk + bi;
        if (Lfull >= total) return false;
        if (p.ksplit > 1) {
            t.kslice = Lfull / sc.tiles;
            L = Lfull - t.kslice * sc.tiles;
        } else {
            L = Lfull;
        }
    } else {
        // Whole tiles: every XCD sweeps its contiguous chunk (a multiple of its `slots` blocks), then one more
        // round for the tiles left over if they are not cut.  Cut tiles are the work of the other two
        // instantiations, launched next, one piece per block: K slices slice-major, so that the blocks of an
        // XCD work on the same slices of K; column halves side by side, so that they share the A rows in L2.
        if (MODE == 0 && bi < sc.chunk) {
            L = xcd * sc.chunk + bi;
        } else {
            const int round = MODE == 0 ? bi - sc.chunk : bi;
            if (round >= slots) return false;
            const int c = xcd * slots + round;
            if (MODE == 0) {
                if (sc.sl > 1 || sc.halves || c >= sc.rem) return false;
                L = sc.t_full + c;
            } else if (MODE == 1) {
                if (sc.sl <= 1 || c >= sc.rem * sc.sl) return false;
                const int pz = c / sc.rem, j = c - pz * sc.rem;
                L = sc.t_full + j;
                t.kslice = pz; t.ks = sc.sl; t.part = j * sc.sl + pz;
            } else {
                if (!sc.halves || c >= 2 * sc.rem) return false;
                L = sc.t_full + (c >> 1);
                t.half = c & 1;
            }
        }
    }
    int mt;
    tile_coords(p, n_mt, L, mt, t.nt);
    const int4 te = reinterpret_cast<const int4*>(p.table + 4)[mt];
    t.unit = te.x; t.row0 = te.y; t.nrows = te.z;
    const int src = t.unit < p.m ? 0 : (t.unit < p.m + p.G ? 1 : 2);
    const int widx = t.unit - (src == 0 ? 0 : (src == 1 ? p.m : p.m + p.G));
    const size_t wsz = (size_t)p.N * p.K;
    t.Wa = (src == 0 ? p.wa0 : (src == 1 ? p.wa1 : p.wa2)) + (size_t)widx * wsz;
    t.Wb = p.wb0 ? (src == 0 ? p.wb0 : (src == 1 ? p.wb1 : p.wb2)) + (size_t)widx * wsz : nullptr;
    t.n0 = t.nt * BNC;
    return true;
}

// fp32 partial tile of a K slice: 256 x 256 floats, row-major, no masking (the scratch holds whole tiles)
template <int FM, int FN, int TM, int TN>
__device__ __forceinline__ void store_partial16(float* __restrict__ dst, const f32x4 (&acc)[FM][FN], int wm, int wn,
                                                int lane)
{
#pragma unroll
    for (int i = 0; i < FM; ++i) {
        float* drow = dst + (wm * TM + i * 16 + (lane & 15)) * 256 + wn * TN + 4 * (lane >> 4);
#pragma unroll
        for (int j = 0; j < FN; ++j)
            *reinterpret_cast<float4*>(drow + j * 16) = make_float4(acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]);
    }
}

// Sums the partial tiles of the K-split tail in slice order and writes the output rows: GEMM2 as they are
// (half precision), GEMM1 through SwiGLU (bf16; tile columns alternate 16 gate and 16 up columns of the same
// 16 outputs).  A block handles 4 rows of one tail tile at a time, a thread 4 tile columns; G is the grid of
// the GEMM launch this one follows.
template <bool SWIGLU>
__global__ void __launch_bounds__(256) gemm_tail_sum_kernel(GemmArgs p, int G)
{
    const int n_mt = p.table[0];
    const int tiles = n_mt * p.n_ntiles;
    const int t_full = tiles / G * G, rem = tiles - t_full;
    const int sl = tail_split(G, rem, p.K / 64);
    if (sl <= 1) return;
    const int c = (threadIdx.x & 63) * 4;
    if (SWIGLU && ((c >> 4) & 1)) return;                 // up columns are read by the thread of their gate columns
    // how many tiles are left over only the device knows: a fixed grid strides over (tile, 4-row strip)
    for (int item = blockIdx.x; item < rem * 64; item += gridDim.x) {
        const int j = item >> 6, strip = item & 63;
        int mt, nt;
        tile_coords(p, n_mt, t_full + j, mt, nt);
        const int4 te = reinterpret_cast<const int4*>(p.table + 4)[mt];
        const int row0 = te.y, nrows = te.z;
        const int r = strip * 4 + (threadIdx.x >> 6);
        if (r >= nrows) continue;
        // output column of tile column c
        const int ocol = SWIGLU ? nt * 128 + ((c >> 7) * 4 + ((c & 127) >> 5)) * 16 + (c & 15) : nt * 256 + c;
        if (ocol >= p.N) continue;
        const float* src = p.partial + (size_t)j * sl * 65536 + r * 256 + c;
        constexpr int NV = SWIGLU ? 2 : 1;
        float4 v[NV][16];                                     // tail_split() yields at most 16 slices
#pragma unroll
        for (int pz = 0; pz < 16; ++pz)
            if (pz < sl) {
#pragma unroll
                for (int h = 0; h < NV; ++h) v[h][pz] = *reinterpret_cast<const float4*>(src + (size_t)pz * 65536 + h * 16);
            }
        float4 a[NV];
#pragma unroll
        for (int h = 0; h < NV; ++h) {
            a[h] = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int pz = 0; pz < 16; ++pz)
                if (pz < sl) { a[h].x += v[h][pz].x; a[h].y += v[h][pz].y; a[h].z += v[h][pz].z; a[h].w += v[h][pz].w; }
        }
        unsigned short* orow = reinterpret_cast<unsigned short*>(p.out) + (long)(row0 + r) * p.ldo + ocol;
        if (SWIGLU)
            *reinterpret_cast<uint2*>(orow) = make_uint2(pack_bf16(swiglu(a[0].x, a[NV - 1].x), swiglu(a[0].y, a[NV - 1].y)),
                                                         pack_bf16(swiglu(a[0].z, a[NV - 1].z), swiglu(a[0].w, a[NV - 1].w)));
        else
            *reinterpret_cast<uint2*>(orow) = make_uint2(pack_f16(a[0].x, a[0].y), pack_f16(a[0].z, a[0].w));
    }
}

template <bool SWIGLU, int MODE>
__device__ __forceinline__ void w4_block(const GemmArgs& p, const int block, const int n_blocks)
{
    constexpr int BM = 256, BN = 256, BK = 64, NW = 4;
    using L = Lds<BK>;
    // MODE 2 (column half of a tile): the wave tile is 128 x 64, half the MFMAs and half the B rows per k tile;
    // loads, buffers, barrier and the order of the load slots are those of the full tile at half the spacing
    constexpr int TM = 128, TN = MODE == 2 ? 64 : 128, FM = TM / 16, FN = TN / 16;
    constexpr int RB = L::RB, RPG = L::RPG;
    constexpr int ABUF = BM * RB, BBUF = BN * RB;        // 32 KiB each
    constexpr int B_BASE = 2 * ABUF;
    constexpr int HL = BM / RPG / NW;                    // 8 loads of A rows per wave and k tile
    constexpr int HLB = MODE == 2 ? HL / 2 : HL;         // and 8 (column half: 4) of B rows
    constexpr int NM = FM * FN;                          // MFMAs of one step (64; column half: 32)
    constexpr int EV = NM / 8;                           // MFMAs per load slot
    constexpr int BAR = 6 * EV;                          // the barrier: three quarters into step 0
    constexpr int NRD = 2 * (FM + FN);                   // fragment reads of a step, one per two MFMAs
    static_assert(NRD <= BAR, "the fragment reads of a step end before its barrier");
    constexpr int BNC = SWIGLU ? BN / 2 : BN;
    // GEMM1 gathers its A rows (tokens of the unit); GEMM2 reads consecutive rows of H, which is padded by
    // one tile of rows so that the rows of a ragged tile need no clamping.
    constexpr bool GATHER = SWIGLU;
    constexpr int NOA = GATHER ? HL : 1, NBA = GATHER ? 1 : HL;
    static_assert(2 * ABUF + 3 * BBUF <= 160 * 1024, "LDS budget of one CU");
    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int xcd = block & 7, slots = n_blocks >> 3;
    int bi = block >> 3;
    const Sched sc = make_sched<MODE>(p, slots);
    Tile t;
    if (!decode_tile_at<BNC, MODE>(p, sc, xcd, bi, slots, t)) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);
    // wave tile: rows wm * 128 .., B-tile rows wn * TN ..  (column half h of a tile: the 64-row quarters 2h, 2h+1)
    const int wm = wave >> 1, wn = MODE == 2 ? 2 * t.half + (wave & 1) : (wave & 1);
    const int q0 = MODE == 2 ? (HL / 2) * __builtin_amdgcn_readfirstlane(t.half) : 0;   // first B load of the half

    // Load i of a wave covers rows (wave + 4 i) * 8 .. + 8 of the A (or B) tile.  An address is a
    // wave-uniform base (scalar registers) plus a 32-bit lane offset: gathered A rows have one lane offset
    // per load from the start of A; consecutive A rows (GEMM2) and the B rows of a load are 8 consecutive
    // rows, so one lane offset serves all loads and the base moves.  The swizzle term ((row/2)&7) is the
    // same for every load of a lane because (wave + 4 i) * 4 == 4 * (wave & 1) (mod 8).
    const int r8 = lane >> 3;
    const int csw = (lane & 7) ^ ((((wave & 1) << 2) + (r8 >> 1)) & 7);
    const unsigned offB = (unsigned)((long)r8 * p.K * 2 + csw * 16);
    unsigned offA[NOA];
    const bf16_t* baseA[NBA];
    const bf16_t* baseB[HLB];
    int nk = 0, last = 0;

    // Source rows of the 64 A rows this wave loads per k tile (gathered A only), one per lane: lane k holds
    // the row behind load k/8, row k%8; the loads pick theirs up with a cross-lane read in setup_tile.
    auto gather_rows = [&](const Tile& tt) -> int {
        const int row = (wave + (lane >> 3) * NW) * RPG + (lane & 7);
        const int r = row < tt.nrows ? row : 0;          // ragged tiles re-read row 0; such rows are never stored
        return p.gather ? p.gather[tt.row0 + r] : tt.row0 + r;
    };
    auto setup_tile = [&](const Tile& tt, int grows) {
        int k_first;
        k_range<BK>(p, tt, k_first, nk);
        // an empty K slice (more planes than k tiles): the first loads are still issued, from k tile 0, and
        // never read; the tile is stored as zeros
        if (nk <= 0) k_first = 0;
        last = nk > 0 ? nk - 1 : 0;
        if (GATHER) {
#pragma unroll
            for (int i = 0; i < HL; ++i)
                offA[GATHER ? i : 0] = (unsigned)((long)__shfl(grows, i * 8 + r8) * p.lda * 2 + csw * 16);
            baseA[0] = uniform_ptr(p.A + (size_t)k_first * BK);
        } else {
            offA[0] = (unsigned)((long)r8 * p.lda * 2 + csw * 16);
#pragma unroll
            for (int i = 0; i < HL; ++i)
                baseA[GATHER ? 0 : i] =
                    uniform_ptr(p.A + (size_t)(tt.row0 + (wave_s + i * NW) * RPG) * p.lda + (size_t)k_first * BK);
        }
#pragma unroll
        for (int q = 0; q < HLB; ++q) {
            const int g = wave_s + NW * (q + q0);         // 8-row group inside the B tile, 0..31
            const bf16_t* W = tt.Wa;
            int col0;
            if (SWIGLU) {
                const int w_n = g >> 4, j16 = (g & 15) >> 1;
                col0 = tt.n0 + (w_n * 4 + (j16 >> 1)) * 16 + (g & 1) * 8;
                if (j16 & 1) W = tt.Wb;
            } else {
                col0 = tt.n0 + g * 8;
            }
            col0 = min(col0, p.N - 8);                    // columns past N are never stored
            baseB[q] = uniform_ptr(W + (size_t)col0 * p.K + (size_t)k_first * BK);
        }
    };
    // one direct load: 8 rows x 128 bytes into 1 KiB of LDS
    auto load_a = [&](int i, int tile, int abuf) {
        const char* src = reinterpret_cast<const char*>(baseA[GATHER ? 0 : i] + (long)tile * BK) + offA[GATHER ? i : 0];
        char* dst = smem + abuf * ABUF + (wave_s + i * NW) * 1024;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                         (__attribute__((address_space(3))) void*)dst, 16, 0, 0);
    };
    auto load_b = [&](int q, int tile, int bbuf) {
        const char* src = reinterpret_cast<const char*>(baseB[q] + (long)tile * BK) + offB;
        char* dst = smem + B_BASE + bbuf * BBUF + (wave_s + (q + q0) * NW) * 1024;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                         (__attribute__((address_space(3))) void*)dst, 16, 0, 0);
    };
    // first k tiles of an output tile: tiles 0 and 1, and the first two B loads of tile 2
    auto issue_prologue = [&]() {
#pragma unroll
        for (int i = 0; i < HL; ++i) load_a(i, 0, 0);
#pragma unroll
        for (int q = 0; q < HLB; ++q) load_b(q, 0, 0);
#pragma unroll
        for (int i = 0; i < HL; ++i) load_a(i, min(1, last), 1);
#pragma unroll
        for (int q = 0; q < HLB; ++q) load_b(q, min(1, last), 1);
#pragma unroll
        for (int q = 0; q < 2; ++q) load_b(q, min(2, last), 2);
    };

    const int a_off = (wm * TM + (lane & 15)) * RB;
    const int b_off = B_BASE + (wn * TN + (lane & 15)) * RB;
    const int swz = ((lane & 15) / L::WR) & (L::CPR - 1);
    bf16x8 fa[2][FM], fb[2][FN];
    auto read_frag_a = [&](int abuf, int half, int i, int buf) {
        const int sw = ((half * 4 + (lane >> 4)) ^ swz) << 4;
        fa[buf][i] = *reinterpret_cast<const bf16x8*>(smem + abuf * ABUF + a_off + i * 16 * RB + sw);
    };
    auto read_frag_b = [&](int bbuf, int half, int j, int buf) {
        const int sw = ((half * 4 + (lane >> 4)) ^ swz) << 4;
        fb[buf][j] = *reinterpret_cast<const bf16x8*>(smem + bbuf * BBUF + b_off + j * 16 * RB + sw);
    };

    setup_tile(t, GATHER ? gather_rows(t) : 0);
    issue_prologue();

    for (;;) {
        // the next output tile of this block, or this one again when there is none (its index load is
        // issued either way, so the number of loads in flight does not depend on it)
        Tile tn;
        const bool has_next = decode_tile_at<BNC, MODE>(p, sc, xcd, bi + slots, slots, tn);
        if (!has_next) tn = t;
        const int gnext = GATHER ? gather_rows(tn) : 0;

        f32x4 acc[FM][FN];
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.0f;
        // pin the accumulators to the accumulation registers on both sides of the loop: left to itself the
        // register allocator sometimes trades them against the fragments and spills
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j) asm volatile("" : "+a"(acc[i][j]));

        if (nk > 0) {
            // k tile 0 has landed once at most the HL + HLB + 2 younger loads of the first batch, and the index
            // load after them, are in flight (stores of the previous epilogue only make this wait longer)
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(HL + HLB + 2 + (GATHER ? 1 : 0)));
            lds_barrier();
#pragma unroll
            for (int i = 0; i < FM; ++i) read_frag_a(0, 0, i, 0);
#pragma unroll
            for (int j = 0; j < FN; ++j) read_frag_b(0, 0, j, 0);
            __builtin_amdgcn_s_waitcnt(0xC07F);

            int b_cur = 0;                                // B buffer of tile kt (kt mod 3)
            for (int kt = 0; kt < nk; ++kt) {
                const int a_cur = kt & 1;
                const int b_nxt = b_cur == 2 ? 0 : b_cur + 1;
                const int b_nn = b_nxt == 2 ? 0 : b_nxt + 1;          // B buffer of tile kt+2 (= of tile kt-1)
                const int t2 = min(kt + 2, last), t3 = min(kt + 3, last);
#pragma unroll
                for (int st = 0; st < 2; ++st) {
                    // fragments of the next step: second half of this tile, or first half of the next tile
                    const int a_rd = st == 0 ? a_cur : a_cur ^ 1;
                    const int b_rd = st == 0 ? b_cur : b_nxt;
#pragma unroll
                    for (int i = 0; i < FM; ++i)
#pragma unroll
                        for (int j = 0; j < FN; ++j) {
                            const int mi = i * FN + j;
                            if (st == 0 && mi == BAR) {
                                // my reads of tile kt are done (both its buffers may be refilled) and my loads
                                // of tile kt+1 have landed: everything but the HLB youngest requests
                                __builtin_amdgcn_sched_barrier(0);
                                __builtin_amdgcn_s_waitcnt(vmcnt_lgkm0_imm(HLB));
                                lds_barrier();
                                __builtin_amdgcn_sched_barrier(0);
                            }
                            acc[i][j] =
                                __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[st][j], fa[st][i], acc[i][j], 0, 0, 0);
                            if (mi < NRD && (mi & 1) == 0) {      // fragment reads, one per two MFMAs
                                const int r = mi >> 1;
                                __builtin_amdgcn_sched_barrier(0);
                                if (r < FN) read_frag_b(b_rd, st ^ 1, r, st ^ 1);
                                else read_frag_a(a_rd, st ^ 1, r - FN, st ^ 1);
                                __builtin_amdgcn_sched_barrier(0);
                            }
                            // One direct load per slot of EV MFMAs (eight for the full tile: closer together they
                            // queue up in the texture path and hold the wave).  After the barrier: the A rows of
                            // tile kt+2 into the A buffer just left, then the B rows of tile kt+3 into tile kt's
                            // B buffer, all but the first two of them during the first three quarters of the
                            // next tile's first step.
                            if (mi % EV == 0) {
                                const int slot = mi / EV;
                                __builtin_amdgcn_sched_barrier(0);
                                if (st == 0 && slot < HLB - 2) load_b(slot + 2, t2, b_nn);
                                if (st == 0 && slot >= 6) load_a(slot - 6, t2, a_cur);
                                if (st == 1 && slot < 6) load_a(slot + 2, t2, a_cur);
                                if (st == 1 && slot >= 6) load_b(slot - 6, t3, b_cur);
                                __builtin_amdgcn_sched_barrier(0);
                            }
                        }
                    __builtin_amdgcn_sched_barrier(0);
                    __builtin_amdgcn_s_waitcnt(0xC07F);   // next step's fragments are in registers
                    __builtin_amdgcn_sched_barrier(0);
                }
                b_cur = b_nxt;
            }
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));     // clamped tail requests still target this block's LDS
            lds_barrier();                                // everyone has left the LDS buffers
        }
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j) asm volatile("" : "+a"(acc[i][j]));

        // the index load has returned by now (all loads were waited for above); saying so here keeps the
        // compiler from waiting for it, and with it for the next tile's first loads, inside the epilogue
        asm volatile("" ::"v"(gnext));
        const Tile tcur = t;
        if (has_next) {
            // request the first k tiles of the next output tile, then let them land behind the epilogue
            t = tn;
            bi += slots;
            setup_tile(t, gnext);
            issue_prologue();
        }
        {
            // lane-derived epilogue values are recomputed per tile instead of living through the main loop
            int lane_e;
            asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(lane_e));
            const int wn_e = MODE == 2 ? q0 / 2 + (wave_s & 1) : (wave_s & 1);
            if constexpr (MODE == 1)
                store_partial16<FM, FN, TM, TN>(p.partial + (size_t)tcur.part * 65536, acc, wave_s >> 1, wn_e, lane_e);
            else if constexpr (MODE == 0)
                store_tile16_lines<FM, FN, TM, TN, SWIGLU>(p, tcur, acc, wave_s >> 1, wn_e, lane_e,
                                                           smem + B_BASE + 2 * BBUF + (wave_s + 2 * NW) * 1024);
            else
                store_tile16<FM, FN, TM, TN, SWIGLU>(p, tcur, acc, wave_s >> 1, wn_e, lane_e);
        }
        if (!has_next) break;
    }
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
}

// One launch: G blocks (one per CU) for the whole tiles and, where the left-over tiles may be cut (p.partial
// set), 2 G more behind them: G for column halves, G for K slices.  They are independent work, so a CU
// picks one up as soon as its block of whole tiles is done; a launch uses at most one of the two kinds
// (only the device knows which), the blocks of the other return at once.  Block id mod 8 is the XCD in all
// three ranges (G is a multiple of 8).
template <bool SWIGLU>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) ffn_gemm_w4_kernel(GemmArgs p)
{
    const int g = p.partial != nullptr ? (int)gridDim.x / 3 : (int)gridDim.x;
    const int b = blockIdx.x;
    if (b < g) w4_block<SWIGLU, 0>(p, b, g);
    else if (b < 2 * g) w4_block<SWIGLU, 2>(p, b - g, g);
    else w4_block<SWIGLU, 1>(p, b - 2 * g, g);
}

// ------------------------------------------------------------------------------------------------
// combine: one thread = 8 columns of one token; rows summed in slot order, shared experts first.
// ------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) combine_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ Y,
                                                      const int32_t* __restrict__ token_rows,
                                                      const float* __restrict__ row_weight, bf16_t* __restrict__ out,
                                                      int T, int d, int K, int Ns, int add_residual, int ksplit, long plane)
{
    const int chunks = d >> 3;
    const long gid = (long)blockIdx.x * 256 + threadIdx.x;
    if (gid >= (long)T * chunks) return;
    const int t = (int)(gid / chunks), c8 = (int)(gid - (long)t * chunks) * 8;
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.0f;
    typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
    auto add_row = [&](const bf16_t* rowp, float (&a)[8]) {                 // a row of x (bf16)
        const uint4 q = *reinterpret_cast<const uint4*>(rowp + c8);
        const unsigned int w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            a[2 * e] += __uint_as_float(w[e] << 16);
            a[2 * e + 1] += __uint_as_float(w[e] & 0xFFFF0000u);
        }
    };
    auto add_y_row = [&](const bf16_t* rowp, float (&a)[8]) {               // a row of Y (half precision)
        const uint4 q = *reinterpret_cast<const uint4*>(rowp + c8);
        const unsigned int w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const f16x2 h = __builtin_bit_cast(f16x2, w[e]);
            a[2 * e] += (float)h[0];
            a[2 * e + 1] += (float)h[1];
        }
    };
    // The token's rows in the order of the sum (shared experts first, then the TopK entries), eight at a time:
    // their indices and weights first, then all their loads, then the additions in order, so that a thread keeps
    // several 16-byte loads in flight instead of one.  A row's K-split planes are summed first, then the sum is
    // multiplied by the row's weight.
    if (add_residual) add_row(x + (long)t * d, acc);
    const int slots = K + Ns;
    const int32_t* tr = token_rows + (long)t * slots;
    constexpr int CB = 8;                                 // rows in flight per thread
    for (int s0 = 0; s0 < slots; s0 += CB) {
        int r[CB];
        float w[CB];
#pragma unroll
        for (int u = 0; u < CB; ++u) {
            const int sp = s0 + u;
            r[u] = sp < slots ? tr[sp < Ns ? K + sp : sp - Ns] : -1;
        }
#pragma unroll
        for (int u = 0; u < CB; ++u) w[u] = r[u] >= 0 ? row_weight[r[u]] : 0.0f;
        if (ksplit == 1) {
            uint4 q[CB];
#pragma unroll
            for (int u = 0; u < CB; ++u)
                q[u] = r[u] >= 0 ? *reinterpret_cast<const uint4*>(Y + (long)r[u] * d + c8) : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
            for (int u = 0; u < CB; ++u) {
                if (r[u] < 0) continue;
                const unsigned int v[4] = {q[u].x, q[u].y, q[u].z, q[u].w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const f16x2 h = __builtin_bit_cast(f16x2, v[e]);
                    acc[2 * e] += w[u] * (float)h[0];
                    acc[2 * e + 1] += w[u] * (float)h[1];
                }
            }
        } else {
#pragma unroll
            for (int u = 0; u < CB; ++u) {
                if (r[u] < 0) continue;
                float part[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) part[e] = 0.0f;
                for (int pz = 0; pz < ksplit; ++pz) add_y_row(Y + pz * plane + (long)r[u] * d, part);
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[e] += w[u] * part[e];
            }
        }
    }
    uint4 o;
    o.x = pack_bf16(acc[0], acc[1]);
    o.y = pack_bf16(acc[2], acc[3]);
    o.z = pack_bf16(acc[4], acc[5]);
    o.w = pack_bf16(acc[6], acc[7]);
    *reinterpret_cast<uint4*>(out + (long)t * d + c8) = o;
}

// ------------------------------------------------------------------------------------------------
// Launchers.  Kernels that need more dynamic LDS than the default limit get the attribute once per device in
// init_ffn_kernels (never inside a launch path: the call is not allowed under stream capture).
// ------------------------------------------------------------------------------------------------
template <int BM, int BN, int WM, int WN, int BK, int NSTAGE>
constexpr int small_lds() { return NSTAGE * (BM + BN) * BK * 2; }
constexpr int kPpLds = 3 * (128 + 256) * 64 * 2;
constexpr int kW4Lds = 160 * 1024;

template <typename Kern>
static hipError_t set_lds(Kern kern, int lds)
{
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
}

hipError_t init_ffn_kernels()
{
    hipError_t e;
    if ((e = set_lds(ffn_gemm_kernel<64, 256, 1, 4, 64, 3, true>, small_lds<64, 256, 1, 4, 64, 3>())) != hipSuccess) return e;
    if ((e = set_lds(ffn_gemm_kernel<64, 256, 1, 4, 64, 3, false>, small_lds<64, 256, 1, 4, 64, 3>())) != hipSuccess) return e;
    if ((e = set_lds(ffn_gemm_kernel<32, 256, 1, 4, 64, 4, true>, small_lds<32, 256, 1, 4, 64, 4>())) != hipSuccess) return e;
    if ((e = set_lds(ffn_gemm_kernel<32, 256, 1, 4, 64, 4, false>, small_lds<32, 256, 1, 4, 64, 4>())) != hipSuccess) return e;
    if ((e = set_lds(ffn_gemm_pp_kernel<128, 64, 3, true>, kPpLds)) != hipSuccess) return e;
    if ((e = set_lds(ffn_gemm_pp_kernel<128, 64, 3, false>, kPpLds)) != hipSuccess) return e;
    if ((e = set_lds(ffn_gemm_w4_kernel<true>, kW4Lds)) != hipSuccess) return e;
    if ((e = set_lds(ffn_gemm_w4_kernel<false>, kW4Lds)) != hipSuccess) return e;
    return hipSuccess;
}

template <typename Kern>
static hipError_t launch_tiles(Kern kern, int threads, int lds, int bn_cols, GemmArgs a, int max_mtiles, hipStream_t s)
{
    a.n_ntiles = ceil_div(a.N, bn_cols);
    const long total = (long)max_mtiles * a.n_ntiles * a.ksplit;
    const int grid = (int)((total + 7) / 8 * 8);
    kern<<<grid, threads, lds, s>>>(a);
    return hipGetLastError();
}

template <int BM, int BN, int WM, int WN, int BK, int NSTAGE, bool SWIGLU>
static hipError_t launch_small(const GemmArgs& a, int max_mtiles, hipStream_t s)
{
    constexpr int LDS = small_lds<BM, BN, WM, WN, BK, NSTAGE>();
    static_assert(LDS <= 160 * 1024, "LDS budget of one CU");
    return launch_tiles(ffn_gemm_kernel<BM, BN, WM, WN, BK, NSTAGE, SWIGLU>, WM * WN * 64, LDS, SWIGLU ? BN / 2 : BN, a,
                        max_mtiles, s);
}

template <bool SWIGLU>
static hipError_t launch_pp(const GemmArgs& a, int max_mtiles, hipStream_t s)
{
    return launch_tiles(ffn_gemm_pp_kernel<128, 64, 3, SWIGLU>, 512, kPpLds, SWIGLU ? 128 : 256, a, max_mtiles, s);
}

template <bool SWIGLU>
static hipError_t launch_w4(const GemmArgs& a, int max_mtiles, int n_cu, hipStream_t s)
{
    auto kern = ffn_gemm_w4_kernel<SWIGLU>;
    GemmArgs g = a;
    g.n_ntiles = ceil_div(g.N, SWIGLU ? 128 : 256);
    const long total = (long)max_mtiles * g.n_ntiles * g.ksplit;
    // one block per CU (the LDS footprint allows no second one), a multiple of 8 so every XCD has the same
    // number of blocks; fewer when there cannot be that many tiles
    const int grid = (int)std::min<long>((total + 7) / 8 * 8, std::max(8, n_cu / 8 * 8));
    if (g.ksplit != 1 || grid > g.partial_cap) g.partial = nullptr;
    // at most grid - 1 tiles are left over after the last full round of `grid` tiles
    const int max_tail = (int)std::min<long>(total, grid - 1);
    if (max_tail <= 0) g.partial = nullptr;
    kern<<<g.partial ? 3 * grid : grid, 256, kW4Lds, s>>>(g);
    if (g.partial) gemm_tail_sum_kernel<SWIGLU><<<std::min(max_tail * 64, 2048), 256, 0, s>>>(g, grid);
    return hipGetLastError();
}

template <bool SWIGLU>
static hipError_t dispatch_gemm(int bm, const GemmArgs& a, int max_mtiles, int n_cu, hipStream_t s)
{
    switch (bm) {
        case 256: return launch_w4<SWIGLU>(a, max_mtiles, n_cu, s);
        case 128: return launch_pp<SWIGLU>(a, max_mtiles, s);
        case 64: return launch_small<64, 256, 1, 4, 64, 3, SWIGLU>(a, max_mtiles, s);
        default: return launch_small<32, 256, 1, 4, 64, 4, SWIGLU>(a, max_mtiles, s);
    }
}

hipError_t launch_ffn(const Dims& D, int u_lo, int u_hi, int Fdim, const TilePlan& plan, const bf16_t* x,
                      const int32_t* gather, const int32_t* unit_cnt, const int32_t* unit_off,
                      const FfnWeights& experts, const FfnWeights& united, const FfnWeights& shared,
                      int32_t* table, bool table_built, bf16_t* H, bf16_t* Y, float* partial, hipStream_t s)
{
    DeviceInfo dev;
    hipError_t e = ensure_device_init(&dev);
    if (e != hipSuccess) return e;
    const int n_units = u_hi - u_lo;
    if (!table_built) {
        ProfScope ps(MOE_STAGE_TILES, s);
        TileJobs jobs;
        jobs.n = 1; jobs.cap = D.tile_cap;
        jobs.job[0].u_lo = u_lo; jobs.job[0].u_hi = u_hi; jobs.job[0].plan = plan; jobs.job[0].table = table;
        jobs.job[1] = jobs.job[0];
        tile_table_kernel<<<1, 64, 0, s>>>(unit_cnt, unit_off, jobs);
    }
    const int max_mtiles = (int)std::min<int64_t>(D.row_cap / plan.bm + n_units, D.tile_cap);
    GemmArgs g1;
    g1.A = x; g1.lda = D.d; g1.gather = gather; g1.table = nullptr;
    g1.wa0 = experts.w1; g1.wa1 = united.w1; g1.wa2 = shared.w1;
    g1.wb0 = experts.w3; g1.wb1 = united.w3; g1.wb2 = shared.w3;
    g1.m = D.m; g1.G = D.G; g1.N = Fdim; g1.K = D.d;
    g1.out = H; g1.ldo = D.Fmax;
    g1.n_ntiles = 0;                            // set by the launcher from its tile width
    g1.group_m = tuning().group_m ? tuning().group_m : (plan.bm == 256 ? 8 : 4);
    g1.ksplit = 1; g1.plane = 0;
    g1.out32 = nullptr; g1.partial = partial; g1.partial_cap = D.tail_blocks;
    g1.table = table;
    {
        ProfScope ps(MOE_STAGE_GEMM1, s);
        e = dispatch_gemm<true>(plan.bm, g1, max_mtiles, dev.n_cu, s);
        if (e != hipSuccess) return e;
    }
    GemmArgs g2;
    g2.A = H; g2.lda = D.Fmax; g2.gather = nullptr; g2.table = nullptr;
    g2.wa0 = experts.w2; g2.wa1 = united.w2; g2.wa2 = shared.w2;
    g2.wb0 = g2.wb1 = g2.wb2 = nullptr;
    g2.m = D.m; g2.G = D.G; g2.N = D.d; g2.K = Fdim;
    g2.out = Y; g2.ldo = D.d;
    g2.n_ntiles = 0;
    g2.group_m = g1.group_m;
    g2.ksplit = D.ksplit; g2.plane = D.y_plane;
    g2.out32 = nullptr; g2.partial = partial; g2.partial_cap = D.tail_blocks;
    g2.table = table;
    {
        ProfScope ps(MOE_STAGE_GEMM2, s);
        e = dispatch_gemm<false>(plan.bm, g2, max_mtiles, dev.n_cu, s);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// ------------------------------------------------------------------------------------------------
// Plain GEMM for the distillation trainer: C[M][N] (fp32) = A[M][K] . B[N][K]^T, bf16 operands, through
// the 64-row kernel with a one-unit tile table (table: 4 + 4 * ceil(M/64) ints of scratch).
// ------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) plain_table_kernel(int32_t* __restrict__ table, int M)
{
    const int n_mt = (M + 63) / 64;
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i == 0) { table[0] = n_mt; table[1] = 0; table[2] = 0; table[3] = 0; }
    if (i < n_mt) reinterpret_cast<int4*>(table + 4)[i] = make_int4(0, i * 64, min(64, M - i * 64), 0);
}

hipError_t launch_plain_gemm(const bf16_t* A, const bf16_t* B, int M, int N, int K, float* C, int32_t* table,
                             hipStream_t s)
{
    const int n_mt = ceil_div(M, 64);
    plain_table_kernel<<<ceil_div(n_mt, 256), 256, 0, s>>>(table, M);
    GemmArgs g;
    g.A = A; g.lda = K; g.gather = nullptr; g.table = table;
    g.wa0 = B; g.wa1 = g.wa2 = nullptr; g.wb0 = g.wb1 = g.wb2 = nullptr;
    g.m = 1; g.G = 0; g.N = N; g.K = K;
    g.out = nullptr; g.ldo = N; g.n_ntiles = 0; g.group_m = 4; g.ksplit = 1; g.plane = 0;
    g.out32 = C; g.partial = nullptr; g.partial_cap = 0; 
    return launch_small<64, 256, 1, 4, 64, 3, false>(g, n_mt, s);
}

hipError_t launch_combine(const Dims& D, const bf16_t* x, const bf16_t* Y, const int32_t* token_rows,
                          const float* row_weight, bf16_t* out, hipStream_t s)
{
    ProfScope ps(MOE_STAGE_COMBINE, s);
    const long n = (long)D.T * (D.d / 8);
    combine_kernel<<<(int)((n + 255) / 256), 256, 0, s>>>(x, Y, token_rows, row_weight, out, D.T, D.d, D.K, D.Ns, D.add_residual,
                                                          D.ksplit, D.y_plane);
    return hipGetLastError();
}

}  // namespace bmoe
