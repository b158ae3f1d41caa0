// Internal declarations shared by the translation units of libbrownout_moe.so.
// Host-side launchers only; every kernel lives in the .hip file that launches it.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/brownout_moe.h"

namespace bmoe {

typedef __bf16 bf16_t;

constexpr int kMaxExperts = 256;  // m
constexpr int kMaxTopK = 32;      // K
constexpr int kMaxShared = 8;     // N_s
constexpr int kMaxUnits = kMaxExperts + kMaxExperts + kMaxShared;  // U
constexpr int kSegTokens = 64;    // tokens per routing segment (one wavefront)
constexpr int kSmallSegs = 16;    // batches of at most this many segments are routed by ONE block
constexpr int kFewExpertsTokens = 2048;   // at most 16 experts and this many tokens: the fp64 gate (no matrix cores)
constexpr int kMinTileRows = 32;  // smallest GEMM M tile
constexpr int kTailBlocks = 256;  // largest grid of the persistent GEMM whose K-split tail has scratch (one block per CU)

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Measurement switches, read from the environment ONCE (when the library is loaded); all unset in normal use.
struct Tuning {
    int force_bm;      // BROWNOUT_MOE_BM = 32/64/128/256: one tile height for every unit (0: not forced)
    int group_m;       // BROWNOUT_MOE_GM: M tiles per L2 super-tile of the GEMMs (0: 8 for 256-row tiles, else 4)
    int force_ksplit;  // BROWNOUT_MOE_KSPLIT = 1/2/4: K planes of GEMM2 with small tiles (0: not forced)
};
const Tuning& tuning();

// One-time set-up per device: kernel attributes (dynamic LDS sizes), CU count.  Done by moe_init and by
// moe_workspace_size; the launch paths only check that it has happened (and do it if not, which works
// everywhere except under stream capture).
struct DeviceInfo { int n_cu; };
hipError_t ensure_device_init(DeviceInfo* info);
hipError_t init_ffn_kernels();      // ffn.hip
hipError_t init_route_kernels();    // route.hip

// How the rows of the units are cut into GEMM M tiles: one tile height for every unit of a launch, decided on
// the host from the expected rows per unit (the real counts stay on the device).
struct TilePlan {
    int bm;      // 256, 128, 64 or 32
};
TilePlan make_tile_plan(int64_t expected_rows_per_unit);

// Derived sizes of one (config, T) problem.
struct Dims {
    int T, d, F, m, K, way, G, Ns, Fs, U, slots, m_pad, Fmax;
    int score_fn, add_residual, gate_format;
    int64_t row_cap;   // rows the row lists can hold: T*(K+Ns)
    int n_seg;         // routing segments
    int tile_cap;      // entries of one GEMM tile table
    int ksplit;        // K slices of GEMM2 (partial products in separate planes of Y)
    int64_t y_plane;   // elements between two planes of Y
    int tail_blocks;   // fp32 tiles in the scratch of the persistent GEMM's K-split tail (a bound on its grid)
};
Dims make_dims(const moe_config& c, int T);

// Carving of the caller's workspace.  All offsets are multiples of 256 bytes.
struct Workspace {
    size_t topk_idx, topk_w, expert_cnt, expert_unit, expert_in_s1, unit_cnt, unit_off, row_token, row_weight,
        token_rows, n_rows, near_tie;                 // default homes of the moe_route_out fields
    size_t gate_split;                                // [3][m_pad][d] bf16
    size_t seg_cnt, seg_off;                          // [n_seg][U] int32
    size_t route_total;                               // bytes of the pieces above (all that routing alone needs)
    size_t tiles0, tiles1;                            // two GEMM tile tables: int32[4] header + int4 entries
    size_t H;                                         // [h_rows][Fmax] bf16
    size_t Y;                                         // [y_rows][d], IEEE half (2 bytes; carried as bf16_t*)
    size_t ones;                                      // [T] fp32 (build_united)
    size_t partial, partial_bytes;                    // fp32 tiles of GEMM2's K-split tail (256-row tiles, one plane)
    size_t total;
    int64_t h_rows, y_rows;
};
Workspace carve_workspace(const Dims& D);

// Resolved device pointers of the routing artefacts (caller's or workspace's).
struct RouteBufs {
    int32_t* topk_idx; float* topk_w; int32_t* expert_cnt; int32_t* expert_unit; uint8_t* expert_in_s1;
    int32_t* unit_cnt; int32_t* unit_off; int32_t* row_token; float* row_weight; int32_t* token_rows;
    int32_t* n_rows; uint8_t* near_tie;
};

// ---- profiling hooks (api.hip) ----
void prof_begin(int stage, hipStream_t s);
void prof_end(int stage, hipStream_t s);
struct ProfScope {
    int stage; hipStream_t s;
    ProfScope(int st, hipStream_t str) : stage(st), s(str) { prof_begin(stage, s); }
    ~ProfScope() { prof_end(stage, s); }
};

// ---- routing (route.hip) ----
struct TileJobs;
// gate: fp32 [m][d] (D.gate_format MOE_GATE_FP32; split into gate_split on the way) or the packed pieces
// (MOE_GATE_PACKED; gate_split unused).  jobs: GEMM tile tables to build once the unit counts are known
// (jobs.n == 0: none).
hipError_t launch_route(const Dims& D, const bf16_t* x, const void* gate, const float* gate_bias,
                        double threshold, int full_brownout, const RouteBufs& R, bf16_t* gate_split,
                        int32_t* seg_cnt, int32_t* seg_off, const TileJobs& jobs, hipStream_t s);
hipError_t launch_pack_gate(const float* gate_w, int m, int m_pad, int d, bf16_t* packed, hipStream_t s);

// ---- FFN (ffn.hip) ----
struct FfnWeights { const bf16_t *w1, *w3, *w2; };
// Runs W2(silu(W1 x)*(W3 x)) for the rows of units [u_lo,u_hi) listed in (unit_cnt, unit_off, gather),
// writes Y[row][d] = FFN(x[gather ? gather[row] : row]) (the row weights are applied by the combine).  Fdim is the FFN width of
// these units.  Weight source of unit u: u<m experts[u]; u<m+G united[u-m]; else shared[u-m-G].
// plan / table: how the rows are cut into M tiles and where the tile table lives; table_built: the routing
// kernels have already written it (else a small kernel does, from unit_cnt / unit_off).
hipError_t launch_ffn(const Dims& D, int u_lo, int u_hi, int Fdim, const TilePlan& plan, const bf16_t* x,
                      const int32_t* gather, const int32_t* unit_cnt, const int32_t* unit_off,
                      const FfnWeights& experts, const FfnWeights& united, const FfnWeights& shared,
                      int32_t* table, bool table_built, bf16_t* H, bf16_t* Y, float* partial, hipStream_t s);
hipError_t launch_combine(const Dims& D, const bf16_t* x, const bf16_t* Y, const int32_t* token_rows,
                          const float* row_weight, bf16_t* out, hipStream_t s);

// ---- united experts (united.hip) ----
// C[M][N] fp32 = A[M][K] . B[N][K]^T (bf16 operands, K a multiple of 64, N a multiple of 64); table: scratch of
// 4 + 4 * ceil(M/64) ints.
hipError_t launch_plain_gemm(const bf16_t* A, const bf16_t* B, int M, int N, int K, float* C, int32_t* table,
                             hipStream_t s);
hipError_t launch_united_mean(const bf16_t* w, int m, int way, size_t n_elem, bf16_t* u, hipStream_t s);
hipError_t launch_single_unit(int32_t* unit_cnt, int32_t* unit_off, int U, int u, int n, float* ones,
                              hipStream_t s);
hipError_t launch_zero_f32(float* p, int n, hipStream_t s);
// loss[g] += scale * sum_{e<n} (a[e]-b[e])^2   (one block, deterministic)
hipError_t launch_sqdiff_accumulate(const bf16_t* a, const bf16_t* b, size_t n, float scale, float* loss_g,
                                    hipStream_t s);

// United-expert distillation (distill.hip).  buf: distill_buffer_bytes(n, d, F) bytes of device memory.
size_t distill_buffer_bytes(int n, int d, int F);
float* distill_tbar(void* buf, int n, int d, int F);      // [n][d] mean teacher output, filled by the caller
float* distill_floor(void* buf, int n, int d, int F);     // [1] loss at the mean teacher output
hipError_t launch_fill_f32(float* p, size_t n, float v, hipStream_t s);
hipError_t launch_teacher_mean(const bf16_t* y_half, float* tbar, size_t n, float inv_k, hipStream_t s);
hipError_t launch_teacher_spread(const bf16_t* y_half, const float* tbar, size_t n, float scale, float* floor_,
                                 hipStream_t s);
hipError_t distill_group(const bf16_t* x, int n, int d, int F, bf16_t* w1u, bf16_t* w3u, bf16_t* w2u, int steps,
                         float lr, float* hist, void* buf, hipStream_t s);

// Probes (probe.hip): sustained rate of a pure MFMA loop on the caller's operand bits (operands: 64 KiB of
// bf16, sink: 2 MiB), and of a read-only sweep over buf (sink: 4 bytes).  Both wait for the stream.
hipError_t probe_mfma(const void* operands, void* sink, hipStream_t s, double* tflops);
hipError_t probe_hbm_read(const void* buf, size_t bytes, void* sink, hipStream_t s, double* gbs);

}  // namespace bmoe
