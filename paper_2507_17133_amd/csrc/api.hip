// C ABI of libbrownout_moe.so: argument validation, workspace carving, kernel sequencing, profiling.
#include "internal.h"
#include "tiles.h"

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

// Scratch of moe_route_static (callers that cannot allocate): routing work space of a stated, modest size
// that lives in the library's own device image.  In host code this name is only a handle for
// hipGetSymbolAddress; the device address is looked up once per device in ensure_device_init.
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace bmoe {

constexpr int kMixedRows = 384;      // expected rows per unit from which 256-row tiles are used
constexpr int kMaxDevices = 64;

static Tuning read_tuning()
{
    Tuning t{0, 0, 0};
    if (const char* e = std::getenv("BROWNOUT_MOE_BM")) {
        const int v = std::atoi(e);
        if (v == 32 || v == 64 || v == 128 || v == 256) t.force_bm = v;
    }
    if (const char* e = std::getenv("BROWNOUT_MOE_GM")) t.group_m = std::max(1, std::min(64, std::atoi(e)));
    if (const char* e = std::getenv("BROWNOUT_MOE_KSPLIT")) {
        const int v = std::atoi(e);
        if (v == 1 || v == 2 || v == 4) t.force_ksplit = v;
    }
    return t;
}
const Tuning& tuning()
{
    static const Tuning t = read_tuning();       // read once, when first asked for
    return t;
}

static std::mutex g_init_mutex;
static bool g_init_done[kMaxDevices] = {false};
static DeviceInfo g_dev_info[kMaxDevices];
static void* g_scratch_ptr[kMaxDevices] = {nullptr};

hipError_t ensure_device_init(DeviceInfo* info)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_init_mutex);
    if (!g_init_done[dev]) {
        (void)tuning();
        if ((e = init_ffn_kernels()) != hipSuccess) return e;
        if ((e = init_route_kernels()) != hipSuccess) return e;
        int n_cu = 0;
        if ((e = hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return e;
        void* sp = nullptr;
        if ((e = hipGetSymbolAddress(&sp, HIP_SYMBOL(scratch))) != hipSuccess) return e;
        g_dev_info[dev].n_cu = n_cu;
        g_scratch_ptr[dev] = sp;
        g_init_done[dev] = true;
    }
    if (info) *info = g_dev_info[dev];
    return hipSuccess;
}

static void* static_scratch_of_current_device()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    return g_scratch_ptr[dev];
}

static thread_local std::string g_hip_error;

static moe_status hip_fail(hipError_t e, const char* where)
{
    g_hip_error = std::string(where) + ": " + hipGetErrorString(e);
    (void)hipGetLastError();
    return MOE_ERR_HIP;
}

// GEMM tile height from the expected rows per expert when every unit gets the same height.
static int pick_tile_rows(int64_t expected_rows_per_unit)
{
    if (tuning().force_bm) return tuning().force_bm;
    if (expected_rows_per_unit >= kMixedRows) return 256;
    // one tile should hold an expert's rows with room for the spread around the mean: a second, nearly
    // empty tile would stream the expert's weights a second time
    if (expected_rows_per_unit >= 48) return 128;
    if (expected_rows_per_unit >= 24) return 64;
    return 32;
}

TilePlan make_tile_plan(int64_t expected_rows_per_unit)
{
    TilePlan p;
    p.bm = pick_tile_rows(expected_rows_per_unit);
    return p;
}

Dims make_dims(const moe_config& c, int T)
{
    Dims D;
    D.T = T; D.d = c.d_model; D.F = c.d_ff; D.m = c.n_experts; D.K = c.top_k; D.way = c.way;
    D.G = ceil_div(c.n_experts, c.way);
    D.Ns = c.n_shared; D.Fs = c.n_shared > 0 ? c.d_ff_shared : 0;
    D.U = D.m + D.G + D.Ns;
    D.slots = D.K + D.Ns;
    D.m_pad = ceil_div(D.m, 16) * 16;
    D.Fmax = D.F > D.Fs ? D.F : D.Fs;
    D.score_fn = c.score_fn; D.add_residual = c.add_residual;
    D.gate_format = c.gate_format;
    D.row_cap = (int64_t)T * D.slots;
    D.n_seg = ceil_div(T, kSegTokens);
    D.tile_cap = (int)(D.row_cap / kMinTileRows) + D.U;
    // GEMM2 has few, long tiles (N = d): split K (at most 4 ways) until about four rounds of blocks fill
    // the 256 CUs; more slices only add prologues and planes for the combine to sum.
    const int bm = pick_tile_rows((int64_t)T * D.K / D.m);
    const int64_t tiles2 = (D.row_cap / bm + (D.m + D.G) / 2 + D.Ns) * (int64_t)ceil_div(D.d, 256);
    int ks = 1;
    while (ks < 4 && tiles2 * ks < 1024 && (D.F / 64) / (ks * 2) >= 8) ks *= 2;
    if (bm == 256) ks = 1;                                // the persistent kernel balances its tail itself
    if (tuning().force_ksplit) ks = tuning().force_ksplit;
    D.ksplit = ks;
    D.y_plane = D.row_cap * (int64_t)D.d;
    const int64_t max_tiles = (D.row_cap / 256 + D.U) * (int64_t)std::max(ceil_div(D.d, 256), ceil_div(D.Fmax, 128));
    D.tail_blocks = (int)std::min<int64_t>(kTailBlocks, (max_tiles + 7) / 8 * 8);
    return D;
}

// Rows of Y the workspace holds: an upper bound of rows x K planes over every batch of at most T tokens, so
// that a workspace sized for T_max serves every smaller batch.  More than one plane is only chosen while
// GEMM2 has few tiles (make_dims): 2 planes need fewer than 1024 tiles of at most 128 rows, 4 planes fewer
// than 512, which bounds the rows such a batch can have.
static int64_t y_rows_bound(const Dims& D)
{
    const int64_t nt_d = ceil_div(D.d, 256);
    const int64_t lim2 = 128 * (1024 / nt_d) + 128, lim4 = 128 * (512 / nt_d) + 128;
    int64_t rows = std::max<int64_t>(D.row_cap, 2 * (int64_t)D.T);
    rows = std::max(rows, 2 * std::min(D.row_cap, lim2));
    rows = std::max(rows, 4 * std::min(D.row_cap, lim4));
    if (tuning().force_ksplit) rows = std::max(rows, D.row_cap * tuning().force_ksplit);
    return rows;
}

// Every piece grows (weakly) with T, so the total does: moe_workspace_size(T_max) covers every T <= T_max.
// The routing pieces come first: carve_route_only() is the prefix moe_route_static needs.
static void carve_route_pieces(const Dims& D, Workspace& W, size_t& o)
{
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    W.topk_idx = take((size_t)D.T * D.K * 4);
    W.topk_w = take((size_t)D.T * D.K * 4);
    W.expert_cnt = take((size_t)D.m * 4);
    W.expert_unit = take((size_t)D.m * 4);
    W.expert_in_s1 = take((size_t)D.m);
    W.unit_cnt = take((size_t)D.U * 4);
    W.unit_off = take((size_t)(D.U + 1) * 4);
    W.row_token = take((size_t)D.row_cap * 4);
    W.row_weight = take((size_t)D.row_cap * 4);
    W.token_rows = take((size_t)D.row_cap * 4);
    W.n_rows = take(4);
    W.near_tie = take((size_t)D.T);
    // the pieces of an fp32 gate matrix.  A packed gate of more than 16 experts brings them; with at most 16
    // experts the gate is fp32 rows in either format, cut on the way only beyond kFewExpertsTokens tokens
    const bool no_pieces = D.m_pad == 16 ? D.T <= kFewExpertsTokens : D.gate_format == MOE_GATE_PACKED;
    W.gate_split = take(no_pieces ? 0 : (size_t)3 * D.m_pad * D.d * 2);
    W.seg_cnt = take((size_t)D.n_seg * D.U * 4);
    W.seg_off = take((size_t)D.n_seg * D.U * 4);
}

Workspace carve_workspace(const Dims& D)
{
    Workspace W;
    size_t o = 0;
    carve_route_pieces(D, W, o);
    W.route_total = o;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    W.tiles0 = take(16 + (size_t)D.tile_cap * 16);
    W.tiles1 = take(16 + (size_t)D.tile_cap * 16);
    W.h_rows = D.row_cap;
    W.y_rows = y_rows_bound(D);
    // one tile of rows past the end: GEMM2's ragged last tile reads (and discards) whole tiles of H
    W.H = take((size_t)(W.h_rows + 256) * D.Fmax * 2);
    W.Y = take((size_t)W.y_rows * D.d * 2);
    W.ones = take((size_t)D.T * 4);
    // K-split tail of the persistent 256-row GEMMs: one fp32 tile per block of their grid.  256-row tiles can
    // occur from kMixedRows tokens on (a shared expert, or one unit holding all calibration tokens).
    W.partial = 0;
    W.partial_bytes = 0;
    if (D.T >= kMixedRows || tuning().force_bm == 256) {
        W.partial_bytes = (size_t)D.tail_blocks * 256 * 256 * 4;
        W.partial = take(W.partial_bytes);
    }
    W.total = o;
    return W;
}

static moe_status check_config(const moe_config* c)
{
    if (!c) return MOE_ERR_INVALID_ARG;
    if (c->gate_format != MOE_GATE_FP32 && c->gate_format != MOE_GATE_PACKED) return MOE_ERR_INVALID_ARG;
    if (c->n_experts < 1 || c->top_k < 1 || c->way < 1 || c->n_shared < 0) return MOE_ERR_INVALID_ARG;
    if (c->top_k > c->n_experts) return MOE_ERR_INVALID_ARG;
    if (c->score_fn != 0 && c->score_fn != 1) return MOE_ERR_INVALID_ARG;
    if (c->add_residual != 0 && c->add_residual != 1) return MOE_ERR_INVALID_ARG;
    if (c->d_model <= 0 || c->d_ff <= 0 || c->d_model % 64 || c->d_ff % 64) return MOE_ERR_SHAPE;
    if (c->n_shared > 0 && (c->d_ff_shared <= 0 || c->d_ff_shared % 64)) return MOE_ERR_SHAPE;
    if (c->n_experts > kMaxExperts || c->top_k > kMaxTopK || c->n_shared > kMaxShared) return MOE_ERR_SHAPE;
    return MOE_OK;
}

static moe_status check_T(const moe_config* c, int32_t T)
{
    if (T <= 0) return MOE_ERR_INVALID_ARG;
    if ((int64_t)T * (c->top_k + c->n_shared) > ((int64_t)1 << 30)) return MOE_ERR_SHAPE;
    // byte offsets into the activations are 32-bit in the 256-row GEMM
    if ((int64_t)T * c->d_model * 2 >= ((int64_t)1 << 32)) return MOE_ERR_UNSUPPORTED;
    return MOE_OK;
}

static bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

static moe_status check_weights(const moe_ffn_weights* w)
{
    if (!w || !w->w1 || !w->w3 || !w->w2) return MOE_ERR_INVALID_ARG;
    if (misaligned(w->w1) || misaligned(w->w3) || misaligned(w->w2)) return MOE_ERR_ALIGNMENT;
    return MOE_OK;
}

static FfnWeights to_ffn(const moe_ffn_weights* w)
{
    FfnWeights f{nullptr, nullptr, nullptr};
    if (w) {
        f.w1 = static_cast<const bf16_t*>(w->w1);
        f.w3 = static_cast<const bf16_t*>(w->w3);
        f.w2 = static_cast<const bf16_t*>(w->w2);
    }
    return f;
}

template <typename Tp>
static Tp* at(void* ws, size_t off) { return reinterpret_cast<Tp*>(static_cast<char*>(ws) + off); }

static RouteBufs resolve_route(const moe_route_out* o, void* ws, const Workspace& W)
{
    RouteBufs R;
    R.topk_idx = (o && o->topk_idx) ? o->topk_idx : at<int32_t>(ws, W.topk_idx);
    R.topk_w = (o && o->topk_w) ? o->topk_w : at<float>(ws, W.topk_w);
    R.expert_cnt = (o && o->expert_cnt) ? o->expert_cnt : at<int32_t>(ws, W.expert_cnt);
    R.expert_unit = (o && o->expert_unit) ? o->expert_unit : at<int32_t>(ws, W.expert_unit);
    R.expert_in_s1 = (o && o->expert_in_s1) ? o->expert_in_s1 : at<uint8_t>(ws, W.expert_in_s1);
    R.unit_cnt = (o && o->unit_cnt) ? o->unit_cnt : at<int32_t>(ws, W.unit_cnt);
    R.unit_off = (o && o->unit_off) ? o->unit_off : at<int32_t>(ws, W.unit_off);
    R.row_token = (o && o->row_token) ? o->row_token : at<int32_t>(ws, W.row_token);
    R.row_weight = (o && o->row_weight) ? o->row_weight : at<float>(ws, W.row_weight);
    R.token_rows = (o && o->token_rows) ? o->token_rows : at<int32_t>(ws, W.token_rows);
    R.n_rows = (o && o->n_rows) ? o->n_rows : at<int32_t>(ws, W.n_rows);
    R.near_tie = (o && o->near_tie) ? o->near_tie : at<uint8_t>(ws, W.near_tie);
    return R;
}

static moe_status check_route_ptr_alignment(const moe_route_out* o)
{
    const void* ps[] = {o->topk_idx, o->topk_w, o->expert_cnt, o->expert_unit, o->unit_cnt, o->unit_off,
                        o->row_token, o->row_weight, o->token_rows, o->n_rows};
    for (const void* p : ps)
        if (p && (reinterpret_cast<uintptr_t>(p) & 3u)) return MOE_ERR_ALIGNMENT;
    return MOE_OK;
}

// ---------------------------------------------------------------- profiling
struct ProfRecord { int stage; hipEvent_t a, b; };
static unsigned g_prof_mask = 0;
static std::vector<ProfRecord> g_prof_records;
static std::vector<hipEvent_t> g_prof_pool;
static hipEvent_t g_prof_open[MOE_N_STAGES];
static bool g_prof_is_open[MOE_N_STAGES] = {false};
constexpr size_t kProfMaxRecords = 4096 * MOE_N_STAGES;

static hipEvent_t prof_event()
{
    if (!g_prof_pool.empty()) {
        hipEvent_t e = g_prof_pool.back();
        g_prof_pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

void prof_begin(int stage, hipStream_t s)
{
    if (!(g_prof_mask & (1u << stage)) || g_prof_records.size() >= kProfMaxRecords) return;
    hipEvent_t e = prof_event();
    if (!e) return;
    (void)hipEventRecord(e, s);
    g_prof_open[stage] = e;
    g_prof_is_open[stage] = true;
}

void prof_end(int stage, hipStream_t s)
{
    if (!g_prof_is_open[stage]) return;
    g_prof_is_open[stage] = false;
    hipEvent_t e = prof_event();
    if (!e) { g_prof_pool.push_back(g_prof_open[stage]); return; }
    (void)hipEventRecord(e, s);
    g_prof_records.push_back(ProfRecord{stage, g_prof_open[stage], e});
}

}  // namespace bmoe

using namespace bmoe;

extern "C" {

const char* moe_status_string(moe_status s)
{
    switch (s) {
        case MOE_OK: return "ok";
        case MOE_ERR_INVALID_ARG: return "invalid argument";
        case MOE_ERR_SHAPE: return "unsupported shape";
        case MOE_ERR_ALIGNMENT: return "misaligned pointer";
        case MOE_ERR_WORKSPACE: return "workspace missing or too small";
        case MOE_ERR_UNSUPPORTED: return "not implemented";
        case MOE_ERR_HIP: return "HIP runtime error";
        default: return "unknown status";
    }
}

const char* moe_last_hip_error(void) { return g_hip_error.c_str(); }

moe_status moe_workspace_size(const moe_config* cfg, int32_t T_max, size_t* bytes)
{
    moe_status st = check_config(cfg);
    if (st != MOE_OK) return st;
    if (!bytes) return MOE_ERR_INVALID_ARG;
    st = check_T(cfg, T_max);
    if (st != MOE_OK) return st;
    *bytes = carve_workspace(make_dims(*cfg, T_max)).total;
    // a caller sizes its workspace before its first launch: take the chance to do the per-device set-up, so
    // that even a first call made under stream capture finds it done (no device, e.g. a CPU-only host: skip)
    if (ensure_device_init(nullptr) != hipSuccess) (void)hipGetLastError();
    return MOE_OK;
}

moe_status moe_init(void)
{
    hipError_t e = ensure_device_init(nullptr);
    return e == hipSuccess ? MOE_OK : hip_fail(e, "moe_init");
}

moe_status moe_gate_packed_size(const moe_config* cfg, size_t* bytes)
{
    moe_status st = check_config(cfg);
    if (st != MOE_OK) return st;
    if (!bytes) return MOE_ERR_INVALID_ARG;
    *bytes = (size_t)3 * (ceil_div(cfg->n_experts, 16) * 16) * cfg->d_model * 2;
    return MOE_OK;
}

moe_status moe_pack_gate(const moe_config* cfg, const float* gate_w, void* packed, size_t packed_bytes, void* stream)
{
    moe_status st = check_config(cfg);
    if (st != MOE_OK) return st;
    if (!gate_w || !packed) return MOE_ERR_INVALID_ARG;
    if (misaligned(gate_w) || misaligned(packed)) return MOE_ERR_ALIGNMENT;
    const int m_pad = ceil_div(cfg->n_experts, 16) * 16;
    if (packed_bytes < (size_t)3 * m_pad * cfg->d_model * 2) return MOE_ERR_WORKSPACE;
    hipError_t e = launch_pack_gate(gate_w, cfg->n_experts, m_pad, cfg->d_model, static_cast<bf16_t*>(packed),
                                    static_cast<hipStream_t>(stream));
    return e == hipSuccess ? MOE_OK : hip_fail(e, "moe_pack_gate");
}

static moe_status check_route_args(const moe_config* cfg, const void* x, int32_t T, const void* gate_w,
                                   const float* gate_bias, double threshold, const moe_route_out* out)
{
    moe_status st = check_config(cfg);
    if (st != MOE_OK) return st;
    st = check_T(cfg, T);
    if (st != MOE_OK) return st;
    if (!x || !gate_w || !out) return MOE_ERR_INVALID_ARG;
    if (!(threshold >= 0.0 && threshold <= 1.0)) return MOE_ERR_INVALID_ARG;
    if (misaligned(x) || misaligned(gate_w) || (gate_bias && (reinterpret_cast<uintptr_t>(gate_bias) & 3u)))
        return MOE_ERR_ALIGNMENT;
    return check_route_ptr_alignment(out);
}

moe_status moe_route(const moe_config* cfg, const void* x, int32_t T, const void* gate_w, const float* gate_bias,
                     double threshold, int32_t use_full_brownout, const moe_route_out* out, void* workspace,
                     size_t workspace_bytes, void* stream)
{
    moe_status st = check_route_args(cfg, x, T, gate_w, gate_bias, threshold, out);
    if (st != MOE_OK) return st;
    const Dims D = make_dims(*cfg, T);
    const Workspace W = carve_workspace(D);
    if (!workspace || workspace_bytes < W.total) return MOE_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return MOE_ERR_ALIGNMENT;
    const RouteBufs R = resolve_route(out, workspace, W);
    hipStream_t s = static_cast<hipStream_t>(stream);
    TileJobs none;
    none.n = 0; none.cap = 0;
    hipError_t e = launch_route(D, static_cast<const bf16_t*>(x), gate_w, gate_bias, threshold,
                                use_full_brownout ? 1 : 0, R, at<bf16_t>(workspace, W.gate_split),
                                at<int32_t>(workspace, W.seg_cnt), at<int32_t>(workspace, W.seg_off), none, s);
    if (e != hipSuccess) return hip_fail(e, "moe_route");
    return MOE_OK;
}

moe_status moe_route_static(const moe_config* cfg, const void* x, int32_t T, const void* gate_w,
                            const float* gate_bias, double threshold, int32_t use_full_brownout,
                            const moe_route_out* out, void* stream)
{
    moe_status st = check_route_args(cfg, x, T, gate_w, gate_bias, threshold, out);
    if (st != MOE_OK) return st;
    const Dims D = make_dims(*cfg, T);
    Workspace W;
    size_t need = 0;
    carve_route_pieces(D, W, need);
    if (need > kStaticScratchBytes) return MOE_ERR_WORKSPACE;          // beyond the stated maximum
    hipError_t e = ensure_device_init(nullptr);                          // first call on this device: looks the scratch up
    if (e != hipSuccess) return hip_fail(e, "moe_route_static/init");
    void* sp = static_scratch_of_current_device();
    if (!sp) return hip_fail(hipErrorInvalidDevice, "moe_route_static/scratch");
    const RouteBufs R = resolve_route(out, sp, W);
    hipStream_t s = static_cast<hipStream_t>(stream);
    TileJobs none;
    none.n = 0; none.cap = 0;
    // everything the kernels read from the scratch they write first in the same call (counters are cleared by
    // the first kernel), so what an earlier call left there does not matter
    e = launch_route(D, static_cast<const bf16_t*>(x), gate_w, gate_bias, threshold, use_full_brownout ? 1 : 0, R,
                     at<bf16_t>(sp, W.gate_split), at<int32_t>(sp, W.seg_cnt), at<int32_t>(sp, W.seg_off), none, s);
    if (e != hipSuccess) return hip_fail(e, "moe_route_static");
    return MOE_OK;
}

moe_status moe_forward(const moe_config* cfg, const void* x, int32_t T, const void* gate_w, const float* gate_bias,
                       const moe_ffn_weights* experts, const moe_ffn_weights* united, const moe_ffn_weights* shared,
                       double threshold, int32_t use_full_brownout, const moe_route_out* route, void* out,
                       void* workspace, size_t workspace_bytes, void* stream)
{
    moe_status st = check_config(cfg);
    if (st != MOE_OK) return st;
    st = check_T(cfg, T);
    if (st != MOE_OK) return st;
    if (!x || !out) return MOE_ERR_INVALID_ARG;
    if (misaligned(x) || misaligned(out)) return MOE_ERR_ALIGNMENT;
    st = check_weights(experts);
    if (st != MOE_OK) return st;
    if (cfg->n_shared > 0) {
        st = check_weights(shared);
        if (st != MOE_OK) return st;
    } else if (shared) {
        return MOE_ERR_INVALID_ARG;
    }
    if (united) {
        st = check_weights(united);
        if (st != MOE_OK) return st;
    }
    if (!route) {
        if (!gate_w) return MOE_ERR_INVALID_ARG;
        if (!(threshold >= 0.0 && threshold <= 1.0)) return MOE_ERR_INVALID_ARG;
        if (misaligned(gate_w) || (gate_bias && (reinterpret_cast<uintptr_t>(gate_bias) & 3u)))
            return MOE_ERR_ALIGNMENT;
        if (!united && threshold < 1.0 && !use_full_brownout) return MOE_ERR_INVALID_ARG;
    } else {
        if (!route->expert_unit || !route->unit_cnt || !route->unit_off || !route->row_token || !route->row_weight ||
            !route->token_rows)
            return MOE_ERR_INVALID_ARG;
        st = check_route_ptr_alignment(route);
        if (st != MOE_OK) return st;
    }
    const Dims D = make_dims(*cfg, T);
    const Workspace W = carve_workspace(D);
    if (!workspace || workspace_bytes < W.total) return MOE_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return MOE_ERR_ALIGNMENT;
    const RouteBufs R = resolve_route(route, workspace, W);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bf16_t* xb = static_cast<const bf16_t*>(x);
    // How the rows are cut into GEMM tiles: routed + united units by the expected rows per expert; shared units
    // (T rows each) with them when they have the same width, else in a launch of their own.
    const bool split_shared = D.Ns > 0 && D.Fs != D.F;
    TileJobs jobs;
    jobs.n = split_shared ? 2 : 1;
    jobs.cap = D.tile_cap;
    jobs.job[0].u_lo = 0; jobs.job[0].u_hi = split_shared ? D.m + D.G : D.U;
    jobs.job[0].plan = make_tile_plan((int64_t)T * D.K / D.m);
    jobs.job[0].table = at<int32_t>(workspace, W.tiles0);
    jobs.job[1].u_lo = D.m + D.G; jobs.job[1].u_hi = D.U;
    jobs.job[1].plan = make_tile_plan(T);
    jobs.job[1].table = at<int32_t>(workspace, W.tiles1);
    hipError_t e;
    if (!route) {
        e = launch_route(D, xb, gate_w, gate_bias, threshold, use_full_brownout ? 1 : 0, R,
                         at<bf16_t>(workspace, W.gate_split), at<int32_t>(workspace, W.seg_cnt),
                         at<int32_t>(workspace, W.seg_off), jobs, s);
        if (e != hipSuccess) return hip_fail(e, "moe_forward/route");
    }
    const bool built = route == nullptr;
    const FfnWeights fe = to_ffn(experts), fu = to_ffn(united), fs = to_ffn(shared);
    bf16_t* H = at<bf16_t>(workspace, W.H);
    bf16_t* Y = at<bf16_t>(workspace, W.Y);
    float* partial = W.partial_bytes ? at<float>(workspace, W.partial) : nullptr;
    for (int j = 0; j < jobs.n; ++j) {
        const TileJob& J = jobs.job[j];
        e = launch_ffn(D, J.u_lo, J.u_hi, j == 0 ? D.F : D.Fs, J.plan, xb, R.row_token, R.unit_cnt, R.unit_off, fe, fu,
                       fs, J.table, built, H, Y, partial, s);
        if (e != hipSuccess) return hip_fail(e, j == 0 ? "moe_forward/ffn" : "moe_forward/ffn_shared");
    }
    e = launch_combine(D, xb, Y, R.token_rows, R.row_weight, static_cast<bf16_t*>(out), s);
    if (e != hipSuccess) return hip_fail(e, "moe_forward/combine");
    return MOE_OK;
}

moe_status moe_build_united(const moe_config* cfg, const moe_ffn_weights* experts, const moe_ffn_weights_out* united_out,
                            const void* calib_x, int32_t n_calib, float* loss_per_group, void* workspace,
                            size_t workspace_bytes, void* stream)
{
    moe_status st = check_config(cfg);
    if (st != MOE_OK) return st;
    st = check_weights(experts);
    if (st != MOE_OK) return st;
    if (!united_out) return MOE_ERR_INVALID_ARG;
    const moe_ffn_weights united_ro{united_out->w1, united_out->w3, united_out->w2};
    st = check_weights(&united_ro);
    if (st != MOE_OK) return st;
    if (n_calib < 0) return MOE_ERR_INVALID_ARG;
    const bool want_loss = calib_x != nullptr && loss_per_group != nullptr && n_calib > 0;
    if (calib_x && misaligned(calib_x)) return MOE_ERR_ALIGNMENT;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int m = cfg->n_experts, way = cfg->way, G = ceil_div(m, way);
    const size_t n_elem = (size_t)cfg->d_model * cfg->d_ff;
    Dims D;
    Workspace W;
    if (want_loss) {
        st = check_T(cfg, n_calib);
        if (st != MOE_OK) return st;
        D = make_dims(*cfg, n_calib);
        W = carve_workspace(D);
        D.ksplit = 1;          // the loss kernel reads single-plane FFN outputs (the carving does not depend on it)
        if (!workspace || workspace_bytes < W.total) return MOE_ERR_WORKSPACE;
        if (reinterpret_cast<uintptr_t>(workspace) & 255u) return MOE_ERR_ALIGNMENT;
    }
    hipError_t e;
    const void* src[3] = {experts->w1, experts->w3, experts->w2};
    void* dst[3] = {united_out->w1, united_out->w3, united_out->w2};
    for (int k = 0; k < 3; ++k) {
        e = launch_united_mean(static_cast<const bf16_t*>(src[k]), m, way, n_elem, static_cast<bf16_t*>(dst[k]), s);
        if (e != hipSuccess) return hip_fail(e, "moe_build_united/mean");
    }
    if (!want_loss) return MOE_OK;

    const FfnWeights fe = to_ffn(experts), fu = to_ffn(&united_ro), fs{nullptr, nullptr, nullptr};
    const TilePlan plan = make_tile_plan(n_calib);
    int32_t* unit_cnt = at<int32_t>(workspace, W.unit_cnt);
    int32_t* unit_off = at<int32_t>(workspace, W.unit_off);
    float* ones = at<float>(workspace, W.ones);
    bf16_t* H = at<bf16_t>(workspace, W.H);
    bf16_t* Yu = at<bf16_t>(workspace, W.Y);
    bf16_t* Yo = Yu + (size_t)n_calib * D.d;
    int32_t* tiles = at<int32_t>(workspace, W.tiles0);
    const bf16_t* xb = static_cast<const bf16_t*>(calib_x);
    e = launch_zero_f32(loss_per_group, G, s);
    if (e != hipSuccess) return hip_fail(e, "moe_build_united/zero");
    auto run_unit = [&](int u, bf16_t* Y) -> hipError_t {
        hipError_t err = launch_single_unit(unit_cnt, unit_off, D.U, u, n_calib, ones, s);
        if (err != hipSuccess) return err;
        return launch_ffn(D, u, u + 1, D.F, plan, xb, nullptr, unit_cnt, unit_off, fe, fu, fs, tiles, false, H, Y,
                          W.partial_bytes ? at<float>(workspace, W.partial) : nullptr, s);
    };
    for (int g = 0; g < G; ++g) {
        const int lo = g * way, hi = lo + way < m ? lo + way : m;
        e = run_unit(m + g, Yu);
        if (e != hipSuccess) return hip_fail(e, "moe_build_united/student");
        for (int i = lo; i < hi; ++i) {
            e = run_unit(i, Yo);
            if (e != hipSuccess) return hip_fail(e, "moe_build_united/teacher");
            e = launch_sqdiff_accumulate(Yu, Yo, (size_t)n_calib * D.d, 1.0f / ((float)(hi - lo) * (float)n_calib),
                                         loss_per_group + g, s);
            if (e != hipSuccess) return hip_fail(e, "moe_build_united/loss");
        }
    }
    return MOE_OK;
}

static moe_status check_distill(const moe_config* cfg, int32_t n_calib)
{
    moe_status st = check_config(cfg);
    if (st != MOE_OK) return st;
    if (n_calib <= 0 || n_calib % 64) return MOE_ERR_SHAPE;
    return check_T(cfg, n_calib);
}

moe_status moe_distill_workspace_size(const moe_config* cfg, int32_t n_calib, size_t* bytes)
{
    if (!bytes) return MOE_ERR_INVALID_ARG;
    moe_status st = check_distill(cfg, n_calib);
    if (st != MOE_OK) return st;
    const Dims D = make_dims(*cfg, n_calib);
    *bytes = align_up(carve_workspace(D).total, 256) + distill_buffer_bytes(n_calib, D.d, D.F);
    return MOE_OK;
}

moe_status moe_distill_united(const moe_config* cfg, const moe_ffn_weights* experts, const moe_ffn_weights_out* united,
                              const void* calib_x, int32_t n_calib, int32_t steps, float lr, float* loss_history,
                              void* workspace, size_t workspace_bytes, void* stream)
{
    moe_status st = check_distill(cfg, n_calib);
    if (st != MOE_OK) return st;
    st = check_weights(experts);
    if (st != MOE_OK) return st;
    if (!united) return MOE_ERR_INVALID_ARG;
    const moe_ffn_weights united_ro{united->w1, united->w3, united->w2};
    st = check_weights(&united_ro);
    if (st != MOE_OK) return st;
    if (!calib_x || steps < 0 || !(lr >= 0.0f)) return MOE_ERR_INVALID_ARG;
    if (misaligned(calib_x)) return MOE_ERR_ALIGNMENT;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int m = cfg->n_experts, way = cfg->way, G = ceil_div(m, way);
    Dims D = make_dims(*cfg, n_calib);
    const Workspace W = carve_workspace(D);
    D.ksplit = 1;
    const TilePlan plan = make_tile_plan(n_calib);
    const size_t fwd_bytes = align_up(W.total, 256);
    if (!workspace || workspace_bytes < fwd_bytes + distill_buffer_bytes(n_calib, D.d, D.F)) return MOE_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return MOE_ERR_ALIGNMENT;
    void* buf = static_cast<char*>(workspace) + fwd_bytes;
    const FfnWeights fe = to_ffn(experts), fu = to_ffn(&united_ro), fs{nullptr, nullptr, nullptr};
    int32_t* unit_cnt = at<int32_t>(workspace, W.unit_cnt);
    int32_t* unit_off = at<int32_t>(workspace, W.unit_off);
    float* ones = at<float>(workspace, W.ones);
    bf16_t* H = at<bf16_t>(workspace, W.H);
    bf16_t* Yo = at<bf16_t>(workspace, W.Y);
    int32_t* tiles = at<int32_t>(workspace, W.tiles0);
    const bf16_t* xb = static_cast<const bf16_t*>(calib_x);
    const size_t nd = (size_t)n_calib * D.d, dF = (size_t)D.d * D.F;
    float* tbar = distill_tbar(buf, n_calib, D.d, D.F);
    float* floor_ = distill_floor(buf, n_calib, D.d, D.F);
    hipError_t e;
    auto teacher = [&](int i) -> hipError_t {
        hipError_t err = launch_single_unit(unit_cnt, unit_off, D.U, i, n_calib, ones, s);
        if (err != hipSuccess) return err;
        return launch_ffn(D, i, i + 1, D.F, plan, xb, nullptr, unit_cnt, unit_off, fe, fu, fs, tiles, false, H, Yo,
                          W.partial_bytes ? at<float>(workspace, W.partial) : nullptr, s);
    };
    for (int g = 0; g < G; ++g) {
        const int lo = g * way, hi = lo + way < m ? lo + way : m, k = hi - lo;
        bf16_t* wu[3] = {static_cast<bf16_t*>(united->w1) + (size_t)g * dF, static_cast<bf16_t*>(united->w3) + (size_t)g * dF,
                         static_cast<bf16_t*>(united->w2) + (size_t)g * dF};
        if (k == 1) {
            // a lone member is its own best student: the minimiser (loss 0) is known, nothing to train
            const void* we[3] = {experts->w1, experts->w3, experts->w2};
            for (int q = 0; q < 3; ++q) {
                e = hipMemcpyAsync(wu[q], static_cast<const bf16_t*>(we[q]) + (size_t)lo * dF, dF * 2,
                                   hipMemcpyDeviceToDevice, s);
                if (e != hipSuccess) return hip_fail(e, "moe_distill_united/copy");
            }
            if (loss_history && (e = launch_fill_f32(loss_history + (size_t)g * (steps + 1), steps + 1, 0.0f, s)) != hipSuccess)
                return hip_fail(e, "moe_distill_united/clear");
            continue;
        }
        if ((e = launch_fill_f32(tbar, nd, 0.0f, s)) != hipSuccess) return hip_fail(e, "moe_distill_united/clear");
        if ((e = launch_fill_f32(floor_, 1, 0.0f, s)) != hipSuccess) return hip_fail(e, "moe_distill_united/clear");
        for (int i = lo; i < hi; ++i) {
            if ((e = teacher(i)) != hipSuccess) return hip_fail(e, "moe_distill_united/teacher");
            if ((e = launch_teacher_mean(Yo, tbar, nd, 1.0f / (float)k, s)) != hipSuccess)
                return hip_fail(e, "moe_distill_united/mean");
        }
        for (int i = lo; i < hi; ++i) {
            if ((e = teacher(i)) != hipSuccess) return hip_fail(e, "moe_distill_united/teacher");
            if ((e = launch_teacher_spread(Yo, tbar, nd, 1.0f / ((float)k * (float)n_calib), floor_, s)) != hipSuccess)
                return hip_fail(e, "moe_distill_united/spread");
        }
        e = distill_group(xb, n_calib, D.d, D.F, wu[0], wu[1], wu[2], steps, lr,
                          loss_history ? loss_history + (size_t)g * (steps + 1) : nullptr, buf, s);
        if (e != hipSuccess) return hip_fail(e, "moe_distill_united/train");
    }
    return MOE_OK;
}

moe_status moe_probe_mfma(const void* operands, size_t operand_bytes, void* sink, size_t sink_bytes, void* stream,
                          double* tflops)
{
    if (!operands || !sink || !tflops) return MOE_ERR_INVALID_ARG;
    if (operand_bytes < 65536 || sink_bytes < ((size_t)2 << 20)) return MOE_ERR_WORKSPACE;
    if (misaligned(operands) || misaligned(sink)) return MOE_ERR_ALIGNMENT;
    hipError_t e = probe_mfma(operands, sink, static_cast<hipStream_t>(stream), tflops);
    return e == hipSuccess ? MOE_OK : hip_fail(e, "moe_probe_mfma");
}

moe_status moe_probe_hbm_read(const void* buf, size_t bytes, void* sink, size_t sink_bytes, void* stream, double* gbs)
{
    if (!buf || !sink || !gbs) return MOE_ERR_INVALID_ARG;
    if (bytes < ((size_t)1 << 20) || sink_bytes < 4) return MOE_ERR_WORKSPACE;
    if (misaligned(buf) || (reinterpret_cast<uintptr_t>(sink) & 3u)) return MOE_ERR_ALIGNMENT;
    hipError_t e = probe_hbm_read(buf, bytes, sink, static_cast<hipStream_t>(stream), gbs);
    return e == hipSuccess ? MOE_OK : hip_fail(e, "moe_probe_hbm_read");
}

moe_status moe_profile_enable(int32_t stage_mask)
{
    g_prof_mask = (unsigned)stage_mask & ((1u << MOE_N_STAGES) - 1u);
    return MOE_OK;
}

moe_status moe_profile_collect(double* total_ms, int64_t* launches)
{
    if (!total_ms || !launches) return MOE_ERR_INVALID_ARG;
    for (int i = 0; i < MOE_N_STAGES; ++i) { total_ms[i] = 0.0; launches[i] = 0; }
    moe_status st = MOE_OK;
    for (const ProfRecord& r : g_prof_records) {
        float ms = 0.0f;
        hipError_t e = hipEventSynchronize(r.b);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, r.a, r.b);
        if (e != hipSuccess) st = hip_fail(e, "moe_profile_collect");
        else { total_ms[r.stage] += (double)ms; launches[r.stage] += 1; }
        g_prof_pool.push_back(r.a);
        g_prof_pool.push_back(r.b);
    }
    g_prof_records.clear();
    return st;
}

}  // extern "C"
