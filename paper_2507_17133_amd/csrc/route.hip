// Routing kernels of the BrownoutMoE layer for gfx950:
//   prep     clear the expert counters (large batches), split fp32 gate weights into three bf16 pieces
//            (also the one-time repack behind moe_pack_gate)
//   gate     affinities s = x.e_i on MFMA (bf16 x 3-piece weights, fp64 running sums; from 32 experts on with
//            the pieces and the x rows staged in LDS, blocks of 16, 32 or 64 tokens) or, for at most 16
//            experts and small batches, in plain fp64; TopK by wavefront shuffles, weights g, expert
//            histogram                                               (Architecture of BrownoutMoE)
//   count    Algorithm 1's S1/S2 split and unit map (every block, from the counts) and the rows
//            each 64-token segment gives each unit                   (Brownout Approach, Algorithm 1)
//   scan     offsets of segments inside units, unit totals (unit offsets: scanned by the scatter blocks)
//   scatter  row lists: row_token, row_weight, token_rows (stable: ascending token inside a unit); its first
//            block also writes the GEMM tile table
//   small    at most 1024 tokens: expert counts, Algorithm 1, both scans, the scatter and the tile table
//            in ONE block
// No floating-point atomics anywhere; integer atomics only where the result does not depend on order.
#include "internal.h"
#include "tiles.h"

#include <algorithm>

namespace bmoe {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ unsigned short f32_to_bf16_bits(float f)
{
    unsigned int u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);  // round to nearest, ties to even
    return (unsigned short)(u >> 16);
}
__device__ __forceinline__ float bf16_bits_to_f32(unsigned short b) { return __uint_as_float(((unsigned int)b) << 16); }

// ------------------------------------------------------------------------------------------------
// prep: expert_cnt = 0; gate_w = hi + mid + lo with bf16 pieces (the three pieces carry 24 bits of
// significand, so x(bf16) * piece products are exact in fp32 and their sum equals x*w to fp32 accuracy).
// Rows m..m_pad-1 of every piece are zero.
// ------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) prep_kernel(const float* __restrict__ gate_w, int m, int m_pad, int d,
                                                   unsigned short* __restrict__ split, int32_t* __restrict__ expert_cnt)
{
    const size_t n = split != nullptr ? (size_t)m_pad * d : 0;   // split == nullptr: only clear the counters
    const size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (expert_cnt != nullptr && gid < (size_t)m) expert_cnt[gid] = 0;
    for (size_t i = gid; i < n; i += (size_t)gridDim.x * blockDim.x) {
        const int e = (int)(i / d);
        const float w = e < m ? gate_w[i] : 0.0f;
        const unsigned short hi = f32_to_bf16_bits(w);
        const float r1 = w - bf16_bits_to_f32(hi);
        const unsigned short mid = f32_to_bf16_bits(r1);
        const float r2 = r1 - bf16_bits_to_f32(mid);
        const unsigned short lo = f32_to_bf16_bits(r2);
        split[i] = hi;
        split[n + i] = mid;
        split[2 * n + i] = lo;
    }
}

// ------------------------------------------------------------------------------------------------
// gate: affinities on MFMA.  Each k chunk is accumulated from zero by 16x16x32 bf16 MFMAs over the low,
// middle and high piece of the gate weights and folded into an fp64 running sum at least every 64 k, which
// keeps the logit within a few 1e-8 of the exact dot product whatever d is.
// ------------------------------------------------------------------------------------------------
struct GateArgs {
    const bf16_t* x; const unsigned short* split; const float* bias;
    int T, d, m, m_pad, K, score_fn, n_stage;
    int32_t* topk_idx; float* topk_w; uint8_t* near_tie;
    int32_t* expert_cnt;   // the launch's expert counts, cleared beforehand (atomics); null for small batches,
                           // whose routing block counts the experts itself
};

// TopK(.,K) of one token by one wavefront: lane holds experts lane, lane+64, ...; K (+1 for the best
// loser) rounds of "best of my candidates, then best across lanes" (higher score, equal scores: lower
// id); lane j keeps the j-th winner, weights are normalised over lanes 0..K-1.
// row_ror:n of a 16-lane row (DPP control 0x120 + n): lane l reads lane (l - n) mod 16 of its row
template <int CTRL>
__device__ __forceinline__ int dpp_i(int v) { return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, false); }
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) { return __int_as_float(dpp_i<CTRL>(__float_as_int(v))); }

// (bv, bi) <- the better of it and (ov, oi): higher score, equal scores: lower id; id 0x7fffffff = none
__device__ __forceinline__ void better(float& bv, int& bi, float ov, int oi)
{
    const bool take = oi != 0x7fffffff && (bi == 0x7fffffff || ov > bv || (ov == bv && oi < bi));
    if (take) { bv = ov; bi = oi; }
}

// the same when both ids are real
__device__ __forceinline__ void better_of_two(float& bv, int& bi, float ov, int oi)
{
    const bool take = ov > bv || (ov == bv && oi < bi);
    if (take) { bv = ov; bi = oi; }
}

__device__ __forceinline__ void topk_token(const GateArgs& p, const float* logit_row, int t, int lane, int* hist)
{
    const int K = p.K;
    const int n_pick = K < p.m ? K + 1 : K;    // one extra pick: the best loser, for the near-tie flag
    float v[4];
    unsigned taken = 0;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const int e = lane + 64 * c;
        v[c] = e < p.m ? logit_row[e] : 0.0f;
        if (e >= p.m) taken |= 1u << c;
    }
    float my_v = 0.0f;
    int my_i = 0;
    for (int j = 0; j < n_pick; ++j) {
        float bv = 0.0f;
        int bi = 0x7fffffff;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if (taken & (1u << c)) continue;
            if (bi == 0x7fffffff || v[c] > bv) { bv = v[c]; bi = lane + 64 * c; }
        }
        // best of the wavefront: inside each row of 16 lanes by rotations (data-parallel primitives, no trip
        // through the LDS crossbar; "better" is idempotent, so four rotations leave the row's best in every
        // lane), then across the four rows through scalar registers
        better(bv, bi, dpp_f<0x121>(bv), dpp_i<0x121>(bi));
        better(bv, bi, dpp_f<0x122>(bv), dpp_i<0x122>(bi));
        better(bv, bi, dpp_f<0x124>(bv), dpp_i<0x124>(bi));
        better(bv, bi, dpp_f<0x128>(bv), dpp_i<0x128>(bi));
        {
            float rv[4];
            int ri[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                rv[q] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(bv), 16 * q));
                ri[q] = __builtin_amdgcn_readlane(bi, 16 * q);
            }
            bv = rv[0];
            bi = ri[0];
#pragma unroll
            for (int q = 1; q < 4; ++q) better(bv, bi, rv[q], ri[q]);
        }
        if ((bi & 63) == lane) taken |= 1u << (bi >> 6);
        if (lane == j) { my_v = bv; my_i = bi; }
    }
    const float top = __shfl(my_v, 0);
    float num = 0.0f;
    if (lane < K) num = p.score_fn == 0 ? expf(my_v - top) : 1.0f / (1.0f + expf(-my_v));
    float den = num;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) den += __shfl_xor(den, off);
    const float nxt = __shfl_down(my_v, 1);
    const bool close = lane + 1 < n_pick && (my_v - nxt) < 1e-6f;
    const unsigned long long any_close = __ballot(close);
    if (lane < K) {
        p.topk_idx[(size_t)t * K + lane] = my_i;
        p.topk_w[(size_t)t * K + lane] = num / den;
        atomicAdd(&hist[my_i], 1);
    }
    if (lane == 0 && p.near_tie != nullptr) p.near_tie[t] = any_close != 0ull ? 1 : 0;
}

// The same for four tokens at a time: token `row` = lane >> 4 of the four is handled by the 16 lanes of its
// row, lane r of the row holding experts r, r+16, ... (NC of them: NC >= m_pad / 16); every reduction stays
// inside the row (rotations), so the four selections run side by side.  A lane's experts that do not exist or
// have been picked hold -infinity (logits are finite, and a row always has an expert left to pick), so a round
// is a branch-free maximum over NC registers (first of equal values: the lower id) and four rotations.
// Needs K + 1 <= 16 (lane j of the row keeps the j-th winner).
// tl: this row's token inside the block's logit array, t: its global index, valid: whether it exists.
template <int NC>
__device__ __forceinline__ void topk_rows(const GateArgs& p, const float* logit, int tl, int t, bool valid, int lane, int* hist)
{
    const int K = p.K, r = lane & 15;
    const int n_pick = K < p.m ? K + 1 : K;
    const float* logit_row = logit + tl * p.m_pad;
    const float none = -__builtin_inff();
    float v[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        const int e = r + 16 * c;
        v[c] = e < p.m ? logit_row[e] : none;
    }
    float my_v = 0.0f;
    int my_i = 0;
    for (int j = 0; j < n_pick; ++j) {
        float bv = v[0];
        int bc = 0;
#pragma unroll
        for (int c = 1; c < NC; ++c)
            if (v[c] > bv) { bv = v[c]; bc = c; }
        int bi = r + 16 * bc;
        better_of_two(bv, bi, dpp_f<0x121>(bv), dpp_i<0x121>(bi));
        better_of_two(bv, bi, dpp_f<0x122>(bv), dpp_i<0x122>(bi));
        better_of_two(bv, bi, dpp_f<0x124>(bv), dpp_i<0x124>(bi));
        better_of_two(bv, bi, dpp_f<0x128>(bv), dpp_i<0x128>(bi));
        const int wc = (bi & 15) == r ? (bi >> 4) : -1;     // the winner leaves its lane's candidates
#pragma unroll
        for (int c = 0; c < NC; ++c)
            if (c == wc) v[c] = none;
        if (r == j) { my_v = bv; my_i = bi; }
    }
    const float top = __shfl(my_v, lane & ~15);
    float num = 0.0f;
    if (r < K) num = p.score_fn == 0 ? expf(my_v - top) : 1.0f / (1.0f + expf(-my_v));
    float den = num;
    den += dpp_f<0x121>(den);
    den += dpp_f<0x122>(den);
    den += dpp_f<0x124>(den);
    den += dpp_f<0x128>(den);
    const float nxt = __shfl(my_v, (lane & ~15) | ((r + 1) & 15));
    const bool close = r + 1 < n_pick && (my_v - nxt) < 1e-6f;
    const unsigned long long any_close = __ballot(close);
    if (valid) {
        if (r < K) {
            p.topk_idx[(size_t)t * K + r] = my_i;
            p.topk_w[(size_t)t * K + r] = num / den;
            atomicAdd(&hist[my_i], 1);
        }
        if (r == 0 && p.near_tie != nullptr) p.near_tie[t] = ((any_close >> (lane & 48)) & 0xFFFFull) != 0ull ? 1 : 0;
    }
}

// gate for at most 16 experts in batches beyond kFewExpertsTokens tokens: one block = 16 tokens x the one tile of
// experts, 8 wavefronts that split K.  A stage is 256 k: the 48 rows of the three gate pieces and the 16 x rows,
// as four pieces of 64 k (rows of 128 bytes = whole lines, brought in by direct global->LDS loads, 8 rows per
// wave instruction; a wave that lets every lane fetch its own 16-byte fragment instead spends its time on tag
// look-ups: 16 rows x 64 bytes per instruction).  Wave w multiplies the 32-wide half w&1 of piece w>>1 of every
// stage, three MFMAs (low, middle, high piece) folded into fp64 sums; the eight partial sums of a logit are added
// in wave order through LDS.  Three stages: two in flight while one is multiplied.
__global__ void __launch_bounds__(512) gate_few_kernel(GateArgs p)
{
    constexpr int RB = 128, SUB = 64 * RB, STAGE = 4 * SUB, NST = 3;
    extern __shared__ __attribute__((aligned(16))) char gsm[];
    __shared__ int hist[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);
    const int t0 = blockIdx.x * 16;
    if (tid < 16) hist[tid] = 0;
    const int n_sub = p.d >> 6, n_stage = (n_sub + 3) >> 2;
    const int sub = wave_s >> 1, sl = wave_s & 1;

    // loader: the four loads of wave w bring rows 8 (4 (w&1) + i) .. +7 of piece w>>1; 16-byte chunk c of row r
    // sits in slot c ^ ((r/2)&7) (conflict-free ds_read_b128)
    const unsigned short* srcp[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = (sl * 4 + i) * 8 + (lane >> 3);
        const int chunk = (lane & 7) ^ ((row >> 1) & 7);
        const unsigned short* src = row < 48 ? p.split + (size_t)row * p.d
                                             : reinterpret_cast<const unsigned short*>(p.x) +
                                                   (size_t)min(t0 + row - 48, p.T - 1) * p.d;
        srcp[i] = src + chunk * 8;
    }
    auto issue = [&](int st, int buf) {
        const int piece = min(st * 4 + sub, n_sub - 1);   // past the end of K: the last piece again, never multiplied
        char* dst = gsm + buf * STAGE + sub * SUB + sl * 4096;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(srcp[i] + piece * 64),
                                             (__attribute__((address_space(3))) void*)(dst + i * 1024), 16, 0, 0);
    };
    // fragment of row (base + lane&15), 32-wide half sl: chunks 4 sl + (lane>>4); bases are multiples of 16 rows
    const int coff = ((sl * 4 + (lane >> 4)) ^ (((lane & 15) >> 1) & 7)) << 4;
    const int roff = (lane & 15) * RB + coff;
    double sum[4] = {0.0, 0.0, 0.0, 0.0};
    for (int q = 0; q < NST - 1; ++q)
        if (q < n_stage) issue(q, q);
    int buf = 0;
    for (int st = 0; st < n_stage; ++st) {
        // loads complete in order: stage st has landed once only the four loads of stage st+1 are outstanding
        if (st + 1 < n_stage) __builtin_amdgcn_s_waitcnt(0x0F74);
        else __builtin_amdgcn_s_waitcnt(0x0F70);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();                     // stage st is in LDS for everyone; stage st-1 is free
        asm volatile("" ::: "memory");
        if (st + NST - 1 < n_stage) issue(st + NST - 1, buf == 0 ? NST - 1 : buf - 1);
        if (st * 4 + sub < n_sub) {
            const char* St = gsm + buf * STAGE + sub * SUB + roff;
            const bf16x8 a = *reinterpret_cast<const bf16x8*>(St + 48 * RB);
            const bf16x8 b_hi = *reinterpret_cast<const bf16x8*>(St);
            const bf16x8 b_mid = *reinterpret_cast<const bf16x8*>(St + 16 * RB);
            const bf16x8 b_lo = *reinterpret_cast<const bf16x8*>(St + 32 * RB);
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b_lo, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b_mid, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b_hi, acc, 0, 0, 0);
#pragma unroll
            for (int v = 0; v < 4; ++v) sum[v] += (double)acc[v];
        }
        buf = buf + 1 == NST ? 0 : buf + 1;
    }
    __syncthreads();                                      // every wave is done with the stages: reuse them
    double* part = reinterpret_cast<double*>(gsm);        // [wave][token][expert]
    float* logit = reinterpret_cast<float*>(gsm + 8 * 256 * 8);
    // MFMA 16x16 result layout: lane holds column (lane&15) = expert, rows 4*(lane>>4)+v = tokens
#pragma unroll
    for (int v = 0; v < 4; ++v) part[(wave * 16 + 4 * (lane >> 4) + v) * 16 + (lane & 15)] = sum[v];
    __syncthreads();
    if (tid < 256) {
        double s = 0.0;
#pragma unroll
        for (int w = 0; w < 8; ++w) s += part[w * 256 + tid];
        const int e = tid & 15;
        if (p.bias != nullptr && e < p.m) s += (double)p.bias[e];
        logit[tid] = (float)s;
    }
    __syncthreads();
    if (wave < 4) {                                       // four tokens per wavefront (K + 1 <= m_pad = 16 picks)
        const int tl = wave * 4 + (lane >> 4);
        const bool valid = t0 + tl < p.T;
        topk_rows<1>(p, logit, valid ? tl : wave * 4, t0 + tl, valid && t0 + wave * 4 < p.T, lane, hist);
    }
    __syncthreads();
    if (p.expert_cnt != nullptr && tid < p.m && hist[tid] > 0) atomicAdd(&p.expert_cnt[tid], hist[tid]);
}

// ------------------------------------------------------------------------------------------------
// gate for at most 16 experts and at most kFewExpertsTokens tokens: plain fp64 arithmetic, no matrix cores.
// With so few experts and tokens what the gate needs is many blocks in flight (a CU pulls its share of x and
// the whole gate matrix at the rate of the few loads it keeps in flight), not MFMA tiles padded from m to 16
// columns: 15 us instead of 24 for 256 tokens of width 4096.  (Beyond a few thousand tokens the MFMA gate, which
// reads the gate matrix once per 16 tokens, is faster again: 28 us against 44 at 4096 tokens.)  One block = TPB tokens, 256 threads; thread t multiplies the k range
// 8t .. 8t+7 (+2048, ...) of the tokens' rows with every centroid, products and sums in double (a bf16 times an
// fp32 value is exact there), the 256 partial sums of a (token, expert) pair are added in a fixed order through
// LDS, and one wavefront per token takes TopK.  The centroids are read as fp32 rows (for at most 16 experts the
// packed form of the gate is a copy of them).
// ------------------------------------------------------------------------------------------------
template <int M, int TPB>
__global__ void __launch_bounds__(256) gate_small_kernel(GateArgs p, const float* __restrict__ gate_w)
{
    constexpr int NP = TPB * M;                           // (token, expert) pairs of the block
    __shared__ double part[NP][33];
    __shared__ float logit[TPB][16];
    __shared__ int hist[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int t0 = blockIdx.x * TPB;
    if (tid < 16) hist[tid] = 0;
    double acc[TPB][M];
#pragma unroll
    for (int q = 0; q < TPB; ++q)
#pragma unroll
        for (int e = 0; e < M; ++e) acc[q][e] = 0.0;
    for (int k = tid * 8; k < p.d; k += 2048) {
        double xv[TPB][8];
#pragma unroll
        for (int q = 0; q < TPB; ++q) {
            const int t = min(t0 + q, p.T - 1);
            const uint4 raw = *reinterpret_cast<const uint4*>(p.x + (size_t)t * p.d + k);
            const unsigned w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                xv[q][2 * c] = (double)__uint_as_float(w[c] << 16);
                xv[q][2 * c + 1] = (double)__uint_as_float(w[c] & 0xFFFF0000u);
            }
        }
#pragma unroll
        for (int e = 0; e < M; ++e) {
            double wv[8];
            if (e < p.m) {
                {
                    const float4 a = *reinterpret_cast<const float4*>(gate_w + (size_t)e * p.d + k);
                    const float4 b = *reinterpret_cast<const float4*>(gate_w + (size_t)e * p.d + k + 4);
                    wv[0] = a.x; wv[1] = a.y; wv[2] = a.z; wv[3] = a.w;
                    wv[4] = b.x; wv[5] = b.y; wv[6] = b.z; wv[7] = b.w;
                }
#pragma unroll
                for (int q = 0; q < TPB; ++q)
#pragma unroll
                    for (int c = 0; c < 8; ++c) acc[q][e] = fma(xv[q][c], wv[c], acc[q][e]);
            }
        }
    }
    // the 256 partial sums of a pair: eight neighbouring lanes first (three exchange steps), then the 32 group
    // sums in order by one thread
#pragma unroll
    for (int q = 0; q < TPB; ++q)
#pragma unroll
        for (int e = 0; e < M; ++e) {
            double v = acc[q][e];
            v += __shfl_xor(v, 1);
            v += __shfl_xor(v, 2);
            v += __shfl_xor(v, 4);
            if ((lane & 7) == 0) part[q * M + e][tid >> 3] = v;
        }
    __syncthreads();
    if (tid < NP) {
        const int q = tid / M, e = tid - q * M;
        if (e < p.m) {
            double s = 0.0;
            for (int i = 0; i < 32; ++i) s += part[tid][i];
            if (p.bias != nullptr) s += (double)p.bias[e];
            logit[q][e] = (float)s;
        }
    }
    __syncthreads();
    if (wave < TPB && t0 + wave < p.T) topk_token(p, logit[wave], t0 + wave, lane, hist);
    if (p.expert_cnt != nullptr) {                        // large batches: the launch's counts (cleared beforehand)
        __syncthreads();
        if (tid < p.m && hist[tid] > 0) atomicAdd(&p.expert_cnt[tid], hist[tid]);
    }
}

// ------------------------------------------------------------------------------------------------
// gate for many experts and many tokens: one block = 16*TG tokens x all experts, 2*TG wavefronts
// (token group tg = wave % TG, expert half eh = wave / TG).  The three weight pieces of a 32-wide k
// step ([3][m_pad] rows of 64 bytes) are staged in LDS by global_load_lds_dwordx4 (3 stages) and read
// together with the block's x rows and read by every wave, so the split gate matrix is fetched once per
// 16*TG tokens instead of once per 16.
// ------------------------------------------------------------------------------------------------
// s_waitcnt vmcnt(n) for a run-time n (the instruction takes an immediate): waits for at most the largest
// listed value <= n, which is never too lax.
__device__ __forceinline__ void wait_vmcnt_at_most(int n)
{
    if (n >= 48) __builtin_amdgcn_s_waitcnt(0xCF70);        // vmcnt 48: low four bits 0, bits 15:14 = 3
    else if (n >= 32) __builtin_amdgcn_s_waitcnt(0x8F70);
    else if (n >= 24) __builtin_amdgcn_s_waitcnt(0x4F78);
    else if (n >= 20) __builtin_amdgcn_s_waitcnt(0x4F74);
    else if (n >= 16) __builtin_amdgcn_s_waitcnt(0x4F70);
    else if (n >= 12) __builtin_amdgcn_s_waitcnt(0x0F7C);
    else if (n >= 9) __builtin_amdgcn_s_waitcnt(0x0F79);
    else if (n >= 8) __builtin_amdgcn_s_waitcnt(0x0F78);
    else if (n >= 6) __builtin_amdgcn_s_waitcnt(0x0F76);
    else if (n >= 4) __builtin_amdgcn_s_waitcnt(0x0F74);
    else if (n >= 3) __builtin_amdgcn_s_waitcnt(0x0F73);
    else if (n >= 2) __builtin_amdgcn_s_waitcnt(0x0F72);
    else if (n >= 1) __builtin_amdgcn_s_waitcnt(0x0F71);
    else __builtin_amdgcn_s_waitcnt(0x0F70);
}

template <int TG, int NTH, int KB, int MT, int EG>
__global__ void __launch_bounds__((TG / MT) * EG * 64) gate_tiled_kernel(GateArgs p)
{
    // A wave multiplies MT token tiles (16 tokens each) by NTH expert tiles: TG / MT groups of token tiles x
    // EG groups of NTH expert tiles (EG NTH >= expert tiles).  MT = 2 halves the B fragments read from LDS per MFMA.
    static_assert(TG % MT == 0, "token tiles per wave");
    // KB = k elements per stage: 64 (rows of 128 bytes, whole cache lines: what bounds this kernel is the number
    // of line requests a CU keeps in flight, not bytes) where three such stages fit the LDS, else 32
    constexpr int NWV = (TG / MT) * EG;                 // waves: token-tile groups x expert groups
    constexpr int RB = KB * 2, CPR = RB / 16, WR = 256 / RB, RPL = 1024 / RB, NSL = KB / 32;
    const int NST = p.n_stage;                          // LDS stages: as many as fit, at most 8
    extern __shared__ __attribute__((aligned(16))) char gsm[];
    __shared__ int hist[kMaxExperts];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tg = (wave % (TG / MT)) * MT, eh = wave / (TG / MT);   // first token tile, expert group
    const int t0 = blockIdx.x * (16 * TG);
    const int n_tiles = p.m_pad >> 4;
    const int w_rows = 3 * p.m_pad;                     // LDS rows of one stage: [piece][expert], then the x rows
    const int rows = w_rows + 16 * TG;
    const int groups = rows / RPL;                      // RPL rows (1 KiB) per wave-wide load
    const int stage_bytes = rows * RB;
    for (int i = tid; i < p.m_pad; i += NWV * 64) hist[i] = 0;

    // loader: wave w moves row groups w, w+NWV, ...; lane -> row lane/CPR, 16-byte slot lane%CPR holding
    // chunk (lane%CPR) ^ ((row/WR)&(CPR-1))  (conflict-free ds_read_b128 on the 64-bank LDS)
    const int ksteps = p.d / KB;
    // the source address of every load of a stage is fixed up to the k offset: computed once, not per step
    constexpr int MAXM = KB == 64 ? 128 : kMaxExperts;  // the launcher takes KB = 64 for at most 128 experts
    constexpr int MAXS = (3 * MAXM + 16 * TG + RPL * NWV - 1) / (RPL * NWV);
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);
    const unsigned short* srcp[MAXS];
#pragma unroll
    for (int i = 0; i < MAXS; ++i) {
        const int row = min((wave + i * NWV) * RPL + lane / CPR, rows - 1);
        const int chunk = (lane % CPR) ^ ((row / WR) & (CPR - 1));
        const unsigned short* src;
        if (row < w_rows) src = p.split + (size_t)row * p.d;
        else src = reinterpret_cast<const unsigned short*>(p.x) + (size_t)min(t0 + row - w_rows, p.T - 1) * p.d;
        srcp[i] = src + chunk * 8;
    }
    auto issue = [&](int ks, int buf) {
        char* dst = gsm + buf * stage_bytes + wave_s * 1024;
#pragma unroll
        for (int i = 0; i < MAXS; ++i)
            if (wave_s + i * NWV < groups)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(srcp[i] + ks * KB),
                                                 (__attribute__((address_space(3))) void*)(dst + i * NWV * 1024), 16, 0, 0);
    };

    double sum[MT][NTH][4];
    f32x4 acc[MT][NTH];
    bool tile_ok[NTH];
    int boff[NTH];
    // the swizzle term of a row depends on the lane only: expert tiles start at multiples of 16 rows, the x
    // rows at 3 * m_pad + 16 * tg, and 16 / WR is a multiple of CPR
    const int swz = ((lane & 15) / WR) & (CPR - 1);
#pragma unroll
    for (int nt = 0; nt < NTH; ++nt) {
        const int tile = eh * NTH + nt;
        tile_ok[nt] = tile < n_tiles;
        boff[nt] = ((tile_ok[nt] ? tile : 0) * 16 + (lane & 15)) * RB;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int v = 0; v < 4; ++v) sum[mt][nt][v] = 0.0;
        }
    }
    const int aoff = (w_rows + tg * 16 + (lane & 15)) * RB;
    // All loads of the loop go to LDS and complete in order per wave: at the top of step ks the loads of
    // stage ks are older than those of the later stages, which may stay in flight.
    const int young = groups / NWV;                     // loads of one stage every wave issues at least
    for (int q = 0; q < NST - 1; ++q)
        if (q < ksteps) issue(q, q);
    int buf = 0, buf_ld = NST - 1;                      // stage read at step ks = ks mod NST; stage refilled = (ks-1) mod NST
    for (int ks = 0; ks < ksteps; ++ks) {
        // stages ks+1 .. ks+NST-2 (those that exist) may stay in flight: at least `young` loads each
        wait_vmcnt_at_most(min(NST - 2, ksteps - 1 - ks) * young);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();                   // stage ks is in LDS for everyone; stage ks-1 is free
        asm volatile("" ::: "memory");
        if (ks + NST - 1 < ksteps) issue(ks + NST - 1, buf_ld);
        const char* St = gsm + buf * stage_bytes;
        buf_ld = buf;
        buf = buf + 1 == NST ? 0 : buf + 1;
#pragma unroll
        for (int sl = 0; sl < NSL; ++sl) {              // 32-wide k slices of the stage
            const int coff = ((sl * 4 + (lane >> 4)) ^ swz) << 4;
            bf16x8 a[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) a[mt] = *reinterpret_cast<const bf16x8*>(St + aoff + mt * 16 * RB + coff);
            // low piece first in every expert tile (the sum of a tile is taken in that order); piece by piece
            // across the tiles, so that consecutive MFMAs do not wait for each other's result
            bf16x8 b[3][NTH];
#pragma unroll
            for (int pz = 0; pz < 3; ++pz)
#pragma unroll
                for (int nt = 0; nt < NTH; ++nt)
                    b[pz][nt] = *reinterpret_cast<const bf16x8*>(St + pz * p.m_pad * RB + boff[nt] + coff);
#pragma unroll
            for (int pz = 2; pz >= 0; --pz)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int nt = 0; nt < NTH; ++nt)
                        acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[mt], b[pz][nt], acc[mt][nt], 0, 0, 0);
        }
        // into the fp64 sums after every 64 k (d is a multiple of 64)
        if (KB == 64 || (ks & 1) == 1 || ks + 1 == ksteps) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < NTH; ++nt) {
#pragma unroll
                    for (int v = 0; v < 4; ++v) sum[mt][nt][v] += (double)acc[mt][nt][v];
                    acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
                }
        }
    }
    __syncthreads();                                    // every wave is done with the stages: reuse as logits
    float* logit = reinterpret_cast<float*>(gsm);       // [16*TG][m_pad]
#pragma unroll
    for (int nt = 0; nt < NTH; ++nt) {
        if (!tile_ok[nt]) continue;
        const int e = (eh * NTH + nt) * 16 + (lane & 15);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int tok = (tg + mt) * 16 + 4 * (lane >> 4) + v;
                double s = sum[mt][nt][v];
                if (p.bias != nullptr && e < p.m) s += (double)p.bias[e];
                logit[tok * p.m_pad + e] = (float)s;
            }
    }
    __syncthreads();
    if (p.K + 1 <= 16) {
        // four tokens per wavefront at a time
        for (int tok = wave * 4; tok < 16 * TG; tok += NWV * 4) {
            const int tl = tok + (lane >> 4);
            const bool valid = t0 + tl < p.T;
            const int tls = valid ? tl : tok;
            const bool ok = valid && t0 + tok < p.T;
            if (n_tiles <= 4) topk_rows<4>(p, logit, tls, t0 + tl, ok, lane, hist);
            else if (n_tiles <= 8) topk_rows<8>(p, logit, tls, t0 + tl, ok, lane, hist);
            else topk_rows<16>(p, logit, tls, t0 + tl, ok, lane, hist);
        }
    } else {
        for (int tok = wave; tok < 16 * TG; tok += NWV) {
            if (t0 + tok >= p.T) break;
            topk_token(p, logit + tok * p.m_pad, t0 + tok, lane, hist);
        }
    }
    __syncthreads();
    if (p.expert_cnt != nullptr)                        // small batches: the routing block counts the experts itself
        for (int i = tid; i < p.m; i += NWV * 64)
            if (hist[i] > 0) atomicAdd(&p.expert_cnt[i], hist[i]);
}

// ------------------------------------------------------------------------------------------------
// Algorithm 1 on the expert counts, one thread per expert (m <= 256).  Sorting is implicit: expert j
// precedes expert i in the order "count descending, id ascending" iff cnt_j > cnt_i or (equal and
// j < i); P_i = tokens covered before i is the sum of the counts of those j.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ void brownout_decide(const int* cnt_s, unsigned char* s2_s, int* unit_s, int m, int way,
                                                double threshold, int full, int tid, bool write,
                                                int32_t* expert_unit, uint8_t* expert_in_s1)
{
    // cnt_s: 16-byte aligned, zero from m up to the next multiple of 4 (a count of 0 adds nothing to P or S).
    // Four counts per LDS read, and sums in 32 bits (the counts add up to T K <= 2^30): the loop is bound by the
    // latency of its reads.
    bool in_s1 = false;
    if (tid < m) {
        const int c = cnt_s[tid];
        int P = 0, S = 0;
        const int4* c4 = reinterpret_cast<const int4*>(cnt_s);
        const int n4 = (m + 3) >> 2;
#pragma unroll 4
        for (int q = 0; q < n4; ++q) {
            const int4 v = c4[q];
            const int j = 4 * q;
            S += (v.x + v.y) + (v.z + v.w);
            P += (v.x > c || (v.x == c && j < tid)) ? v.x : 0;
            P += (v.y > c || (v.y == c && j + 1 < tid)) ? v.y : 0;
            P += (v.z > c || (v.z == c && j + 2 < tid)) ? v.z : 0;
            P += (v.w > c || (v.w == c && j + 3 < tid)) ? v.w : 0;
        }
        in_s1 = (double)P < (double)S * threshold;
        s2_s[tid] = (!in_s1 && c > 0) ? 1 : 0;
    }
    __syncthreads();
    if (tid < m) {
        const int g = tid / way, lo = g * way, hi = min(m, lo + way);
        int members = 0;
        for (int i = lo; i < hi; ++i) members += s2_s[i];
        int unit = tid;
        if (s2_s[tid]) {
            if (full) unit = -1;
            else if (members >= 2) unit = m + g;
        }
        unit_s[tid] = unit;
        if (write) {
            if (expert_unit) expert_unit[tid] = unit;
            if (expert_in_s1) expert_in_s1[tid] = in_s1 ? 1 : 0;
        }
    }
    __syncthreads();
}

struct RowArgs {
    const int32_t* topk_idx; const float* topk_w; const int32_t* expert_cnt;
    int32_t* expert_unit; uint8_t* expert_in_s1;
    int T, K, m, way, G, Ns, U, n_seg, full;
    double threshold;
    int32_t* seg_cnt; int32_t* seg_off;
    int32_t* unit_cnt; int32_t* unit_off; int32_t* n_rows;
    int32_t* row_token; float* row_weight; int32_t* token_rows;
    int32_t* expert_cnt_out;                               // small batches: the routing block counts the experts itself
    TileJobs jobs;                                         // GEMM tile tables to build (jobs.n == 0: none)
};

// One bit per token of the segment in bm[u]: token has a row in unit u.
__device__ __forceinline__ void mark_units(const RowArgs& p, const int* unit_s, unsigned long long* bm, int t, int lane)
{
    if (t < p.T) {
        const int32_t* idx = p.topk_idx + (size_t)t * p.K;
        for (int j = 0; j < p.K; ++j) {
            const int u = unit_s[idx[j]];
            if (u < 0) continue;
            atomicOr(&bm[u], 1ull << lane);   // a repeated united unit sets the same bit again
        }
        for (int s = 0; s < p.Ns; ++s) atomicOr(&bm[p.m + p.G + s], 1ull << lane);
    }
}

__global__ void __launch_bounds__(256) route_count_kernel(RowArgs p)
{
    __shared__ __attribute__((aligned(16))) int cnt_s[kMaxExperts];
    __shared__ int unit_s[kMaxExperts];
    __shared__ unsigned char s2_s[kMaxExperts];
    __shared__ unsigned long long bm[4][kMaxUnits];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    static_assert(kMaxExperts <= 256 && kMaxExperts % 4 == 0, "one thread per count, counts read four at a time");
    if (tid < kMaxExperts) cnt_s[tid] = tid < p.m ? p.expert_cnt[tid] : 0;
    for (int i = tid; i < 4 * kMaxUnits; i += 256) (&bm[0][0])[i] = 0ull;
    __syncthreads();
    brownout_decide(cnt_s, s2_s, unit_s, p.m, p.way, p.threshold, p.full, tid, blockIdx.x == 0, p.expert_unit,
                    p.expert_in_s1);
    const int seg = blockIdx.x * 4 + wave;
    mark_units(p, unit_s, bm[wave], seg * kSegTokens + lane, lane);
    __syncthreads();
    if (seg < p.n_seg)
        for (int u = lane; u < p.U; u += 64) p.seg_cnt[(size_t)seg * p.U + u] = __popcll(bm[wave][u]);
}

// One wavefront per unit: exclusive scan of the unit's rows over the segments (lane l owns a contiguous
// chunk of segments), and the unit's total.
__global__ void __launch_bounds__(256) route_scan_kernel(RowArgs p)
{
    const int lane = threadIdx.x & 63;
    const int u = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (u >= p.U) return;
    const int per = (p.n_seg + 63) / 64;
    const int s_lo = min(p.n_seg, lane * per), s_hi = min(p.n_seg, s_lo + per);
    int local = 0;
    for (int sgm = s_lo; sgm < s_hi; ++sgm) local += p.seg_cnt[(size_t)sgm * p.U + u];
    int incl = local;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int o = __shfl_up(incl, off);
        if (lane >= off) incl += o;
    }
    int run = incl - local;
    for (int sgm = s_lo; sgm < s_hi; ++sgm) {
        const int c = p.seg_cnt[(size_t)sgm * p.U + u];
        p.seg_off[(size_t)sgm * p.U + u] = run;
        run += c;
    }
    if (lane == 63) p.unit_cnt[u] = incl;
}

// Exclusive scan of unit_cnt into LDS (every block of the scatter needs all unit offsets); off_s[U] = total.
__device__ __forceinline__ void unit_offsets(const int32_t* unit_cnt, int U, int* off_s, int* wsum, int tid)
{
    const int lane = tid & 63, wave = tid >> 6;
    const int per = (U + 255) / 256;
    int local = 0;
    for (int q = 0; q < per; ++q) {
        const int u = tid * per + q;
        if (u < U) local += unit_cnt[u];
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
    for (int q = 0; q < per; ++q) {
        const int u = tid * per + q;
        if (u < U) {
            off_s[u] = base;
            base += unit_cnt[u];
            if (u == U - 1) off_s[U] = base;
        }
    }
    __syncthreads();
}

// Rows of token t (lane `lane` of its segment): off_s = first row of every unit, soff = rows of every unit
// in earlier segments, bmw = the segment's token bitmaps.
__device__ __forceinline__ void scatter_token(const RowArgs& p, const int* unit_s, const unsigned long long* bmw,
                                              const int* off_s, const int32_t* soff, int t, int lane)
{
    const unsigned long long below = (1ull << lane) - 1ull;
    const int32_t* idx = p.topk_idx + (size_t)t * p.K;
    const float* wts = p.topk_w + (size_t)t * p.K;
    const int slots = p.K + p.Ns;
    for (int j = 0; j < p.K; ++j) {
        const int u = unit_s[idx[j]];
        int row = -1;
        if (u >= 0) {
            bool first = true;
            if (u >= p.m)
                for (int q = 0; q < j; ++q)
                    if (unit_s[idx[q]] == u) first = false;
            if (first) {
                row = off_s[u] + soff[u] + __popcll(bmw[u] & below);
                float w = wts[j];
                if (u >= p.m)
                    for (int q = j + 1; q < p.K; ++q)
                        if (unit_s[idx[q]] == u) w += wts[q];     // merged entries, added in TopK order
                p.row_token[row] = t;
                p.row_weight[row] = w;
            }
        }
        p.token_rows[(size_t)t * slots + j] = row;
    }
    for (int s = 0; s < p.Ns; ++s) {
        const int u = p.m + p.G + s;
        const int row = off_s[u] + soff[u] + __popcll(bmw[u] & below);
        p.row_token[row] = t;
        p.row_weight[row] = 1.0f;
        p.token_rows[(size_t)t * slots + p.K + s] = row;
    }
}

__global__ void __launch_bounds__(256) route_scatter_kernel(RowArgs p)
{
    __shared__ int unit_s[kMaxExperts];
    __shared__ unsigned long long bm[4][kMaxUnits];
    __shared__ int off_s[kMaxUnits + 1];
    __shared__ int wsum[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    unit_offsets(p.unit_cnt, p.U, off_s, wsum, tid);
    if (blockIdx.x == 0) {
        for (int u = tid; u <= p.U; u += 256) p.unit_off[u] = off_s[u];
        if (tid == 0 && p.n_rows) p.n_rows[0] = off_s[p.U];
        if (wave < p.jobs.n) build_tile_table(p.unit_cnt, off_s, p.jobs.job[wave], p.jobs.cap, lane);
    }
    if (tid < p.m) unit_s[tid] = p.expert_unit[tid];
    for (int i = tid; i < 4 * kMaxUnits; i += 256) (&bm[0][0])[i] = 0ull;
    __syncthreads();
    const int seg = blockIdx.x * 4 + wave;
    const int t = seg * kSegTokens + lane;
    mark_units(p, unit_s, bm[wave], t, lane);
    __syncthreads();
    if (t >= p.T) return;
    scatter_token(p, unit_s, bm[wave], off_s, p.seg_off + (size_t)seg * p.U, t, lane);
}

// Small batches (at most 16 segments = 1024 tokens): Algorithm 1, the per-segment bitmaps, both scans and
// the scatter in ONE block of 16 wavefronts, one segment per wavefront, everything in LDS.  Dynamic LDS:
// bitmaps [16][U] (8 bytes) then segment offsets [16][U] (4 bytes).
__global__ void __launch_bounds__(1024) route_small_kernel(RowArgs p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char rsm[];
    __shared__ __attribute__((aligned(16))) int cnt_s[kMaxExperts];
    __shared__ int unit_s[kMaxExperts];
    __shared__ unsigned char s2_s[kMaxExperts];
    __shared__ int ucnt_s[kMaxUnits];
    __shared__ int off_s[kMaxUnits + 1];
    unsigned long long* bm = reinterpret_cast<unsigned long long*>(rsm);                      // [16][U]
    int* segoff = reinterpret_cast<int*>(rsm + (size_t)kSmallSegs * p.U * 8);                  // [16][U]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // cnt_i (the input of Algorithm 1) straight from the TopK lists: at most 1024 tokens, one thread each
    if (tid < kMaxExperts) cnt_s[tid] = 0;
    for (int i = tid; i < kSmallSegs * p.U; i += 1024) bm[i] = 0ull;
    __syncthreads();
    if (tid < p.T)
        for (int j = 0; j < p.K; ++j) atomicAdd(&cnt_s[p.topk_idx[(size_t)tid * p.K + j]], 1);
    __syncthreads();
    if (tid < p.m) p.expert_cnt_out[tid] = cnt_s[tid];
    brownout_decide(cnt_s, s2_s, unit_s, p.m, p.way, p.threshold, p.full, tid, true, p.expert_unit, p.expert_in_s1);
    const int t = wave * kSegTokens + lane;
    mark_units(p, unit_s, bm + (size_t)wave * p.U, t, lane);
    __syncthreads();
    for (int u = tid; u < p.U; u += 1024) {
        int run = 0;
        for (int sgm = 0; sgm < kSmallSegs; ++sgm) {
            segoff[sgm * p.U + u] = run;
            run += __popcll(bm[(size_t)sgm * p.U + u]);
        }
        ucnt_s[u] = run;
        p.unit_cnt[u] = run;
    }
    __syncthreads();
    if (wave == 0) {                                     // exclusive scan of the unit counts by one wavefront
        const int per = (p.U + 63) / 64;
        const int lo = min(p.U, lane * per), hi = min(p.U, lo + per);
        int local = 0;
        for (int u = lo; u < hi; ++u) local += ucnt_s[u];
        int incl = local;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int o = __shfl_up(incl, off);
            if (lane >= off) incl += o;
        }
        int run = incl - local;
        for (int u = lo; u < hi; ++u) {
            off_s[u] = run;
            run += ucnt_s[u];
        }
        if (lane == 63) off_s[p.U] = incl;
    }
    __syncthreads();
    for (int u = tid; u <= p.U; u += 1024) p.unit_off[u] = off_s[u];
    if (tid == 0 && p.n_rows) p.n_rows[0] = off_s[p.U];
    // the GEMM tile tables, by the last wavefronts (the first ones hold the tokens of a short batch)
    if (15 - wave < p.jobs.n) build_tile_table(ucnt_s, off_s, p.jobs.job[15 - wave], p.jobs.cap, lane);
    if (t < p.T) scatter_token(p, unit_s, bm + (size_t)wave * p.U, off_s, segoff + wave * p.U, t, lane);
}

constexpr int kGateFewLds = 3 * 4 * 64 * 128;          // three stages of four 64-row pieces (gate_few_kernel)
constexpr int kGateLds = 160 * 1024;                    // LDS of one CU (the tiled gate also holds a 1 KiB histogram)

#define BMOE_GATE_TILED_ALL(X) \
    X(4, 2, 64, 1, 2) X(4, 2, 32, 1, 2) X(4, 4, 64, 1, 2) X(4, 1, 32, 2, 8) X(4, 2, 32, 2, 8) \
    X(2, 2, 64, 1, 2) X(2, 2, 32, 1, 2) X(2, 1, 64, 2, 8) X(2, 4, 32, 1, 2) X(2, 2, 32, 2, 8) \
    X(1, 1, 64, 1, 8) X(1, 2, 32, 1, 8) X(1, 1, 64, 1, 4)

hipError_t init_route_kernels()
{
    hipError_t e;
#define BMOE_SET(TG_, NTH_, KB_, MT_, EG_)                                                                  \
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(gate_tiled_kernel<TG_, NTH_, KB_, MT_, EG_>),  \
                            hipFuncAttributeMaxDynamicSharedMemorySize, kGateLds - 1024);                \
    if (e != hipSuccess) return e;
    BMOE_GATE_TILED_ALL(BMOE_SET)
#undef BMOE_SET
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(gate_few_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                            kGateFewLds);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(route_small_kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, kSmallSegs * kMaxUnits * 12);
}

hipError_t launch_pack_gate(const float* gate_w, int m, int m_pad, int d, bf16_t* packed, hipStream_t s)
{
    if (m_pad == 16)     // at most 16 experts: the fp64 gate reads fp32 rows, the packed form is a copy of them
        return hipMemcpyAsync(packed, gate_w, (size_t)m * d * 4, hipMemcpyDeviceToDevice, s);
    const size_t n = (size_t)m_pad * d;
    const int blocks = (int)std::min<size_t>((n + 255) / 256, 2048);
    prep_kernel<<<blocks, 256, 0, s>>>(gate_w, m, m_pad, d, reinterpret_cast<unsigned short*>(packed), nullptr);
    return hipGetLastError();
}

hipError_t launch_route(const Dims& D, const bf16_t* x, const void* gate, const float* gate_bias,
                        double threshold, int full_brownout, const RouteBufs& R, bf16_t* gate_split,
                        int32_t* seg_cnt, int32_t* seg_off, const TileJobs& jobs, hipStream_t s)
{
    hipError_t e = ensure_device_init(nullptr);
    if (e != hipSuccess) return e;
    const bool small = D.n_seg <= kSmallSegs;            // one block routes the whole batch (and counts the experts)
    const bool packed = D.gate_format == MOE_GATE_PACKED;
    // At most 16 experts: the gate matrix is fp32 rows in either format, and up to kFewExpertsTokens tokens the
    // plain fp64 gate reads them as they are (larger batches: cut here on every call, 6 us, then the MFMA gate).
    const bool few_fmt = D.m_pad == 16;
    const bool few = few_fmt && D.T <= kFewExpertsTokens;
    // Preparation: cut an fp32 gate matrix into its pieces (only the MFMA gates need them) and clear the expert
    // counters (only large batches use them).  A small batch with a packed gate or few experts needs neither.
    const bool split = !few && (!packed || few_fmt);
    if (split || !small) {
        ProfScope ps(MOE_STAGE_PREP, s);
        const size_t n = split ? (size_t)D.m_pad * D.d : (size_t)D.m;
        const int blocks = (int)std::min<size_t>((n + 255) / 256, 2048);
        prep_kernel<<<blocks, 256, 0, s>>>(split ? static_cast<const float*>(gate) : nullptr, D.m, D.m_pad, D.d,
                                           split ? reinterpret_cast<unsigned short*>(gate_split) : nullptr,
                                           small ? nullptr : R.expert_cnt);
    }
    {
        ProfScope ps(MOE_STAGE_GATE, s);
        GateArgs g;
        g.x = x;
        g.split = split ? reinterpret_cast<const unsigned short*>(gate_split) : static_cast<const unsigned short*>(gate);
        g.bias = gate_bias;
        g.T = D.T; g.d = D.d; g.m = D.m; g.m_pad = D.m_pad; g.K = D.K; g.score_fn = D.score_fn; g.n_stage = 3;
        const int n_tiles = D.m_pad / 16;
        g.topk_idx = R.topk_idx; g.topk_w = R.topk_w; g.near_tie = R.near_tie;
        g.expert_cnt = small ? nullptr : R.expert_cnt;
        const int half_tiles = ceil_div(n_tiles, 2);
        // 32 experts and more: LDS-staged variant, with wider token tiles once the batch fills the CUs with them
        const int tgw = n_tiles < 2 ? 0 : (n_tiles >= 4 && D.T >= 64 * 192 ? 4 : (n_tiles >= 4 && D.T >= 32 * 192 ? 2 : 1));
        if (few) {
            const float* gw = static_cast<const float*>(gate);      // fp32 rows in either gate format
            if (D.m <= 8) gate_small_kernel<8, 1><<<D.T, 256, 0, s>>>(g, gw);
            else gate_small_kernel<16, 1><<<D.T, 256, 0, s>>>(g, gw);
        } else if (tgw != 0) {
            const int rows = 3 * D.m_pad + 16 * tgw;
            const bool wide = D.m_pad <= 128 && 3 * rows * 128 <= kGateLds - 1024;    // 64-wide k stages fit
            const int stage = rows * (wide ? 128 : 64);
            g.n_stage = std::max(3, std::min(8, (kGateLds - 1024) / stage));
            const int lds = std::max(g.n_stage * stage, 16 * tgw * D.m_pad * 4);
            const int blocks = ceil_div(D.T, 16 * tgw);
#define BMOE_GATE_TILED(TG_, NTH_, KB_, MT_, EG_) \
    gate_tiled_kernel<TG_, NTH_, KB_, MT_, EG_><<<blocks, (TG_ / MT_) * EG_ * 64, lds, s>>>(g)
            // Wave layouts, each measured against its neighbours (more, smaller waves win: the loop is bound by
            // the latency of its LDS reads and barrier, not by bytes).  Up to 4 expert tiles: a wave holds one
            // token tile and half of the experts.  Up to 8: two token tiles and one expert tile per wave, 8 expert
            // groups.  Up to 16: two token tiles and two expert tiles, 8 groups.
            static_assert(kMaxExperts <= 256, "8 expert groups of two tiles cover every expert");
            if (tgw == 1) {
                if (n_tiles <= 4) BMOE_GATE_TILED(1, 1, 64, 1, 4);
                else if (n_tiles <= 8) BMOE_GATE_TILED(1, 1, 64, 1, 8);      // (wide stages always fit here)
                else BMOE_GATE_TILED(1, 2, 32, 1, 8);
            } else if (tgw == 4) {
                if (half_tiles <= 2) { if (wide) BMOE_GATE_TILED(4, 2, 64, 1, 2); else BMOE_GATE_TILED(4, 2, 32, 1, 2); }
                else if (half_tiles <= 4) { if (wide) BMOE_GATE_TILED(4, 4, 64, 1, 2); else BMOE_GATE_TILED(4, 1, 32, 2, 8); }
                else BMOE_GATE_TILED(4, 2, 32, 2, 8);
            } else {
                if (half_tiles <= 2) { if (wide) BMOE_GATE_TILED(2, 2, 64, 1, 2); else BMOE_GATE_TILED(2, 2, 32, 1, 2); }
                else if (half_tiles <= 4) { if (wide) BMOE_GATE_TILED(2, 1, 64, 2, 8); else BMOE_GATE_TILED(2, 4, 32, 1, 2); }
                else BMOE_GATE_TILED(2, 2, 32, 2, 8);
            }
#undef BMOE_GATE_TILED
        } else {
            // at most 16 experts beyond kFewExpertsTokens tokens
            gate_few_kernel<<<ceil_div(D.T, 16), 512, kGateFewLds, s>>>(g);
        }
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    RowArgs p;
    p.topk_idx = R.topk_idx; p.topk_w = R.topk_w; p.expert_cnt = R.expert_cnt;
    p.expert_unit = R.expert_unit; p.expert_in_s1 = R.expert_in_s1;
    p.T = D.T; p.K = D.K; p.m = D.m; p.way = D.way; p.G = D.G; p.Ns = D.Ns; p.U = D.U; p.n_seg = D.n_seg;
    p.full = full_brownout; p.threshold = threshold;
    p.seg_cnt = seg_cnt; p.seg_off = seg_off; p.unit_cnt = R.unit_cnt; p.unit_off = R.unit_off; p.n_rows = R.n_rows;
    p.row_token = R.row_token; p.row_weight = R.row_weight; p.token_rows = R.token_rows;
    p.expert_cnt_out = R.expert_cnt;
    p.jobs = jobs;
    if (small) {
        ProfScope ps(MOE_STAGE_COUNT, s);
        route_small_kernel<<<1, 1024, (size_t)kSmallSegs * D.U * 12, s>>>(p);
        return hipGetLastError();
    }
    const int seg_blocks = ceil_div(D.n_seg, 4);
    {
        ProfScope ps(MOE_STAGE_COUNT, s);
        route_count_kernel<<<seg_blocks, 256, 0, s>>>(p);
    }
    {
        ProfScope ps(MOE_STAGE_SCAN, s);
        route_scan_kernel<<<ceil_div(D.U, 4), 256, 0, s>>>(p);
    }
    {
        ProfScope ps(MOE_STAGE_SCATTER, s);
        route_scatter_kernel<<<seg_blocks, 256, 0, s>>>(p);
    }
    return hipGetLastError();
}

}  // namespace bmoe
