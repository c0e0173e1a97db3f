// lm_head_topk: the draft model's fp16 language-model head (a GEMV-shaped fp16 x fp16 product over a
// vocabulary-sized weight, HBM-bound), the log-softmax of its logits and their top-k.  Contract in
// include/w4a16.h.
#include "internal.h"

namespace w4 {

typedef _Float16 half8v __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kLmDepth = 4;        // macro steps of weights in flight per wavefront
constexpr int kLmStepK = 128;      // k per macro step: 256 contiguous bytes of every weight row
constexpr int kLmChunk = 512;      // logits per wavefront of the top-k pass
constexpr int kLmThreads = 256;
constexpr int kLmMaxTopK = 64;

// Packed LM-head weight: the vocabulary (padded to a multiple of 16 with zero rows) is cut into tiles
// of 16 tokens; tile t is one contiguous run of K / 32 blocks of 1 KB, block s holding W[16 t + c]
// [32 s + 8 r .. + 7] at byte (16 r + c) * 16 -- the first operand of one 16x16x32 MFMA for lane
// (r, c), so a wavefront's loads are 1 KB contiguous each and its whole tile is one linear stream.
__global__ void lm_head_pack_kernel(const _Float16 *__restrict__ W, u32x4 *__restrict__ packed, int V, int K,
                                    long long total)
{
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;   // one 16-byte piece each
    if (idx >= total) return;
    const int lane = (int)(idx & 63);
    const long long blk = idx >> 6;
    const int steps = K / 32;
    const int s = (int)(blk % steps);
    const int tile = (int)(blk / steps);
    const int r = lane >> 4, c = lane & 15;
    const int v = tile * 16 + c;
    u32x4 piece = {0u, 0u, 0u, 0u};
    if (v < V) piece = *reinterpret_cast<const u32x4 *>(W + (size_t)v * K + 32 * s + 8 * r);
    packed[idx] = piece;
}

// Logits.  A wavefront owns one vocabulary tile (16 tokens = the rows of the MFMA result, the up to 16
// hidden-state rows its columns) and streams the tile's K / 32 blocks with a ring of kLmDepth macro
// steps (4 blocks = 4 KB each) in flight; the x fragments (at most 16 x K fp16, L2-resident) are
// re-read per wavefront, which works on two neighbouring tiles at once so that each fragment serves
// both.  Tiles lie K * 32 bytes apart, a power of two for the usual hidden sizes:
// wavefronts that all walked k from 0 would ask the same few memory channels at any moment, so each
// starts at macro step (tile mod steps) and wraps around.
template <bool EVEN, int TWL, int MTL, int DEPTH>
__global__ __launch_bounds__(256) void lm_head_logits_kernel(const _Float16 *__restrict__ x,
                                                             const u32x4 *__restrict__ packed,
                                                             float *__restrict__ logits, int M, int V, int K, int tiles)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane >> 4, c = lane & 15;
    const int tile0 = (blockIdx.x * 4 + wave) * TWL;   // TWL consecutive tiles share every x fragment
    if (tile0 >= tiles) return;   // no barrier in this kernel
    const int steps = K / kLmStepK;
    const u32x4 *wp[TWL];
#pragma unroll
    for (int t = 0; t < TWL; ++t)   // a tile past the end repeats the last one; its logits are not stored
        wp[t] = packed + (size_t)min(tile0 + t, tiles - 1) * (K / 32) * 64 + lane;
    const u32x4 *xp[MTL];           // MTL row tiles of 16 hidden-state rows; rows >= M repeat row M-1, never stored
#pragma unroll
    for (int mt = 0; mt < MTL; ++mt) xp[mt] = reinterpret_cast<const u32x4 *>(x + (size_t)min(mt * 16 + c, M - 1) * K + 8 * r);
    u32x4 w[DEPTH][TWL][4], xf[DEPTH][MTL][4];
    const int rot = (tile0 / TWL) % steps;
    auto load = [&](int s, int slot) {
        int sr = s + rot;              // uniform
        sr = sr >= steps ? sr - steps : sr;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
#pragma unroll
            for (int t = 0; t < TWL; ++t) w[slot][t][j] = __builtin_nontemporal_load(wp[t] + (sr * 4 + j) * 64);
#pragma unroll
            for (int mt = 0; mt < MTL; ++mt) xf[slot][mt][j] = xp[mt][(sr * 4 + j) * 4];
        }
    };
    float4v acc[TWL][MTL];
#pragma unroll
    for (int t = 0; t < TWL; ++t)
#pragma unroll
        for (int mt = 0; mt < MTL; ++mt) acc[t][mt] = (float4v){0.f, 0.f, 0.f, 0.f};
    auto compute = [&](int slot) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int t = 0; t < TWL; ++t)
#pragma unroll
                for (int mt = 0; mt < MTL; ++mt)
                    acc[t][mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8v, w[slot][t][j]),
                                                                        __builtin_bit_cast(half8v, xf[slot][mt][j]),
                                                                        acc[t][mt], 0, 0, 0);
    };
    if constexpr (EVEN) {   // steps is a multiple of the ring depth: every load of the steady state is unconditional
#pragma unroll
        for (int u = 0; u < DEPTH; ++u) load(u, u);
        int s0 = 0;
        for (; s0 + DEPTH < steps; s0 += DEPTH) {
#pragma unroll
            for (int u = 0; u < DEPTH; ++u) {
                compute(u);
                load(s0 + u + DEPTH, u);
            }
        }
#pragma unroll
        for (int u = 0; u < DEPTH; ++u) compute(u);
    } else {
#pragma unroll
        for (int u = 0; u < DEPTH; ++u)
            if (u < steps) load(u, u);
        for (int s0 = 0; s0 < steps; s0 += DEPTH) {
#pragma unroll
            for (int u = 0; u < DEPTH; ++u) {
                if (s0 + u < steps) {   // uniform
                    compute(u);
                    if (s0 + u + DEPTH < steps) load(s0 + u + DEPTH, u);
                }
            }
        }
    }
    // lane (r, c) holds the logits of tokens 16 tile + 4 r .. + 3 for hidden-state row 16 mt + c
#pragma unroll
    for (int t = 0; t < TWL; ++t)
#pragma unroll
        for (int mt = 0; mt < MTL; ++mt) {
            const int v0 = (tile0 + t) * 16 + 4 * r, row = mt * 16 + c;
            if (row < M && tile0 + t < tiles) {
                float *dst = logits + (size_t)row * V + v0;
                if ((V & 3) == 0 && v0 + 3 < V) {
                    *reinterpret_cast<float4v *>(dst) = acc[t][mt];
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (v0 + i < V) dst[i] = acc[t][mt][i];
                }
            }
        }
}

// (value, token) pairs ordered by value, equal values by ascending token
struct Cand {
    float val;
    int idx;
};
// (bitwise operators on purpose: no short-circuit branches in the scan loops)
__device__ __forceinline__ bool better(const Cand &a, const Cand &b) { return (a.val > b.val) | ((a.val == b.val) & (a.idx < b.idx)); }

// Wavefront-wide maximum / minimum, returned to every lane, on the data-parallel-primitive path of the
// vector ALU (no LDS round trips): quad butterflies, rotations inside each row of 16 lanes, then the
// four row results are read into scalars.
template <int CTRL>
__device__ __forceinline__ int dpp_move(int v)
{
    return __builtin_amdgcn_update_dpp(v, v, CTRL, 0xF, 0xF, false);
}
constexpr int kQuadXor1 = 0xB1, kQuadXor2 = 0x4E, kRowRor4 = 0x124, kRowRor8 = 0x128;

__device__ __forceinline__ float wave_max(float v)
{
    v = fmaxf(v, __builtin_bit_cast(float, dpp_move<kQuadXor1>(__builtin_bit_cast(int, v))));
    v = fmaxf(v, __builtin_bit_cast(float, dpp_move<kQuadXor2>(__builtin_bit_cast(int, v))));
    v = fmaxf(v, __builtin_bit_cast(float, dpp_move<kRowRor4>(__builtin_bit_cast(int, v))));
    v = fmaxf(v, __builtin_bit_cast(float, dpp_move<kRowRor8>(__builtin_bit_cast(int, v))));
    const int iv = __builtin_bit_cast(int, v);
    const float a = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 0));
    const float b = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 16));
    const float c = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 32));
    const float d = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 48));
    return fmaxf(fmaxf(a, b), fmaxf(c, d));
}

__device__ __forceinline__ int wave_min(int v)
{
    v = min(v, dpp_move<kQuadXor1>(v));
    v = min(v, dpp_move<kQuadXor2>(v));
    v = min(v, dpp_move<kRowRor4>(v));
    v = min(v, dpp_move<kRowRor8>(v));
    return min(min(__builtin_amdgcn_readlane(v, 0), __builtin_amdgcn_readlane(v, 16)),
               min(__builtin_amdgcn_readlane(v, 32), __builtin_amdgcn_readlane(v, 48)));
}

// best pair of the wavefront, returned to every lane: the largest value, and among the lanes that
// hold it the smallest token
__device__ __forceinline__ Cand wave_best(Cand mine)
{
    const float vmax = wave_max(mine.val);
    const int imin = wave_min(mine.val == vmax ? mine.idx : 0x7FFFFFFF);
    return {vmax, imin};
}

// butterfly sum over the wavefront (fixed order), returned to every lane
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

constexpr float kNegInf = -__builtin_inff();
constexpr int kNoToken = 0x7FFFFFFF;

// Pass 1 over the logits: one WAVEFRONT per chunk of 512 logits of one row (no barriers: the top_k
// rounds are shuffles only).  Per chunk: maximum, sum of exp(l - max) and the chunk's top_k
// (value, token) pairs, largest first.  Lane l holds logits l, l + 64, ... of the chunk.
__global__ __launch_bounds__(kLmThreads) void lm_head_chunk_kernel(const float *__restrict__ logits, int V, int top_k,
                                                                   int chunks, float *__restrict__ chunk_max,
                                                                   float *__restrict__ chunk_sum,
                                                                   float *__restrict__ cand_val, int *__restrict__ cand_idx)
{
    constexpr int kPerLane = kLmChunk / 64;
    fetch_arguments_together(logits, V, top_k, chunks, chunk_max, chunk_sum, cand_val, cand_idx);
    const int lane = threadIdx.x & 63;
    const int chunk = blockIdx.x * (kLmThreads / 64) + (threadIdx.x >> 6), m = blockIdx.y;
    if (chunk >= chunks) return;
    const float *row = logits + (size_t)m * V;
    const int base = chunk * kLmChunk + lane;
    float val[kPerLane];
#pragma unroll
    for (int i = 0; i < kPerLane; ++i) val[i] = base + 64 * i < V ? row[base + 64 * i] : kNegInf;
    // a lane's tokens ascend with i, so a strict comparison keeps the lowest token among equal values;
    // retired and padding entries are -inf and never win
    auto lane_best = [&]() {
        Cand b = {kNegInf, kNoToken};
#pragma unroll
        for (int i = 0; i < kPerLane; ++i) {
            const bool win = val[i] > b.val;
            b.val = win ? val[i] : b.val;
            b.idx = win ? base + 64 * i : b.idx;
        }
        return b;
    };
    Cand mine = lane_best();
    Cand best = wave_best(mine);
    const float mx = best.val;   // every chunk holds at least one token
    float se = 0.f;
#pragma unroll
    for (int i = 0; i < kPerLane; ++i) se += __expf(val[i] - mx);   // exp(-inf) = 0 for the padding
    se = wave_sum(se);
    const size_t slot = (size_t)m * chunks + chunk;
    if (lane == 0) {
        chunk_max[slot] = mx;
        chunk_sum[slot] = se;
    }
    for (int round = 0; round < top_k; ++round) {
        if (round > 0) best = wave_best(mine);
        if (lane == 0) {
            cand_val[slot * top_k + round] = best.val;
            cand_idx[slot * top_k + round] = best.idx;
        }
        if (best.idx == mine.idx && best.idx != kNoToken) {   // the owner retires the winner and looks again
#pragma unroll
            for (int i = 0; i < kPerLane; ++i) val[i] = best.idx == base + 64 * i ? kNegInf : val[i];
            mine = lane_best();
        }
    }
}

// Pass 2: one wavefront per row merges the chunks: log of the sum of exponentials, then a k-way merge of
// the chunks' candidate lists (each already sorted, largest first), which sit in LDS: lane l owns the
// lists of chunks l, l + 64, ... and keeps their current heads in registers; per round the best head of
// the wavefront is emitted and its owner advances that list.
constexpr int kLmListsPerLane = 8;            // chunks <= 512
constexpr int kLmMaxCandidates = 8192;        // chunks * top_k, 64 KB of LDS
__global__ __launch_bounds__(kLmThreads) void lm_head_merge_kernel(const float *__restrict__ chunk_max,
                                                           const float *__restrict__ chunk_sum,
                                                           const float *__restrict__ cand_val,
                                                           const int *__restrict__ cand_idx, int chunks, int top_k,
                                                           int32_t *__restrict__ top_idx, float *__restrict__ top_logprob)
{
    extern __shared__ float lds_f[];
    fetch_arguments_together(chunk_max, chunk_sum, cand_val, cand_idx, chunks, top_k, top_idx, top_logprob);
    const int m = blockIdx.x, lane = threadIdx.x & 63;
    const int total = chunks * top_k;
    float *lval = lds_f;
    int *lidx = reinterpret_cast<int *>(lds_f + total);
    // the first wavefront's share of the chunk maxima and sums, requested together with the lists
    float cmax[kLmListsPerLane], csum[kLmListsPerLane];
#pragma unroll
    for (int h = 0; h < kLmListsPerLane; ++h) {
        const int ch = lane + 64 * h, chc = ch < chunks ? ch : chunks - 1;   // clamped address, value discarded:
        const float a = chunk_max[(size_t)m * chunks + chc];                 // no branch around the load
        const float b = chunk_sum[(size_t)m * chunks + chc];
        cmax[h] = ch < chunks ? a : kNegInf;
        csum[h] = ch < chunks ? b : 0.f;
    }
    {   // all four wavefronts stage the lists, every load of a thread in flight at once: whether a round of
        // loads happens is a uniform decision and a lane past the end reads the last entry (and drops it), so
        // no load sits under a per-lane condition, which would be compiled as a branch with a wait of its own
        constexpr int kPer = kLmMaxCandidates / kLmThreads;
        const int rounds = (total + kLmThreads - 1) / kLmThreads;
        float sv[kPer];
        int si[kPer];
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            if (i < rounds) {
                const int e = threadIdx.x + kLmThreads * i, ec = e < total ? e : total - 1;
                sv[i] = cand_val[(size_t)m * total + ec];
                si[i] = cand_idx[(size_t)m * total + ec];
            }
        }
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            const int e = threadIdx.x + kLmThreads * i;
            if (i < rounds && e < total) {
                lval[e] = sv[i];
                lidx[e] = si[i];
            }
        }
    }
    __syncthreads();
    if (threadIdx.x >= 64) return;   // the merge itself is one wavefront's work
    float mx = kNegInf;
#pragma unroll
    for (int h = 0; h < kLmListsPerLane; ++h) mx = fmaxf(mx, cmax[h]);
    mx = wave_max(mx);
    float se = 0.f;
#pragma unroll
    for (int h = 0; h < kLmListsPerLane; ++h) se += csum[h] * __expf(cmax[h] - mx);   // absent chunks: 0 * exp(-inf) = 0
    se = wave_sum(se);
    const float lse = mx + __logf(se);
    Cand head[kLmListsPerLane];
    int ptr[kLmListsPerLane];
#pragma unroll
    for (int h = 0; h < kLmListsPerLane; ++h) {
        const int ch = lane + 64 * h;
        ptr[h] = 0;
        head[h] = ch < chunks ? Cand{lval[ch * top_k], lidx[ch * top_k]} : Cand{kNegInf, kNoToken};
    }
    for (int round = 0; round < top_k; ++round) {
        Cand mine = {kNegInf, kNoToken};
#pragma unroll
        for (int h = 0; h < kLmListsPerLane; ++h) {
            const bool win = better(head[h], mine);
            mine.val = win ? head[h].val : mine.val;
            mine.idx = win ? head[h].idx : mine.idx;
        }
        const Cand best = wave_best(mine);
        if (lane == 0) {
            top_idx[m * top_k + round] = best.idx;
            top_logprob[m * top_k + round] = best.val - lse;
        }
        if (best.idx == mine.idx && best.idx != kNoToken) {   // the owner advances the list the winner came from
#pragma unroll
            for (int h = 0; h < kLmListsPerLane; ++h) {
                if (head[h].idx == best.idx) {
                    ++ptr[h];
                    const int e = (lane + 64 * h) * top_k + ptr[h];
                    head[h] = ptr[h] < top_k ? Cand{lval[e], lidx[e]} : Cand{kNegInf, kNoToken};
                }
            }
        }
    }
}

static int lm_chunks(int V) { return (V + kLmChunk - 1) / kLmChunk; }

static int check_lm_head(int M, int V, int K, int top_k)
{
    if (M < 1 || V < 1 || K < 1 || top_k < 1 || top_k > V) return W4A16_EINVAL;
    if (K % kLmStepK != 0) return W4A16_EINVAL;
    if (M > W4A16_MAX_M || top_k > kLmMaxTopK) return W4A16_EUNSUP;
    if (lm_chunks(V) > 64 * kLmListsPerLane || (long long)lm_chunks(V) * top_k > kLmMaxCandidates) return W4A16_EUNSUP;
    return W4A16_OK;
}

}  // namespace w4

using namespace w4;

extern "C" {

size_t lm_head_packed_bytes(int V, int K)
{
    if (V < 1 || K < 1 || K % kLmStepK != 0) return 0;
    return (size_t)((V + 15) / 16) * 16 * K * sizeof(_Float16);
}

int lm_head_pack(const void *W, void *packed, int V, int K, void *stream)
{
    if (V < 1 || K < 1 || K % kLmStepK != 0) return W4A16_EINVAL;
    if (!W || !packed) return W4A16_ENULL;
    if (misaligned(W) || misaligned(packed)) return W4A16_EALIGN;
    const long long total = (long long)((V + 15) / 16) * (K / 32) * 64;
    hipLaunchKernelGGL(lm_head_pack_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                       (const _Float16 *)W, (u32x4 *)packed, V, K, total);
    return launch_status();
}

size_t lm_head_workspace_bytes(int M, int V, int K, int top_k)
{
    if (check_lm_head(M, V, K, top_k) != W4A16_OK) return 0;
    const size_t slots = (size_t)M * lm_chunks(V);
    return slots * 2 * sizeof(float) + slots * top_k * (sizeof(float) + sizeof(int)) + 256;
}

int lm_head_topk(const void *x, const void *packed, int M, int V, int K, int top_k, float *logits, int32_t *top_idx,
                 float *top_logprob, void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = check_lm_head(M, V, K, top_k);
    if (rc != W4A16_OK) return rc;
    if (!x || !packed || !logits || !top_idx || !top_logprob) return W4A16_ENULL;
    if (misaligned(x) || misaligned(packed) || misaligned(logits) || misaligned(workspace)) return W4A16_EALIGN;
    if ((reinterpret_cast<uintptr_t>(top_idx) | reinterpret_cast<uintptr_t>(top_logprob)) & 3u) return W4A16_EALIGN;
    if (!workspace || workspace_bytes < lm_head_workspace_bytes(M, V, K, top_k)) return W4A16_EWORKSPACE;
    const int tiles = (V + 15) / 16, chunks = lm_chunks(V);
    const size_t slots = (size_t)M * chunks;
    float *chunk_max = reinterpret_cast<float *>(workspace);
    float *chunk_sum = chunk_max + slots;
    float *cand_val = chunk_sum + slots;
    int *cand_idx = reinterpret_cast<int *>(cand_val + slots * top_k);
    static bool lds_ok = false;   // LDS above 48 KB needs an opt-in, once
    if (!lds_ok) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&lm_head_merge_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kLmMaxCandidates * 8) != hipSuccess)
            return W4A16_EHIP;
        lds_ok = true;
    }
    hipStream_t s = (hipStream_t)stream;
    // tiles per wavefront: every x fragment fetched from L2 serves all of them, which matters once the
    // hidden-state rows differ (K = 4096: M = 16 240 -> 194 us with two, M = 60 567 -> 278 us with four); a
    // single row is a broadcast and runs best with one.  More than 16 rows: up to four row tiles and a
    // ring of two macro steps (registers).
    const int mtl = (M + 15) / 16;
    const int twl = params().lm_tiles > 0 ? params().lm_tiles : (M <= 4 ? 1 : M <= 16 ? 2 : 4);
    if (twl != 1 && twl != 2 && !(twl == 4 && mtl >= 2)) return W4A16_EUNSUP;
    const int depth = mtl > 1 ? 2 : kLmDepth;
    const bool even = (K / kLmStepK) % depth == 0;
    const dim3 grid((unsigned)((tiles + 4 * twl - 1) / (4 * twl)));
#define W4_LM_LAUNCH(TWL_, MTL_, DEPTH_)                                                                                \
    do {                                                                                                                \
        if (even)                                                                                                       \
            hipLaunchKernelGGL((lm_head_logits_kernel<true, TWL_, MTL_, DEPTH_>), grid, dim3(256), 0, s,                \
                               (const _Float16 *)x, (const u32x4 *)packed, logits, M, V, K, tiles);                     \
        else                                                                                                            \
            hipLaunchKernelGGL((lm_head_logits_kernel<false, TWL_, MTL_, DEPTH_>), grid, dim3(256), 0, s,               \
                               (const _Float16 *)x, (const u32x4 *)packed, logits, M, V, K, tiles);                     \
    } while (0)
    if (mtl == 1 && twl == 1) W4_LM_LAUNCH(1, 1, kLmDepth);
    else if (mtl == 1) W4_LM_LAUNCH(2, 1, kLmDepth);
    else if (mtl == 2 && twl == 1) W4_LM_LAUNCH(1, 2, 2);
    else if (mtl == 2 && twl == 2) W4_LM_LAUNCH(2, 2, 2);
    else if (mtl == 2) W4_LM_LAUNCH(4, 2, 2);
    else if (mtl == 3 && twl == 1) W4_LM_LAUNCH(1, 3, 2);
    else if (mtl == 3 && twl == 2) W4_LM_LAUNCH(2, 3, 2);
    else if (mtl == 3) W4_LM_LAUNCH(4, 3, 2);
    else if (twl == 1) W4_LM_LAUNCH(1, 4, 2);
    else if (twl == 2) W4_LM_LAUNCH(2, 4, 2);
    else W4_LM_LAUNCH(4, 4, 2);
#undef W4_LM_LAUNCH
    hipLaunchKernelGGL(lm_head_chunk_kernel, dim3((unsigned)((chunks + kLmThreads / 64 - 1) / (kLmThreads / 64)), (unsigned)M), dim3(kLmThreads), 0, s,
                       (const float *)logits, V, top_k, chunks, chunk_max, chunk_sum, cand_val, cand_idx);
    hipLaunchKernelGGL(lm_head_merge_kernel, dim3((unsigned)M), dim3(kLmThreads), (size_t)chunks * top_k * 8, s, (const float *)chunk_max,
                       (const float *)chunk_sum, (const float *)cand_val, (const int *)cand_idx, chunks, top_k, top_idx,
                       top_logprob);
    return launch_status();
}

}  // extern "C"
