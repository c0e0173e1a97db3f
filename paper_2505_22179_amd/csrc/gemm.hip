// w4a16_gemm: y[M,N] = x[M,K] . dequant(packed)[K,N] for 1 <= M <= 64 on gfx950.
//
// The layer (paper section 2.2: 4-bit weights in groups of 128 with fp16 activations) is bound by
// streaming the packed weight from HBM for every M in range, so the kernel is organised around
// that stream: each wavefront owns one 128-column block and a set of quantisation groups, pulls
// each group's record (8 KB of codes + scales + zero-points, see layout.h) with 16-byte loads
// straight into registers, turns the codes into exact small-integer fp16 values (q - z), and
// feeds them as the second operand of 16x16x32 fp16 MFMA steps whose first operand is the
// matching x fragment.  The group's integer-weight partial product is then folded into the fp32
// accumulators with one multiply-add by the group's scale, so no weight is ever rounded to fp16
// (w = (q - z) * s needs 15 significand bits) and the only rounding is fp32 accumulation.
// Wavefronts of a workgroup split the K range and are summed through LDS; workgroups may split K
// further, in which case fp32 partials go through a caller workspace and are summed in a fixed
// order (by the last workgroup to finish a column block, or by a second kernel), so results do
// not depend on scheduling.
#include "internal.h"

namespace w4 {

typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef _Float16 half4v __attribute__((ext_vector_type(4)));
typedef _Float16 half8v __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kWaves = 4;              // wavefronts per workgroup, each on its own groups
constexpr int kThreads = kWaves * 64;

// x fragments of one group: MT row tiles x four 32-wide k steps, plus the group's scales and zeros
template <int MT>
struct GroupOperands {
    u32x4 a[MT][4];
    u32x4 s;        // eight fp16 scales
    uint32_t z;     // eight 4-bit zero-points
};

__device__ __forceinline__ half2v as_h2(uint32_t u) { return __builtin_bit_cast(half2v, u); }

// (w & mask) | magic in one VALU instruction (the mask rides in an SGPR, the magic in a VGPR:
// VOP3 encodings take no literal on this ISA, which is why the compiler splits it in two)
__device__ __forceinline__ uint32_t and_or(uint32_t w, uint32_t mask, uint32_t magic)
{
    uint32_t out;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(out) : "v"(w), "s"(mask), "v"(magic));
    return out;
}

// eight codes of one packed word -> eight fp16 values (q - z), exactly.
// 0x6400 | q is the fp16 number 1024 + q; 0x6400 | (q << 4) is 1024 + 16 q.
__device__ __forceinline__ half8v dequant8(uint32_t w, half2v zneg, half2v zneg16, uint32_t magic)
{
    const half2v sixteenth = {(_Float16)0.0625f, (_Float16)0.0625f};
    uint32_t w2 = w >> 8;
    half2v b0 = as_h2(and_or(w, 0x000F000Fu, magic)) + zneg;                    // p0 p1
    half2v b1 = as_h2(and_or(w, 0x00F000F0u, magic)) * sixteenth + zneg16;      // p2 p3
    half2v b2 = as_h2(and_or(w2, 0x000F000Fu, magic)) + zneg;                   // p4 p5
    half2v b3 = as_h2(and_or(w2, 0x00F000F0u, magic)) * sixteenth + zneg16;     // p6 p7
    half4v lo = __builtin_shufflevector(b0, b1, 0, 1, 2, 3);
    half4v hi = __builtin_shufflevector(b2, b3, 0, 1, 2, 3);
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

__device__ __forceinline__ u32x4 load_tile(const uint8_t *rec, int t, int lane)
{
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(rec + t * 1024 + lane * 16));
}

template <int MT>
__device__ __forceinline__ void load_operands(GroupOperands<MT> &f, const uint8_t *rec,
                                              const _Float16 *const (&xp)[MT], int g, int c)
{
    f.s = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(rec + kScalesOff + c * 16));
    f.z = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(rec + kZerosOff + c * 4));
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            f.a[mt][j] = *reinterpret_cast<const u32x4 *>(xp[mt] + (size_t)g * kGroup + j * 32);
}

// One quantisation group for this wavefront's eight column tiles.  As soon as a tile's codes have
// been expanded its registers are refilled with the same tile of the wavefront's next group, so
// one group of codes (8 KB per wavefront) is always in flight without a second register set.
template <int MT>
__device__ __forceinline__ void compute_group(const GroupOperands<MT> &f, u32x4 (&w)[kTiles],
                                              float4v (&acc)[kTiles][MT], const uint8_t *next_rec,
                                              bool has_next, int lane, uint32_t magic)
{
#pragma unroll
    for (int t = 0; t < kTiles; ++t) {
        uint32_t z = (f.z >> (4 * t)) & 0xFu;
        uint32_t zz = z | (z << 16);
        half2v zneg = as_h2(zz | 0xE400E400u);            // -(1024 + z)
        half2v zneg16 = as_h2((zz << 4) | 0xD400D400u);   // -(64 + z)
        half8v b[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) b[j] = dequant8(w[t][j], zneg, zneg16, magic);
        if (has_next) w[t] = load_tile(next_rec, t, lane);
        float4v part[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) part[mt] = (float4v){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                part[mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8v, f.a[mt][j]), b[j],
                                                                  part[mt], 0, 0, 0);
        uint32_t sw = f.s[t >> 1];
        _Float16 sh = __builtin_bit_cast(_Float16, (uint16_t)((t & 1) ? (sw >> 16) : (sw & 0xFFFFu)));
        float s = (float)sh;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[t][mt] += s * part[mt];
    }
}

// element e of a column block's fragment-ordered result -> (row m, column n)
template <int MT>
__device__ __forceinline__ void store_elem(_Float16 *__restrict__ y, float v, int e, int nb, int M, int N)
{
    int ln = e & 63, reg = e >> 6;
    int i = reg & 3, tm = reg >> 2;
    int mt = tm % MT, t = tm / MT;
    int m = mt * 16 + 4 * (ln >> 4) + i;
    int n = nb * kBlockCols + t * 16 + (ln & 15);
    if (m < M && n < N) y[(size_t)m * N + n] = (_Float16)v;
}

template <int MT>
__global__ __launch_bounds__(kThreads, (MT == 1 ? 3 : 1)) void gemm_kernel(
    const _Float16 *__restrict__ x, const uint8_t *__restrict__ packed, _Float16 *__restrict__ y,
    float *__restrict__ partial, uint32_t *__restrict__ tickets, int M, int N, int K, int groups, int S, int fused)
{
    extern __shared__ float lds[];
    __shared__ uint32_t ticket_sh;
    constexpr int R = 32 * MT;     // accumulator registers per lane
    constexpr int E = R * 64;      // fp32 results per column block
    constexpr int Q = E / kThreads;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: keeps the group loop scalar
    const int r = lane >> 4, c = lane & 15;
    const int nb = blockIdx.x / S, ks = blockIdx.x % S;
    const int g_begin = (int)((long long)groups * ks / S);
    const int g_end = (int)((long long)groups * (ks + 1) / S);

    const _Float16 *xp[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        int row = mt * 16 + c;
        row = row < M ? row : M - 1;   // rows >= M are never read; their products are never stored
        xp[mt] = x + (size_t)row * K + r * 8;
    }
    const uint8_t *rec0 = packed + record_offset(nb, 0, groups);

    float4v acc[kTiles][MT];
#pragma unroll
    for (int t = 0; t < kTiles; ++t)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[t][mt] = (float4v){0.f, 0.f, 0.f, 0.f};

    GroupOperands<MT> fa, fb;
    u32x4 w[kTiles];
    uint32_t magic = 0x64006400u;
    asm volatile("" : "+v"(magic));   // keep it in a VGPR rather than a literal
    int g = g_begin + wave;
    if (g < g_end) {
        const uint8_t *rec = rec0 + (size_t)g * kRecordBytes;
#pragma unroll
        for (int t = 0; t < kTiles; ++t) w[t] = load_tile(rec, t, lane);
        load_operands<MT>(fa, rec, xp, g, c);
    }
    while (g < g_end) {
        int gn = g + kWaves;
        bool more = gn < g_end;
        const uint8_t *rec = rec0 + (size_t)gn * kRecordBytes;
        if (more) load_operands<MT>(fb, rec, xp, gn, c);
        compute_group<MT>(fa, w, acc, rec, more, lane, magic);
        g = gn;
        if (!more) break;
        gn = g + kWaves;
        more = gn < g_end;
        rec = rec0 + (size_t)gn * kRecordBytes;
        if (more) load_operands<MT>(fa, rec, xp, gn, c);
        compute_group<MT>(fb, w, acc, rec, more, lane, magic);
        g = gn;
    }

    // sum the wavefronts' accumulators through LDS, wave 0 first (fixed order)
#pragma unroll
    for (int t = 0; t < kTiles; ++t)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                lds[(wave * R + (t * MT + mt) * 4 + i) * 64 + lane] = acc[t][mt][i];
    __syncthreads();
    float *mine = partial + (size_t)blockIdx.x * E;
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        int e = tid + kThreads * q;
        float v = lds[e];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) v += lds[w * E + e];
        if (S == 1) store_elem<MT>(y, v, e, nb, M, N);
        else mine[e] = v;
    }
    if (S == 1) return;
    if (!fused) return;
    // the last workgroup of this column block to arrive sums all S partials in split order
    __threadfence();
    __syncthreads();
    if (tid == 0) ticket_sh = atomicAdd(&tickets[nb], 1u);
    __syncthreads();
    if (ticket_sh != (uint32_t)(S - 1)) return;
    __threadfence();
    const float *all = partial + (size_t)nb * S * E;
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        int e = tid + kThreads * q;
        float v = 0.f;
        for (int s = 0; s < S; ++s)
            v += __hip_atomic_load(all + (size_t)s * E + e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        store_elem<MT>(y, v, e, nb, M, N);
    }
    if (tid == 0) __hip_atomic_store(&tickets[nb], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// second pass of the two-kernel split-K mode: one workgroup per column block
template <int MT>
__global__ __launch_bounds__(kThreads) void splitk_reduce_kernel(const float *__restrict__ partial,
                                                                 _Float16 *__restrict__ y, int M, int N, int S)
{
    constexpr int E = 32 * MT * 64;
    constexpr int Q = E / kThreads;
    const int nb = blockIdx.x, tid = threadIdx.x;
    const float *all = partial + (size_t)nb * S * E;
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        int e = tid + kThreads * q;
        float v = 0.f;
        for (int s = 0; s < S; ++s) v += all[(size_t)s * E + e];
        store_elem<MT>(y, v, e, nb, M, N);
    }
}

// ---- host side ---------------------------------------------------------------------------------

static int choose_split(int mt, int nblocks, int groups)
{
    const Params &p = params();
    int cap = groups / kWaves > 0 ? groups / kWaves : 1;   // every wavefront gets at least one group
    if (cap > 64) cap = 64;
    if (p.split_k > 0) return p.split_k < groups ? p.split_k : groups;
    int per_cu = p.wgs_per_cu > 0 ? p.wgs_per_cu : (mt == 1 ? 3 : (mt == 2 ? 2 : 1));
    double target = 256.0 * per_cu;
    int best = 1;
    double best_cost = 1e30;
    for (int s = 1; s <= cap; ++s) {
        double ratio = (double)nblocks * s / target;
        double cost = ratio > 1 ? ratio - 1 : 1 / ratio - 1;
        if (groups % (s * kWaves) != 0) cost += 0.25;       // uneven work per wavefront
        if (cost < best_cost) { best_cost = cost; best = s; }
    }
    return best;
}

static size_t partial_bytes(int mt, int nblocks, int S)
{
    return S > 1 ? (size_t)nblocks * S * (32 * mt * 64) * sizeof(float) : 0;
}

template <int MT>
static int launch(const void *x, const void *packed, void *y, int M, int N, int K, int S, void *workspace,
                  hipStream_t stream)
{
    static bool lds_ok = false;   // LDS above 64 KB needs an opt-in, once per kernel
    const size_t lds_bytes = (size_t)kWaves * 32 * MT * 64 * sizeof(float);
    if (!lds_ok && lds_bytes > 48 * 1024) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_kernel<MT>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes) != hipSuccess)
            return W4A16_EHIP;
        lds_ok = true;
    }
    const int groups = K / kGroup, nblocks = pad_cols(N) / kBlockCols;
    const int fused = params().fused_reduce;
    uint32_t *tickets = reinterpret_cast<uint32_t *>(workspace);
    float *partial = reinterpret_cast<float *>(reinterpret_cast<uint8_t *>(workspace) + kTicketBytes);
    hipLaunchKernelGGL(gemm_kernel<MT>, dim3((unsigned)(nblocks * S)), dim3(kThreads), lds_bytes, stream,
                       (const _Float16 *)x, (const uint8_t *)packed, (_Float16 *)y, partial, tickets, M, N, K,
                       groups, S, fused);
    if (S > 1 && !fused)
        hipLaunchKernelGGL(splitk_reduce_kernel<MT>, dim3((unsigned)nblocks), dim3(kThreads), 0, stream,
                           (const float *)partial, (_Float16 *)y, M, N, S);
    return launch_status();
}

}  // namespace w4

using namespace w4;

extern "C" {

size_t w4a16_workspace_bytes(int M_max, int N, int K, int G)
{
    if (check_weight_shape(N, K, G) != W4A16_OK || M_max < 1 || M_max > W4A16_MAX_M) return 0;
    const int groups = K / kGroup, nblocks = pad_cols(N) / kBlockCols;
    size_t need = 0;
    for (int mt = 1; mt <= (M_max + 15) / 16; ++mt) {
        size_t b = partial_bytes(mt, nblocks, choose_split(mt, nblocks, groups));
        if (b > need) need = b;
    }
    return kTicketBytes + need;
}

int w4a16_gemm(const void *x, const void *packed, void *y, int M, int N, int K, int G,
               void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = check_weight_shape(N, K, G);
    if (rc != W4A16_OK) return rc;
    if (M < 1) return W4A16_EINVAL;
    if (M > W4A16_MAX_M) return W4A16_EUNSUP;
    if (!x || !packed || !y) return W4A16_ENULL;
    if (misaligned(x) || misaligned(packed) || misaligned(y) || misaligned(workspace)) return W4A16_EALIGN;
    const int groups = K / kGroup, nblocks = pad_cols(N) / kBlockCols;
    const int mt = (M + 15) / 16;
    int S = choose_split(mt, nblocks, groups);
    if (S > 1 && nblocks > kMaxTickets) S = 1;
    if (S > 1) {
        if (!workspace) return W4A16_EWORKSPACE;
        if (workspace_bytes < kTicketBytes + partial_bytes(mt, nblocks, S)) return W4A16_EWORKSPACE;
    }
    hipStream_t st = (hipStream_t)stream;
    switch (mt) {
    case 1: return launch<1>(x, packed, y, M, N, K, S, workspace, st);
    case 2: return launch<2>(x, packed, y, M, N, K, S, workspace, st);
    case 3: return launch<3>(x, packed, y, M, N, K, S, workspace, st);
    default: return launch<4>(x, packed, y, M, N, K, S, workspace, st);
    }
}

}  // extern "C"
