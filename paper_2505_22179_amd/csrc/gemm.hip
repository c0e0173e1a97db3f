// w4a16_gemm: y[M,N] = x[M,K] . dequant(packed)[K,N] for 1 <= M <= 64 on gfx950.
//
// The layer (paper section 2.2: 4-bit weights in groups of 128 with fp16 activations) is bound by
// streaming the packed weight from HBM for every M in range, so the kernel is organised around
// that stream: each wavefront owns TW 16-column tiles of one 128-column block and a set of
// quantisation groups, pulls each group's codes (1 KB per tile, see layout.h) with 16-byte loads
// straight into registers, turns them into exact small-integer fp16 values (q - z), and feeds them
// as the second operand of 16x16x32 fp16 MFMA steps whose first operand is the matching x
// fragment.  The group's integer-weight partial product is then folded into the fp32 accumulators
// with one multiply-add by the group's scale, so no weight is ever rounded to fp16
// (w = (q - z) * s needs 15 significand bits) and the only rounding is fp32 accumulation.
// The four wavefronts of a workgroup split the K range and are summed through LDS; workgroups may
// split K further, in which case fp32 partials go through a caller workspace and are summed in a
// fixed order (by the last workgroup to finish a column unit, or by a second kernel), so results
// do not depend on scheduling.
#include "internal.h"
#include "devscope.h"

namespace w4 {

typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef _Float16 half4v __attribute__((ext_vector_type(4)));
typedef _Float16 half8v __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// scales and zero-points of one record, as a lane needs them (column = lane % 16 of every tile)
struct QuantWords {
    u32x4 s;        // eight fp16 scales (all eight tiles of the record)
    uint32_t z;     // eight 4-bit zero-points
};

// x fragments of one group: MT row tiles x four 32-wide k steps, plus the group's scales and zeros
template <int MT>
struct GroupOperands {
    u32x4 a[MT][4];
    QuantWords q;
};

__device__ __forceinline__ half2v as_h2(uint32_t u) { return __builtin_bit_cast(half2v, u); }

// Constants of the code expansion, kept in registers: (w & mask) | magic then selects to the single
// three-operand v_and_or_b32, which takes no literal on this ISA (with literal operands the
// compiler has to split it into an AND and an OR).
struct DequantConsts {
    uint32_t magic;     // 0x6400 in both halves: fp16 1024
    uint32_t mask_lo;   // 0x000F000F
    uint32_t mask_hi;   // 0x00F000F0
    uint32_t magic64;   // 0x5400 in both halves: fp16 64, whose mantissa bits 4..7 count in ones
};

__device__ __forceinline__ DequantConsts dequant_consts()
{
    DequantConsts k = {0x64006400u, 0x000F000Fu, 0x00F000F0u, 0x54005400u};
    asm volatile("" : "+v"(k.magic));    // opaque to constant propagation: stays in a VGPR
    asm volatile("" : "+v"(k.magic64));
    asm volatile("" : "+s"(k.mask_lo));  // stay in SGPRs
    asm volatile("" : "+s"(k.mask_hi));
    return k;
}

// eight codes of one packed word -> eight fp16 values (q - z), exactly.
// 0x6400 | q is the fp16 number 1024 + q; 0x6400 | (q << 4) is 1024 + 16 q.
__device__ __forceinline__ half8v dequant8(uint32_t w, half2v zneg, half2v zneg16, const DequantConsts &k)
{
    const half2v sixteenth = {(_Float16)0.0625f, (_Float16)0.0625f};
    uint32_t w2 = w >> 8;
    half2v b0 = as_h2((w & k.mask_lo) | k.magic) + zneg;                    // p0 p1
    half2v b1 = as_h2((w & k.mask_hi) | k.magic) * sixteenth + zneg16;      // p2 p3
    half2v b2 = as_h2((w2 & k.mask_lo) | k.magic) + zneg;                   // p4 p5
    half2v b3 = as_h2((w2 & k.mask_hi) | k.magic) * sixteenth + zneg16;     // p6 p7
    half4v lo = __builtin_shufflevector(b0, b1, 0, 1, 2, 3);
    half4v hi = __builtin_shufflevector(b2, b3, 0, 1, 2, 3);
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

__device__ __forceinline__ u32x4 load_tile(const uint8_t *rec, int t, int lane)
{
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(rec + t * 1024 + lane * 16));
}

// a pointer the compiler can keep in scalar registers: both halves are read from the first lane
typedef const __attribute__((address_space(1))) uint8_t *global_bytes;   // global, not generic: no flat loads
__device__ __forceinline__ global_bytes uniform_ptr(const uint8_t *p)
{
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (global_bytes)(((uint64_t)hi << 32) | lo);
}
template <typename T>
__device__ __forceinline__ T load_global(global_bytes p)
{
    return *(const __attribute__((address_space(1))) T *)p;
}

// Symmetric weights (paper section 2.2: GPTQ quantises symmetrically, so every zero-point is the mid-code 8):
// kernels instantiated with SYM never read the zero-points and use the constants below instead.
constexpr uint32_t kSymZeros = 0x88888888u;      // the zero-point word such a weight holds
constexpr uint32_t kSymZneg = 0xE408E408u;       // fp16 pair -(1024 + 8)
constexpr uint32_t kSymZneg16 = 0xD480D480u;     // fp16 pair -(64 + 8)

template <int MT, bool SYM = false>
__device__ __forceinline__ void load_operands(GroupOperands<MT> &f, const uint8_t *rec,
                                              const _Float16 *const (&xp)[MT], int g, int c)
{
    f.q.s = *reinterpret_cast<const u32x4 *>(rec + kScalesOff + c * 16);
    if constexpr (SYM) f.q.z = kSymZeros;
    else f.q.z = *reinterpret_cast<const uint32_t *>(rec + kZerosOff + c * 4);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            f.a[mt][j] = *reinterpret_cast<const u32x4 *>(xp[mt] + (size_t)g * kGroup + j * 32);
    __builtin_amdgcn_sched_barrier(0);
}

// scale / zero-point words of this wavefront's TW tiles (tiles t0 .. t0+TW-1 of the record's eight)
template <int TW>
struct TileQuant {
    uint32_t zbits;                 // 4-bit zero-points, tile t in bits 4t..4t+3
    uint32_t sw[(TW + 1) / 2];      // fp16 scales, two per word
};

template <int TW>
__device__ __forceinline__ TileQuant<TW> tile_quant(const QuantWords &f, int t0)
{
    TileQuant<TW> q;
    q.zbits = f.z >> (4 * t0);
    const uint32_t s0 = f.s[0], s1 = f.s[1], s2 = f.s[2], s3 = f.s[3];
    if constexpr (TW == 8) {
        q.sw[0] = s0; q.sw[1] = s1; q.sw[2] = s2; q.sw[3] = s3;
    } else if constexpr (TW == 4) {
        q.sw[0] = t0 ? s2 : s0;
        q.sw[1] = t0 ? s3 : s1;
    } else {
        q.sw[0] = (t0 & 4) ? ((t0 & 2) ? s3 : s2) : ((t0 & 2) ? s1 : s0);
    }
    return q;
}

// the four second operands (k steps) of one tile: exact fp16 (q - z)
template <int TW, bool SYM = false>
__device__ __forceinline__ void dequant_tile(half8v (&b)[4], const u32x4 &w, const TileQuant<TW> &q, int t,
                                             const DequantConsts &magic)
{
    uint32_t z = (q.zbits >> (4 * t)) & 0xFu;
    uint32_t zz = z | (z << 16);
    half2v zneg = as_h2(SYM ? kSymZneg : (zz | 0xE400E400u));              // -(1024 + z)
    half2v zneg16 = as_h2(SYM ? kSymZneg16 : ((zz << 4) | 0xD400D400u));   // -(64 + z)
#pragma unroll
    for (int j = 0; j < 4; ++j) b[j] = dequant8(w[j], zneg, zneg16, magic);
}


// ---- offset-code arithmetic for one row tile (M <= 16) ------------------------------------------
// With few rows the vector ALU, not the matrix pipe, is the scarce unit, and two thirds of its work
// per weight is turning the biased code into (q - z).  Here the second operand keeps the bias:
// 0x6400 | q is 1024 + q in the low-nibble positions, and in the high-nibble ones, where the code
// sits four bits up, 0x5400 | (q << 4) is 64 + q (one unit of those mantissa bits of 64 is 1).  With
// the bias B_k (1024 or 64) of position k, one group and one column give
//     T = sum_k x_k b_k = sum_k x_k q_k + sum_k B_k x_k,
// so with C = sum_k B_k x_k and X = sum_k x_k (two more products of the same fragment with
// constant operands, shared by all column tiles) the group's term is s (T - C - z X).  T - C is
// formed inside the matrix pipe by starting the accumulation from -C.  Every operand is exact in
// fp16 and all sums are fp32: inputs whose products are exact stay exact; otherwise the
// cancellation of the bias costs up to ten bits of the fp32 significand in each group's term, which
// leaves it far more precise than the fp16 result.
constexpr bool kOffsetCodes = true;   // one-row-tile kernels use the arithmetic above

__device__ __forceinline__ half8v offset8(uint32_t w, const DequantConsts &k)
{
    const uint32_t w2 = w >> 8;
    const u32x4 v = {(w & k.mask_lo) | k.magic, (w & k.mask_hi) | k.magic64, (w2 & k.mask_lo) | k.magic,
                     (w2 & k.mask_hi) | k.magic64};
    return __builtin_bit_cast(half8v, v);
}

__device__ __forceinline__ void offset_tile(half8v (&b)[4], const u32x4 &w, const DequantConsts &magic)
{
#pragma unroll
    for (int j = 0; j < 4; ++j) b[j] = offset8(w[j], magic);
}

// -C and X of one group for MT row tiles (every column of the result holds the same value)
template <int MT>
__device__ __forceinline__ void group_sums(const u32x4 (&a)[MT][4], float4v (&negc)[MT], float4v (&xs)[MT])
{
    const u32x4 bias = {0xE400E400u, 0xD400D400u, 0xE400E400u, 0xD400D400u};     // -1024 or -64: the position's bias
    const u32x4 ones = {0x3C003C00u, 0x3C003C00u, 0x3C003C00u, 0x3C003C00u};
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        negc[mt] = (float4v){0.f, 0.f, 0.f, 0.f};
        xs[mt] = (float4v){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            negc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8v, a[mt][j]),
                                                               __builtin_bit_cast(half8v, bias), negc[mt], 0, 0, 0);
            xs[mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8v, a[mt][j]),
                                                             __builtin_bit_cast(half8v, ones), xs[mt], 0, 0, 0);
        }
    }
}

// Symmetric weights: z = 8 everywhere, so -C and -8 X are one sum over the same fragment, with -(1024 + 8) at the
// low-nibble positions and -(64 + 8) at the high-nibble ones.  Started from it, the
// matrix pipe leaves sum_k x_k (q_k - 8) and the fold is a plain multiply-add: four constant products per group
// instead of eight, one fused multiply-add per live accumulator register instead of two.
template <int MT>
__device__ __forceinline__ void group_sums_symmetric(const u32x4 (&a)[MT][4], float4v (&negc)[MT])
{
    const u32x4 bias = {0xE408E408u, 0xD480D480u, 0xE408E408u, 0xD480D480u};     // -1032 or -72
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        negc[mt] = (float4v){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < 4; ++j)
            negc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8v, a[mt][j]),
                                                               __builtin_bit_cast(half8v, bias), negc[mt], 0, 0, 0);
    }
}

__device__ __forceinline__ void fold_symmetric(float4v &acc, const float4v &part, float s, bool more_rows)
{
    acc[0] += s * part[0];
    if (more_rows) {   // uniform: M > 1
        asm volatile("");   // keeps this a branch, as in fold_offset
#pragma unroll
        for (int i = 1; i < 4; ++i) acc[i] += s * part[i];
    }
}

// acc += s (part - z X) for the rows that exist: register i of a lane is row 4 * (lane / 16) + i
__device__ __forceinline__ void fold_offset(float4v &acc, const float4v &part, const float4v &xs, float s, float zf,
                                            bool more_rows)
{
    acc[0] += s * (part[0] - zf * xs[0]);
    if (more_rows) {   // uniform: M > 1
        asm volatile("");   // keeps this a branch: if-converted, M = 1 would pay for all four rows
#pragma unroll
        for (int i = 1; i < 4; ++i) acc[i] += s * (part[i] - zf * xs[i]);
    }
}

// One quantisation group for this wavefront's TW column tiles, software-pipelined over tiles:
// while the matrix pipe works on tile t (its operand `bc` was expanded one stage earlier), the
// vector ALU expands tile t+1 -- or tile 0 of the wavefront's next group at the last stage -- and
// the registers of every expanded tile are refilled at once with the same tile DEPTH groups ahead,
// so the code stream never stalls on its own arithmetic.
//   f, w      operands and codes of this group;  fn, wn  those of the next group (ring neighbour)
//   bc        in: expanded tile 0 of this group; out: expanded tile 0 of the next group
template <int MT, int TW, bool ALWAYS_REFILL, bool OFF = false, bool SYM = false>
__device__ __forceinline__ void compute_group(u32x4 (&a)[MT][4], const QuantWords &f, const QuantWords &fn,
                                              u32x4 (&w)[TW], u32x4 (&wn)[TW], half8v (&bc)[4],
                                              float4v (&acc)[TW][MT], const uint8_t *refill_rec, bool refill,
                                              bool next_group, int t0, int lane, const DequantConsts &magic,
                                              bool more_rows = true)
{
    const TileQuant<TW> q = tile_quant<TW>(f, t0);
    const TileQuant<TW> qn = tile_quant<TW>(fn, t0);
    float4v negc[MT], xs[MT];
    if constexpr (OFF) {
        if constexpr (SYM) group_sums_symmetric<MT>(a, negc);
        else group_sums<MT>(a, negc, xs);
    }
#pragma unroll
    for (int t = 0; t < TW; ++t) {
        // tile t was expanded during the previous stage: its code registers are free again
        if (ALWAYS_REFILL || refill) w[t] = load_tile(refill_rec, t0 + t, lane);
        __builtin_amdgcn_sched_barrier(0);   // loads stay where they are written
        half8v bn[4];
        if constexpr (OFF) {
            if (t + 1 < TW) offset_tile(bn, w[t + 1 < TW ? t + 1 : 0], magic);
            else if (ALWAYS_REFILL || next_group) offset_tile(bn, wn[0], magic);
        } else {
            if (t + 1 < TW) dequant_tile<TW, SYM>(bn, w[t + 1 < TW ? t + 1 : 0], q, t + 1, magic);
            else if (ALWAYS_REFILL || next_group) dequant_tile<TW, SYM>(bn, wn[0], qn, 0, magic);
        }
        float4v part[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) part[mt] = OFF ? negc[mt] : (float4v){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                part[mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8v, a[mt][j]), bc[j],
                                                                  part[mt], 0, 0, 0);
        uint32_t s2 = q.sw[t >> 1];
        _Float16 sh = __builtin_bit_cast(_Float16, (uint16_t)((t & 1) ? (s2 >> 16) : (s2 & 0xFFFFu)));
        float s = (float)sh;
        if constexpr (OFF && SYM) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) fold_symmetric(acc[t][mt], part[mt], s, more_rows);
        } else if constexpr (OFF) {
            const float zf = (float)((q.zbits >> (4 * t)) & 0xFu);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) fold_offset(acc[t][mt], part[mt], xs[mt], s, zf, more_rows);
        } else {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) acc[t][mt] += s * part[mt];
        }
        // interleave: one matrix instruction, then a share of the next tile's expansion
#pragma unroll
        for (int i = 0; i < 4 * MT; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                          // MFMA
            __builtin_amdgcn_sched_group_barrier(0x002, ((OFF ? 24 : SYM ? 36 : 40) + 4 * MT - 1) / (4 * MT), 0);   // VALU
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < 4; ++j) bc[j] = bn[j];
    }
}

// Four consecutive elements e4*4 .. e4*4+3 of a column unit's fragment-ordered result are four
// consecutive columns of one output row: round to fp16 and store them as one 8-byte word.
// Fragment order: e = ((t * MT + mt) * 4 + i) * 64 + lane, row = mt*16 + 4*(lane/16) + i,
// column = first_col + t*16 + lane%16.
// output row of quad e4 (see the fragment order below); partial sums of rows >= M are never moved
template <int MT>
__device__ __forceinline__ int quad_row(int e4)
{
    const int reg = e4 >> 4;
    return ((reg >> 2) % MT) * 16 + 4 * (((e4 * 4) & 63) >> 4) + (reg & 3);
}

// Where the finished sums go.  epi selects what is stored: the sums themselves, the sums plus a
// residual of the same shape (which may be y itself), or -- for a weight whose 16-column tiles
// alternate between a gate projection and an up projection -- silu(gate) * up, half as wide.
// or -- for a q/k/v projection whose heads were packed with their two halves alternating tile by tile -- the
// rotary embedding of the q and k heads and the scatter of q, k and v to their own buffers (kEpiRope).
// The last two are the paired epilogues: one thread finishes a quad of a packed tile 2j together with the
// quad of tile 2j+1 that belongs to it.
constexpr int kEpiNone = 0, kEpiResidual = 1, kEpiSiluMul = 2, kEpiRope = 3;
struct RopeOut {   // arguments of rope_append, minus the fp16 q/k/v rows, which are the linear's own sums
    const int32_t *pos;
    const float *cos_t, *sin_t;
    _Float16 *q, *k_cache, *v_cache;
    int n_pos, P, Hq, Hkv, D;
};
struct Out {
    _Float16 *y;
    const _Float16 *residual;
    int epi;
    RopeOut rope;
    int sym;   // host side only: the caller vouches that every zero-point of the weight is 8
};
__device__ __forceinline__ bool paired_epilogue(const Out &o) { return o.epi >= kEpiSiluMul; }

// The residual of a quad is fetched apart from the store, so that a thread can request the residuals of all
// its quads (and the partial sums it has to add) before it waits for any of them: inside the store, under
// the per-lane bounds test, each load became a branch with a wait of its own -- one memory round trip per
// quad, in a row.  The load is unconditional: a quad outside the matrix reads a clamped address and its value
// is never used (with y == residual that may be a location another thread is writing: just as unused).
template <int MT>
__device__ __forceinline__ half4v load_residual(const Out &o, int e4, int first_col, int M, int N)
{
    half4v r = {(_Float16)0.f, (_Float16)0.f, (_Float16)0.f, (_Float16)0.f};
    if (o.residual) {   // uniform
        int ln = (e4 * 4) & 63, reg = e4 >> 4;
        int i = reg & 3, tm = reg >> 2;
        int mt = tm % MT, t = tm / MT;
        int m = mt * 16 + 4 * (ln >> 4) + i;
        int n = first_col + t * 16 + (ln & 15);
        m = m < M ? m : M - 1;
        n = n < N ? n : N - 4;
        r = *reinterpret_cast<const half4v *>(o.residual + (size_t)m * N + n);
    }
    return r;
}

template <int MT>
__device__ __forceinline__ void store_quad(const Out &o, float4v v, half4v r, int e4, int first_col, int M, int N)
{
    int ln = (e4 * 4) & 63, reg = e4 >> 4;
    int i = reg & 3, tm = reg >> 2;
    int mt = tm % MT, t = tm / MT;
    int m = mt * 16 + 4 * (ln >> 4) + i;
    int n = first_col + t * 16 + (ln & 15);
    if (m < M && n < N) {   // N % 8 == 0 and n % 4 == 0: the quad never straddles the edge
        if (o.residual) v += (float4v){(float)r[0], (float)r[1], (float)r[2], (float)r[3]};   // uniform
        half4v h = {(_Float16)v[0], (_Float16)v[1], (_Float16)v[2], (_Float16)v[3]};
        *reinterpret_cast<half4v *>(o.y + (size_t)m * N + n) = h;
    }
}

template <int MT>
__device__ __forceinline__ void store_quad(const Out &o, float4v v, int e4, int first_col, int M, int N)
{
    store_quad<MT>(o, v, load_residual<MT>(o, e4, first_col, M, N), e4, first_col, M, N);
}

// Sum over the S split-K partials of Q quads, in split order from zero.  The loads are unconditional (a quad of
// rows that do not exist reads whatever the workspace holds; its sum is never stored) and go out four splits
// at a time, so a thread waits for a batch, not for each load: under the row test, or in a plain loop over the
// splits, every partial had been a memory round trip of its own.  LOAD(index) fetches quad `index` of the unit.
constexpr int kSplitBatch = 4;
template <int Q, typename Load>
__device__ __forceinline__ void sum_partials(float4v (&sum)[Q], const int (&e4)[Q], int S, int E4, Load load)
{
#pragma unroll
    for (int q = 0; q < Q; ++q) sum[q] = (float4v){0.f, 0.f, 0.f, 0.f};
    for (int s0 = 0; s0 < S; s0 += kSplitBatch) {
        float4v v[kSplitBatch][Q];
#pragma unroll
        for (int i = 0; i < kSplitBatch; ++i) {
            const int sc = s0 + i < S ? s0 + i : S - 1;   // uniform
#pragma unroll
            for (int q = 0; q < Q; ++q) v[i][q] = load(sc * E4 + e4[q]);
        }
#pragma unroll
        for (int i = 0; i < kSplitBatch; ++i)
            if (s0 + i < S) {   // uniform
#pragma unroll
                for (int q = 0; q < Q; ++q) sum[q] += v[i][q];
            }
    }
}

// Gated epilogue.  In a column unit the quads of one tile are 64 * MT consecutive indices, tile after
// tile, and the tiles alternate gate, up, gate, up ...: pair index idx (0 .. E4/2 - 1) names the gate
// quad gate_quad(idx); its up quad lies 64 * MT further on.
template <int MT>
__device__ __forceinline__ int gate_quad(int idx)
{
    constexpr int kTileQuads = 64 * MT;
    return idx + (idx / kTileQuads) * kTileQuads;
}

__device__ __forceinline__ float silu_mul(float g, float u) { return g / (1.f + __expf(-g)) * u; }

// stores silu(g) * u for gate quad e4 (N is the width of the packed weight; the output is N / 2 wide)
template <int MT>
__device__ __forceinline__ void store_gated(const Out &o, float4v g, float4v u, int e4, int first_col, int M, int N)
{
    int ln = (e4 * 4) & 63, reg = e4 >> 4;
    int i = reg & 3, tm = reg >> 2;
    int mt = tm % MT, t = tm / MT;          // t is even: a gate tile
    int m = mt * 16 + 4 * (ln >> 4) + i;
    int n = (first_col >> 1) + (t >> 1) * 16 + (ln & 15);
    const int width = N >> 1;
    if (m < M && n < width) {
        half4v h = {(_Float16)silu_mul(g[0], u[0]), (_Float16)silu_mul(g[1], u[1]), (_Float16)silu_mul(g[2], u[2]),
                    (_Float16)silu_mul(g[3], u[3])};
        *reinterpret_cast<half4v *>(o.y + (size_t)m * width + n) = h;
    }
}

// Rotary epilogue: lo / hi are the sums of elements d .. d+3 and d + D/2 .. of one head of one row (packed
// tiles 2j and 2j+1 of the head are tile j of its first and of its second half).  They are rounded to fp16
// first and then treated exactly as rope_append treats the linear's fp16 output -- same expressions, same
// results bit for bit: q heads rotated into q, k heads rotated into cache row P + m, v heads copied; a row
// whose position lies outside the tables gets its values appended and nothing else.
// What the epilogue has to fetch -- the row's position, then its table entries -- is asked for by
// prefetch_paired before the sums are formed (unconditionally, from clamped addresses), so that these two
// round trips overlap with the loads of the sums instead of following them.
struct PairedPre {
    int p;            // position of the quad's row
    float4v c, s;     // table entries of elements d .. d+3 at that position (clamped into the tables)
};

template <int MT>
__device__ __forceinline__ PairedPre prefetch_paired(const Out &o, int e4, int first_col, int M, int N)
{
    PairedPre pre = {0, {0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
    if (o.epi != kEpiRope) return pre;   // uniform
    int ln = (e4 * 4) & 63, reg = e4 >> 4;
    int i = reg & 3, tm = reg >> 2;
    int mt = tm % MT, t = tm / MT;
    int m = mt * 16 + 4 * (ln >> 4) + i;
    int pc = first_col + t * 16 + (ln & 15);
    const RopeOut &r = o.rope;
    m = m < M ? m : M - 1;
    pc = pc < N ? pc : N - 32;
    const int D = r.D, h = D >> 1;
    const int within = pc % D;
    const int d = (within >> 5) * 16 + (within & 15);
    pre.p = r.pos[m];
    const int pcl = pre.p < 0 ? 0 : (pre.p < r.n_pos ? pre.p : r.n_pos - 1);
    pre.c = *reinterpret_cast<const float4v *>(r.cos_t + (size_t)pcl * h + d);
    pre.s = *reinterpret_cast<const float4v *>(r.sin_t + (size_t)pcl * h + d);
    return pre;
}

template <int MT>
__device__ __forceinline__ void store_roped(const Out &o, float4v lo, float4v hi, const PairedPre &pre, int e4,
                                            int first_col, int M, int N)
{
    int ln = (e4 * 4) & 63, reg = e4 >> 4;
    int i = reg & 3, tm = reg >> 2;
    int mt = tm % MT, t = tm / MT;          // t is even: a first-half tile
    int m = mt * 16 + 4 * (ln >> 4) + i;
    int pc = first_col + t * 16 + (ln & 15);   // packed column of the first-half quad
    if (m >= M || pc >= N) return;
    const RopeOut &r = o.rope;
    const int D = r.D, h = D >> 1;
    const int head = pc / D, within = pc - head * D;
    const int d = (within >> 5) * 16 + (within & 15);
    const half4v l16 = {(_Float16)lo[0], (_Float16)lo[1], (_Float16)lo[2], (_Float16)lo[3]};
    const half4v h16 = {(_Float16)hi[0], (_Float16)hi[1], (_Float16)hi[2], (_Float16)hi[3]};
    if (head >= r.Hq + r.Hkv) {   // value head: appended as it is
        _Float16 *dst = r.v_cache + ((size_t)(r.P + m) * r.Hkv + (head - r.Hq - r.Hkv)) * D;
        *reinterpret_cast<half4v *>(dst + d) = l16;
        *reinterpret_cast<half4v *>(dst + d + h) = h16;
        return;
    }
    if (pre.p < 0 || pre.p >= r.n_pos) return;
    half4v olo, ohi;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float a = (float)l16[e], b = (float)h16[e];
        olo[e] = (_Float16)keep_f32(fmaf(a, pre.c[e], -b * pre.s[e]));
        ohi[e] = (_Float16)keep_f32(fmaf(b, pre.c[e], a * pre.s[e]));
    }
    _Float16 *dst = head < r.Hq ? r.q + ((size_t)m * r.Hq + head) * D
                                : r.k_cache + ((size_t)(r.P + m) * r.Hkv + (head - r.Hq)) * D;
    *reinterpret_cast<half4v *>(dst + d) = olo;
    *reinterpret_cast<half4v *>(dst + d + h) = ohi;
}

// a paired epilogue for the quad e4 of an even packed tile (a) and its partner 64 * MT quads further on (b)
template <int MT>
__device__ __forceinline__ void store_paired(const Out &o, float4v a, float4v b, const PairedPre &pre, int e4,
                                             int first_col, int M, int N)
{
    if (o.epi == kEpiRope) store_roped<MT>(o, a, b, pre, e4, first_col, M, N);   // uniform
    else store_gated<MT>(o, a, b, e4, first_col, M, N);
}

constexpr int kFlatMaxRows = 4;   // most rows the all-loads-up-front variant stages

// wavefronts per SIMD the register allocator must leave room for: one workgroup has to fit
constexpr int min_waves_per_simd(int mt, int tw, int nw, int depth)
{
    return nw / 4;
}

// Groups [begin, end) of K split ks: every split gets gq = groups / S groups and the first
// grem = groups % S one more.  Quotient and remainder come from the host: no division on the GPU.
struct KRange { int begin, end; };
__device__ __forceinline__ KRange k_range(int ks, int gq, int grem)
{
    const int begin = ks * gq + (ks < grem ? ks : grem);
    return {begin, begin + gq + (ks < grem ? 1 : 0)};
}

// Epilogue shared by the K-split kernels: the NW wavefronts' accumulators are summed through LDS
// in wave order; the sum is stored (S == 1), handed to the second kernel as a partial, or -- fused
// mode -- published with device-scope stores, after which the last workgroup of the column unit to
// take a ticket adds the S partials in split order and stores the result.
template <int MT, int TW, int NW>
__device__ __forceinline__ void finish_unit(const float4v (&acc)[TW][MT], float4v *lds4, uint32_t &ticket_sh,
                                            const Out &y, float *__restrict__ partial,
                                            uint32_t *__restrict__ tickets, int M, int N, int S, int fused, int unit,
                                            int ks, int nb, int t0, int tid, int lane, int wave)
{
    constexpr int kThreads = NW * 64;
    constexpr int R = 4 * TW * MT;
    constexpr int E4 = R * 16;
    constexpr int Q = (E4 + kThreads - 1) / kThreads;
    constexpr bool kRagged = (E4 % kThreads) != 0;
    // sum the wavefronts' accumulators through LDS in wave order
    float *lds = reinterpret_cast<float *>(lds4);
#pragma unroll
    for (int t = 0; t < TW; ++t)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                lds[(wave * R + (t * MT + mt) * 4 + i) * 64 + lane] = acc[t][mt][i];
    __syncthreads();
    const int first_col = nb * kBlockCols + t0 * 16;
    if (S == 1 && paired_epilogue(y)) {   // uniform
        for (int idx = tid; idx < E4 / 2; idx += kThreads) {
            const int e4 = gate_quad<MT>(idx);
            const PairedPre pre = prefetch_paired<MT>(y, e4, first_col, M, N);
            float4v g = lds4[e4], u = lds4[e4 + 64 * MT];
#pragma unroll
            for (int w2 = 1; w2 < NW; ++w2) {
                g += lds4[w2 * E4 + e4];
                u += lds4[w2 * E4 + e4 + 64 * MT];
            }
            store_paired<MT>(y, g, u, pre, e4, first_col, M, N);
        }
        return;
    }
    int quad[Q];   // this thread's quads (clamped where the unit has fewer: those are never stored)
    half4v res[Q];
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        quad[q] = (!kRagged || tid + kThreads * q < E4) ? tid + kThreads * q : E4 - 1;
        if (S == 1) res[q] = load_residual<MT>(y, quad[q], first_col, M, N);   // requested before the LDS sums
    }
    float4v sum[Q];
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        int e4 = tid + kThreads * q;
        float4v v = (float4v){0.f, 0.f, 0.f, 0.f};
        if (!kRagged || e4 < E4) {
            v = lds4[e4];
#pragma unroll
            for (int w2 = 1; w2 < NW; ++w2) v += lds4[w2 * E4 + e4];
        }
        sum[q] = v;
    }
    if (S == 1) {
#pragma unroll
        for (int q = 0; q < Q; ++q)
            if (!kRagged || tid + kThreads * q < E4) store_quad<MT>(y, sum[q], res[q], tid + kThreads * q, first_col, M, N);
        return;
    }
    float *mine = partial + ((size_t)unit * S + ks) * E4 * 4;
    if (!fused) {
        float4v *mine4 = reinterpret_cast<float4v *>(mine);
#pragma unroll
        for (int q = 0; q < Q; ++q)
            if ((!kRagged || tid + kThreads * q < E4) && quad_row<MT>(tid + kThreads * q) < M)
                mine4[tid + kThreads * q] = sum[q];
        return;
    }
    // the last workgroup of this column unit to arrive sums all S partials in split order
    const PartialBuffer all = partial_buffer(partial + (size_t)unit * S * E4 * 4);
#pragma unroll
    for (int q = 0; q < Q; ++q)
        if ((!kRagged || tid + kThreads * q < E4) && quad_row<MT>(tid + kThreads * q) < M)
            store_partial(all, ks * E4 + tid + kThreads * q, sum[q]);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this thread's partials have reached device scope
    __syncthreads();
    if (tid == 0) ticket_sh = __hip_atomic_fetch_add(&tickets[unit], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (ticket_sh != (uint32_t)(S - 1)) return;
    const auto load = [&](int index) { return load_partial(all, index); };
    if (paired_epilogue(y)) {   // uniform
        for (int idx = tid; idx < E4 / 2; idx += kThreads) {
            const int pair[2] = {gate_quad<MT>(idx), gate_quad<MT>(idx) + 64 * MT};
            const PairedPre pre = prefetch_paired<MT>(y, pair[0], first_col, M, N);
            float4v gu[2];
            sum_partials<2>(gu, pair, S, E4, load);
            store_paired<MT>(y, gu[0], gu[1], pre, pair[0], first_col, M, N);
        }
        if (tid == 0) __hip_atomic_store(&tickets[unit], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return;
    }
#pragma unroll
    for (int q = 0; q < Q; ++q) res[q] = load_residual<MT>(y, quad[q], first_col, M, N);
    sum_partials<Q>(sum, quad, S, E4, load);
#pragma unroll
    for (int q = 0; q < Q; ++q)
        if (!kRagged || tid + kThreads * q < E4) store_quad<MT>(y, sum[q], res[q], tid + kThreads * q, first_col, M, N);
    if (tid == 0) __hip_atomic_store(&tickets[unit], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// MT row tiles of 16, TW column tiles per wavefront, NW wavefronts per workgroup (all on the same
// columns, each on its own quantisation groups), DEPTH groups of codes in flight per wavefront.
template <int MT, int TW, int NW, int DEPTH, bool SYM>
__global__ __launch_bounds__(NW * 64, min_waves_per_simd(MT, TW, NW, DEPTH)) void gemm_kernel(
    const _Float16 *__restrict__ x, const uint8_t *__restrict__ packed, const Out y,
    float *__restrict__ partial, uint32_t *__restrict__ tickets, int M, int N, int K, int groups, int S, int fused,
    int gq, int grem)
{
    extern __shared__ float4v lds4[];
    __shared__ uint32_t ticket_sh;
    constexpr int U = DEPTH > 2 ? DEPTH : 2;             // unroll: ring position and x-fragment buffer are static
    constexpr bool kOff = kOffsetCodes && MT == 1;       // offset-code arithmetic for a single row tile
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: keeps the group loop scalar
    const int r = lane >> 4, c = lane & 15;
    const int unit = blockIdx.y, ks = blockIdx.x;                // column unit = TW tiles; grid = (S, units)
    const int nb = (unit * TW) >> 3, t0 = (unit * TW) & 7;
    const KRange kr = k_range(ks, gq, grem);
    const int g_begin = kr.begin, g_end = kr.end;

    const _Float16 *xp[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        int row = mt * 16 + c;
        row = row < M ? row : M - 1;   // rows >= M are never read; their products are never stored
        xp[mt] = x + (size_t)row * K + r * 8;
    }
    const uint8_t *rec0 = packed + record_offset(nb, 0, groups);

    float4v acc[TW][MT];
#pragma unroll
    for (int t = 0; t < TW; ++t)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[t][mt] = (float4v){0.f, 0.f, 0.f, 0.f};

    GroupOperands<MT> fa, fb;
    u32x4 w[DEPTH][TW];
    const DequantConsts magic = dequant_consts();
    // this wavefront's groups are g0, g0 + NW, ...: n_w of them
    const int g0 = g_begin + wave;
    const int n_w = g0 < g_end ? (g_end - g0 + NW - 1) / NW : 0;
    const uint8_t *recw = rec0 + (size_t)g0 * kRecordBytes;       // record of this wavefront's group 0
    constexpr size_t kStep = (size_t)NW * kRecordBytes;            // distance between its consecutive groups
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
        if (d < n_w) {
#pragma unroll
            for (int t = 0; t < TW; ++t) w[d][t] = load_tile(recw + d * kStep, t0 + t, lane);
        }
    }
    half8v bc[4];
    if (n_w > 0) {
        load_operands<MT, SYM>(fa, recw, xp, g0, c);
        if constexpr (kOff) offset_tile(bc, w[0][0], magic);
        else dequant_tile<TW, SYM>(bc, w[0][0], tile_quant<TW>(fa.q, t0), 0, magic);
    }
    int i = 0;
    // steady state: every group handled here has a successor DEPTH groups ahead, so all loads are
    // unconditional and the compiler can count exactly how many may stay in flight at each wait
    for (; i + U + DEPTH <= n_w; i += U) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int gi = i + u;
            load_operands<MT, SYM>((u & 1) ? fa : fb, recw + (size_t)(gi + 1) * kStep, xp, g0 + (gi + 1) * NW, c);
            compute_group<MT, TW, true, kOff, SYM>(((u & 1) ? fb : fa).a, ((u & 1) ? fb : fa).q, ((u & 1) ? fa : fb).q,
                                              w[u % DEPTH], w[(u + 1) % DEPTH], bc, acc,
                                              recw + (size_t)(gi + DEPTH) * kStep, true, true, t0, lane, magic, M > 1);
        }
    }
    // drain: at most U + DEPTH - 1 groups left; ring position and fragment buffer stay static
#pragma unroll
    for (int u = 0; u < U + DEPTH - 1; ++u) {
        const int gi = i + u;
        if (gi < n_w) {   // uniform
            if (gi + 1 < n_w)
                load_operands<MT, SYM>((u & 1) ? fa : fb, recw + (size_t)(gi + 1) * kStep, xp, g0 + (gi + 1) * NW, c);
            compute_group<MT, TW, false, kOff, SYM>(((u & 1) ? fb : fa).a, ((u & 1) ? fb : fa).q, ((u & 1) ? fa : fb).q,
                                               w[u % DEPTH], w[(u + 1) % DEPTH], bc, acc,
                                               recw + (size_t)(gi + DEPTH) * kStep, gi + DEPTH < n_w, gi + 1 < n_w, t0,
                                               lane, magic, M > 1);
        }
    }

    finish_unit<MT, TW, NW>(acc, lds4, ticket_sh, y, partial, tickets, M, N, S, fused, unit, ks, nb, t0, tid, lane, wave);
}

// Variant for M <= 4 and short K ranges: a wavefront owns exactly NG quantisation groups and asks
// for ALL of their codes, scales and zero-points before it computes anything, so the whole weight
// range of the workgroup is in flight at once and nothing in the arithmetic can delay a load.
// The x rows of the workgroup's K range (NW * NG groups) are fetched first -- the oldest loads, so
// waiting for them never waits for weights -- and parked in LDS, from where every wavefront reads
// its first MFMA operands (rows >= M repeat row M-1; their products are never stored).
template <int TW, int NW, int NG>
__global__ __launch_bounds__(NW * 64) void gemm_flat_kernel(
    const _Float16 *__restrict__ x, const uint8_t *__restrict__ packed, const Out y,
    float *__restrict__ partial, uint32_t *__restrict__ tickets, int M, int N, int K, int groups, int S, int fused)
{
    extern __shared__ float4v lds4[];
    __shared__ uint32_t ticket_sh;
    constexpr int kThreads = NW * 64;
    constexpr int kRow16 = NW * NG * 16;          // 16-byte words of x per staged row
    constexpr int kRowStride16 = kRow16 + 1;      // LDS row stride (one word of padding)
    constexpr int XL = (kFlatMaxRows * kRow16 + kThreads - 1) / kThreads;   // x words per thread
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane >> 4, c = lane & 15;
    const int unit = blockIdx.y, ks = blockIdx.x;   // grid = (S, units); groups == S * NW * NG
    const int nb = (unit * TW) >> 3, t0 = (unit * TW) & 7;
    const int g_begin = ks * (NW * NG);

    // 1. x rows of this K range
    u32x4 xr[XL];
    u32x4 *xs = reinterpret_cast<u32x4 *>(lds4);
#pragma unroll
    for (int l = 0; l < XL; ++l) {
        const int u = tid + kThreads * l, row = u / kRow16, col = u % kRow16;
        if (row < M) xr[l] = *reinterpret_cast<const u32x4 *>(x + (size_t)row * K + (size_t)g_begin * kGroup + col * 8);
    }
    // 2. every weight byte of this wavefront: groups g_begin + wave + NW * i
    const uint8_t *recw = packed + record_offset(nb, g_begin + wave, groups);
    u32x4 w[NG][TW];
    QuantWords qw[NG];
#pragma unroll
    for (int i = 0; i < NG; ++i) {
        const uint8_t *rec = recw + (size_t)i * (NW * kRecordBytes);
        qw[i].s = *reinterpret_cast<const u32x4 *>(rec + kScalesOff + c * 16);
        qw[i].z = *reinterpret_cast<const uint32_t *>(rec + kZerosOff + c * 4);
#pragma unroll
        for (int t = 0; t < TW; ++t) w[i][t] = load_tile(rec, t0 + t, lane);
    }
    __builtin_amdgcn_sched_barrier(0);
    // 3. park x
#pragma unroll
    for (int l = 0; l < XL; ++l) {
        const int u = tid + kThreads * l, row = u / kRow16, col = u % kRow16;
        if (row < M) {
            xs[row * kRowStride16 + col] = xr[l];
        }
    }
    __syncthreads();

    float4v acc[TW][1];
#pragma unroll
    for (int t = 0; t < TW; ++t) acc[t][0] = (float4v){0.f, 0.f, 0.f, 0.f};
    const DequantConsts magic = dequant_consts();
    const u32x4 *xrow = xs + (c < M ? c : M - 1) * kRowStride16 + r;
#pragma unroll
    for (int i = 0; i < NG; ++i) {
        u32x4 a[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) a[j] = xrow[(wave + NW * i) * 16 + j * 4];
        const TileQuant<TW> q = tile_quant<TW>(qw[i], t0);
        float4v negc[1], xsum[1];
        if constexpr (kOffsetCodes) {
            const u32x4 (&a1)[1][4] = reinterpret_cast<const u32x4 (&)[1][4]>(a);
            group_sums<1>(a1, negc, xsum);
        }
#pragma unroll
        for (int t = 0; t < TW; ++t) {
            half8v b[4];
            if constexpr (kOffsetCodes) offset_tile(b, w[i][t], magic);
            else dequant_tile<TW>(b, w[i][t], q, t, magic);
            float4v part = kOffsetCodes ? negc[0] : (float4v){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j = 0; j < 4; ++j)
                part = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8v, a[j]), b[j], part, 0, 0, 0);
            uint32_t s2 = q.sw[t >> 1];
            _Float16 sh = __builtin_bit_cast(_Float16, (uint16_t)((t & 1) ? (s2 >> 16) : (s2 & 0xFFFFu)));
            if constexpr (kOffsetCodes)
                fold_offset(acc[t][0], part, xsum[0], (float)sh, (float)((q.zbits >> (4 * t)) & 0xFu), M > 1);
            else
                acc[t][0] += (float)sh * part;
        }
    }
    __syncthreads();   // the x rows are dead: the epilogue reuses their LDS
    finish_unit<1, TW, NW>(acc, lds4, ticket_sh, y, partial, tickets, M, N, S, fused, unit, ks, nb, t0, tid, lane, wave);
}

// Variant for larger M, where re-reading x dominates the on-chip traffic: the four wavefronts of a
// workgroup walk the SAME quantisation groups, each on its own TW column tiles (a column unit of
// 4*TW tiles per workgroup), and the group's x fragments are fetched from L2 once per workgroup
// -- each wavefront fetches the k step equal to its index for all row tiles -- and parked in LDS
// in operand order, double-buffered, so one barrier per group suffices and every wavefront reads
// its first MFMA operands with conflict-free 16-byte LDS loads.  Each wavefront owns its output
// columns outright (no cross-wavefront sum); K may still be split across workgroups, in which
// case the fp32 partials go to the workspace and splitk_reduce_kernel finishes the job.
template <int MT, int TW, int DEPTH>
__global__ __launch_bounds__(256, ((MT == 1 || (MT * TW <= 12 && !(MT == 3 && TW == 4 && DEPTH == 2))) ? 2 : 1)) void gemm_ns_kernel(
    const _Float16 *__restrict__ x, const uint8_t *__restrict__ packed, const Out y,
    float *__restrict__ partial, int M, int N, int K, int groups, int S, int gq, int grem)
{
    extern __shared__ float4v lds4[];
    constexpr int R = 4 * TW * MT;            // accumulator registers per lane
    constexpr int E4 = R * 16;                // float4 results per wavefront
    constexpr int U = DEPTH > 2 ? DEPTH : 2;  // unroll: ring position, x buffer and scale buffer are static
    constexpr int kFragQuads = MT * 4 * 64;   // 16-byte fragments of one group's x tile
    u32x4 *xa = reinterpret_cast<u32x4 *>(lds4);                  // [2][MT*4][64]
    float4v *out4 = lds4;                                         // [4 wavefronts][E4], reuses the x tiles after the loop
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane >> 4, c = lane & 15;
    const int wg_unit = blockIdx.y, ks = blockIdx.x;   // grid = (S, workgroup units)
    const int unit = wg_unit * 4 + wave;                          // this wavefront's column unit
    const int tiles_total = pad_cols(N) / 16;
    const bool active = unit * TW < tiles_total;                  // a ragged last workgroup has idle wavefronts
    const int tile_first = active ? unit * TW : 0;
    const int nb = tile_first >> 3, t0 = tile_first & 7;
    const KRange kr = k_range(ks, gq, grem);
    const int g_begin = kr.begin, g_end = kr.end;
    const int n = g_end - g_begin;

    // what this lane fetches of a group's x tile: MT of its MT * 4 blocks of eight rows x two k steps, whole cache
    // lines, swizzled in LDS (the layout cs_segment describes)
    const _Float16 *xs[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) {
        const int blk = wave * MT + i;
        const int mt = blk >> 2, jp = (blk >> 1) & 1, h = blk & 1, row8 = lane >> 3;
        const int chunk = (lane & 7) ^ (4 * h + (row8 >> 1));
        int row = mt * 16 + h * 8 + row8;
        row = row < M ? row : M - 1;   // rows >= M are never read; their products are never stored
        xs[i] = x + (size_t)row * K + jp * 64 + chunk * 8;
    }
    uint32_t xfrag[2];   // this lane's byte offset in a block pair for even and odd k steps
    {
        const int h = c >> 3, row8 = c & 7, sw = 4 * h + (row8 >> 1);
        xfrag[0] = (uint32_t)(h * 1024 + (row8 * 8 + (r ^ sw)) * 16);
        xfrag[1] = (uint32_t)(h * 1024 + (row8 * 8 + ((4 + r) ^ sw)) * 16);
    }
    const uint8_t *recw = packed + record_offset(nb, g_begin, groups);   // record of group 0 of the range

    float4v acc[TW][MT];
#pragma unroll
    for (int t = 0; t < TW; ++t)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[t][mt] = (float4v){0.f, 0.f, 0.f, 0.f};

    u32x4 w[DEPTH][TW];
    QuantWords qa, qb;
    u32x4 xreg[MT];
    u32x4 a[MT][4];
    const DequantConsts magic = dequant_consts();
    auto load_quant = [&](QuantWords &q, int gi) {
        const uint8_t *rec = recw + (size_t)gi * kRecordBytes;
        q.s = *reinterpret_cast<const u32x4 *>(rec + kScalesOff + c * 16);
        q.z = *reinterpret_cast<const uint32_t *>(rec + kZerosOff + c * 4);
    };
    auto load_x = [&](int gi) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
            xreg[mt] = *reinterpret_cast<const u32x4 *>(xs[mt] + (size_t)(g_begin + gi) * kGroup);
    };
    auto park_x = [&](int buf) {
#pragma unroll
        for (int i = 0; i < MT; ++i) xa[buf * kFragQuads + (wave * MT + i) * 64 + lane] = xreg[i];
    };
    auto fetch_a = [&](int buf) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                a[mt][j] = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const uint8_t *>(xa + buf * kFragQuads) +
                                                           (mt * 2 + (j >> 1)) * 2048 + xfrag[j & 1]);
    };

    half8v bc[4];
    if (n > 0) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d)
            if (d < n)
#pragma unroll
                for (int t = 0; t < TW; ++t) w[d][t] = load_tile(recw + (size_t)d * kRecordBytes, t0 + t, lane);
        load_x(0);
        load_quant(qa, 0);
        park_x(0);
        dequant_tile<TW>(bc, w[0][0], tile_quant<TW>(qa, t0), 0, magic);
    }
    int i = 0;
    // steady state: every group here has successors, all loads are unconditional
    for (; i + U + DEPTH <= n; i += U) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int gi = i + u;
            __syncthreads();   // x tile (u & 1) is parked; nobody still reads the other one
            load_x(gi + 1);
            load_quant((u & 1) ? qa : qb, gi + 1);
            fetch_a(u & 1);
            __builtin_amdgcn_sched_barrier(0);
            compute_group<MT, TW, true>(a, (u & 1) ? qb : qa, (u & 1) ? qa : qb, w[u % DEPTH], w[(u + 1) % DEPTH], bc, acc,
                                        recw + (size_t)(gi + DEPTH) * kRecordBytes, true, true, t0, lane, magic);
            park_x((u & 1) ^ 1);
        }
    }
    // drain
#pragma unroll
    for (int u = 0; u < U + DEPTH - 1; ++u) {
        const int gi = i + u;
        if (gi < n) {   // uniform over the workgroup
            __syncthreads();
            const bool more = gi + 1 < n;
            if (more) {
                load_x(gi + 1);
                load_quant((u & 1) ? qa : qb, gi + 1);
            }
            fetch_a(u & 1);
            compute_group<MT, TW, false>(a, (u & 1) ? qb : qa, (u & 1) ? qa : qb, w[u % DEPTH], w[(u + 1) % DEPTH], bc, acc,
                                         recw + (size_t)(gi + DEPTH) * kRecordBytes, gi + DEPTH < n, more, t0, lane, magic);
            if (more) park_x((u & 1) ^ 1);
        }
    }

    // each wavefront turns its accumulators into row-contiguous quads through its own LDS region
    __syncthreads();   // the x tiles are dead: every wavefront has left the group loop
    float *mine_lds = reinterpret_cast<float *>(out4 + wave * E4);
#pragma unroll
    for (int t = 0; t < TW; ++t)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int k4 = 0; k4 < 4; ++k4) mine_lds[((t * MT + mt) * 4 + k4) * 64 + lane] = acc[t][mt][k4];
    if (!active) return;
    const int first_col = nb * kBlockCols + t0 * 16;
    if (S == 1 && paired_epilogue(y)) {   // uniform
        for (int idx = lane; idx < E4 / 2; idx += 64) {
            const int e4 = gate_quad<MT>(idx);
            const PairedPre pre = prefetch_paired<MT>(y, e4, first_col, M, N);
            store_paired<MT>(y, out4[wave * E4 + e4], out4[wave * E4 + e4 + 64 * MT], pre, e4, first_col, M, N);
        }
        return;
    }
    float4v *part4 = reinterpret_cast<float4v *>(partial) + ((size_t)unit * S + ks) * E4;
    if (S == 1) {   // uniform: all residuals requested first, then the stores
        half4v res[E4 / 64];
#pragma unroll
        for (int q = 0; q < E4 / 64; ++q) res[q] = load_residual<MT>(y, lane + 64 * q, first_col, M, N);
#pragma unroll
        for (int q = 0; q < E4 / 64; ++q) store_quad<MT>(y, out4[wave * E4 + lane + 64 * q], res[q], lane + 64 * q, first_col, M, N);
        return;
    }
#pragma unroll
    for (int q = 0; q < E4 / 64; ++q) {
        const int e4 = lane + 64 * q;
        if (quad_row<MT>(e4) < M) part4[e4] = out4[wave * E4 + e4];
    }
}

// One quantisation group for this wavefront's TW column tiles, tile after tile with no software
// pipelining: few live registers, so that several wavefronts share a SIMD and the hardware overlaps
// one wavefront's code expansion (vector ALU) with another's matrix instructions.  The code
// registers of a tile are refilled, REFILL permitting, as soon as the tile is expanded.
template <int MT, int TW, bool ALWAYS_REFILL, bool SYM>
__device__ __forceinline__ void compute_group_lean(const u32x4 (&a)[MT][4], QuantWords &f, u32x4 (&w)[TW],
                                                   float4v (&acc)[TW][MT], const uint8_t *refill_rec, bool refill,
                                                   int t0, int c, int lane, const DequantConsts &magic)
{
    const TileQuant<TW> q = tile_quant<TW>(f, t0);
    const global_bytes rec = uniform_ptr(refill_rec);
    const uint32_t tile_off = (uint32_t)(t0 * 1024 + lane * 16);
    if (ALWAYS_REFILL || refill) {
        f.s = load_global<u32x4>(rec + (uint32_t)(kScalesOff + c * 16));
        if constexpr (!SYM) f.z = load_global<uint32_t>(rec + (uint32_t)(kZerosOff + c * 4));
    }
#pragma unroll
    for (int t = 0; t < TW; ++t) {
        const uint32_t z = (q.zbits >> (4 * t)) & 0xFu;
        const uint32_t zz = z | (z << 16);
        const half2v zneg = as_h2(SYM ? kSymZneg : (zz | 0xE400E400u));              // -(1024 + z)
        const half2v zneg16 = as_h2(SYM ? kSymZneg16 : ((zz << 4) | 0xD400D400u));   // -(64 + z)
        float4v part[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) part[mt] = (float4v){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const half8v b = dequant8(w[t][j], zneg, zneg16, magic);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                part[mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8v, a[mt][j]), b, part[mt], 0, 0, 0);
        }
        if (ALWAYS_REFILL || refill)
            w[t] = __builtin_nontemporal_load((const __attribute__((address_space(1))) u32x4 *)(rec + (tile_off + (uint32_t)(t * 1024))));
        uint32_t s2 = q.sw[t >> 1];
        _Float16 sh = __builtin_bit_cast(_Float16, (uint16_t)((t & 1) ? (s2 >> 16) : (s2 & 0xFFFFu)));
        float s = (float)sh;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[t][mt] += s * part[mt];
        // tiles stay apart: expanding several ahead of the matrix pipe would cost the registers
        // that the co-resident wavefronts need, and they are what hides this tile's latency
        __builtin_amdgcn_sched_barrier(0);
    }
}

// High-occupancy variant for M > 16.  A workgroup of 4*KS wavefronts owns a column unit of 4*TW
// tiles; wavefront (kset, colq) = (index / 4, index % 4) works on the TW tiles of column quarter
// colq and on every KS-th quantisation group starting at kset, so KS wavefronts share each SIMD.
// Per step the workgroup parks the x fragments of KS consecutive groups in LDS (operand order,
// double-buffered, one barrier per step); the KS partial sums of a column meet in LDS at the end.
// One (column unit, group range) segment of the kernel below: groups g_begin .. g_end-1 of workgroup
// unit wg_unit.  nslots == 1: the segment is the unit's whole K and its sums are stored.  Otherwise it
// is contributor `slot` of `nslots` (ascending group ranges) and its sums go to the workspace, slot
// stride `sstride` per wavefront unit; in last-arriver mode (fused) the contributor that takes the
// last ticket adds all of them in slot order and stores.  Every wavefront of the workgroup passes the
// same barriers whatever it returns through.
template <int MT, int TW, int KS, int DEPTH, bool SYM>
__device__ __forceinline__ void cs_segment(const _Float16 *__restrict__ x, const uint8_t *__restrict__ packed,
                                           const Out &y, float *__restrict__ partial, uint32_t *__restrict__ tickets,
                                           float4v *lds4, uint32_t &ticket_sh, int M, int N, int K, int groups,
                                           int wg_unit, int g_begin, int g_end, int nslots, int slot, int sstride,
                                           int fused)
{
    constexpr int R = 4 * TW * MT;                 // accumulator registers per lane
    constexpr int E4 = R * 16;                     // float4 results per wavefront
    constexpr int kBufQuads = KS * MT * 4 * 64;    // 16-byte fragments of one step's x tiles
    u32x4 *xa = reinterpret_cast<u32x4 *>(lds4);   // [2][KS][MT*4][64]
    float4v *out4 = lds4;                          // [4*KS wavefronts][E4], reuses the x tiles after the loop
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int colq = wave & 3, kset = wave >> 2;
    const int r = lane >> 4, c = lane & 15;
    const int unit = wg_unit * 4 + colq;
    const int tiles_total = pad_cols(N) / 16;
    const bool active = unit * TW < tiles_total;   // a ragged last workgroup has idle column quarters
    const int tile_first = active ? unit * TW : 0;
    const int nb = tile_first >> 3, t0 = tile_first & 7;
    const int S = nslots, ks = slot;
    const int n = g_end - g_begin;
    const int steps = (n + KS - 1) / KS;           // workgroup-uniform
    const int full = n / KS;                       // steps in which every k set has a group
    const int mine = n > kset ? (n - kset + KS - 1) / KS : 0;   // groups of this wavefront: g_begin + kset + KS*i

    // The x tile of a group is kept in LDS as MT * 4 blocks of 1 KB, block (mt, jp, h) = the eight rows
    // 16 mt + 8 h .. + 7 times the 128 bytes of k steps 2 jp and 2 jp + 1, and a wavefront fetches MT of them for
    // its k set, lane l row l / 8: such a load touches whole cache lines (fetching matrix-operand fragments
    // directly -- sixteen rows times 64 bytes per load -- occupies the load path four times as long).  Inside a
    // block the eight 16-byte chunks of a row sit at chunk ^ (4 h + row / 2), which spreads the sixteen rows of
    // a fragment read over all LDS banks.  (Byte offsets from a wavefront-uniform base, so the loads address
    // with a scalar base and a 32-bit lane offset.)
    uint32_t xoff[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) {
        const int blk = colq * MT + i;
        const int mt = blk >> 2, jp = (blk >> 1) & 1, h = blk & 1, row8 = lane >> 3;
        const int chunk = (lane & 7) ^ (4 * h + (row8 >> 1));
        int row = mt * 16 + h * 8 + row8;
        row = row < M ? row : M - 1;   // rows >= M are never read; their products are never stored
        xoff[i] = (uint32_t)(((size_t)row * K + jp * 64 + chunk * 8) * sizeof(_Float16));
    }
    // fragment (mt, j) for lane (r, c) -- row 16 mt + c, elements 32 j + 8 r .. + 7 -- lies in block pair
    // (mt, j / 2) at this lane's offset for even or odd k steps
    uint32_t xfrag[2];
    {
        const int h = c >> 3, row8 = c & 7, sw = 4 * h + (row8 >> 1);
        xfrag[0] = (uint32_t)(h * 1024 + (row8 * 8 + (r ^ sw)) * 16);
        xfrag[1] = (uint32_t)(h * 1024 + (row8 * 8 + ((4 + r) ^ sw)) * 16);
    }
    const uint8_t *xbase = reinterpret_cast<const uint8_t *>(x + (size_t)(g_begin + kset) * kGroup);
    const uint8_t *recw = packed + record_offset(nb, g_begin + (kset < n ? kset : 0), groups);   // group 0 of this wavefront

    float4v acc[TW][MT];
#pragma unroll
    for (int t = 0; t < TW; ++t)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[t][mt] = (float4v){0.f, 0.f, 0.f, 0.f};

    u32x4 w[DEPTH][TW];
    QuantWords qw[DEPTH];
    u32x4 xreg[MT];
    u32x4 a[MT][4];
    const DequantConsts magic = dequant_consts();
    auto load_x = [&](int i) {
        const global_bytes xb = uniform_ptr(xbase + (size_t)i * (KS * kGroup * sizeof(_Float16)));
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) xreg[mt] = load_global<u32x4>(xb + xoff[mt]);
    };
    auto park_x = [&](int buf) {
#pragma unroll
        for (int i = 0; i < MT; ++i) xa[buf * kBufQuads + (kset * MT * 4 + colq * MT + i) * 64 + lane] = xreg[i];
    };
    auto fetch_a = [&](int buf) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                a[mt][j] = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const uint8_t *>(xa + buf * kBufQuads + kset * MT * 4 * 64) +
                                                           (mt * 2 + (j >> 1)) * 2048 + xfrag[j & 1]);
    };
    auto rec_of = [&](int i) { return recw + (size_t)i * (KS * kRecordBytes); };

#pragma unroll
    for (int d = 0; d < DEPTH; ++d)
        if (d < mine) {
            const uint8_t *rec = rec_of(d);
            qw[d].s = *reinterpret_cast<const u32x4 *>(rec + kScalesOff + c * 16);
            if constexpr (SYM) qw[d].z = kSymZeros;
            else qw[d].z = *reinterpret_cast<const uint32_t *>(rec + kZerosOff + c * 4);
#pragma unroll
            for (int t = 0; t < TW; ++t) w[d][t] = load_tile(rec, t0 + t, lane);
        }
    if (mine > 0) {
        load_x(0);
        park_x(0);
    }
    int i = 0;
    // steady state: every wavefront has a group in this step and DEPTH steps further on
    for (; i + 2 * DEPTH <= full; i += DEPTH) {
#pragma unroll
        for (int u = 0; u < DEPTH; ++u) {
            const int gi = i + u;
            __syncthreads();   // x tiles of step gi are parked; nobody still reads the other buffer
            load_x(gi + 1);
            fetch_a(gi & 1);
            __builtin_amdgcn_sched_barrier(0);
            compute_group_lean<MT, TW, true, SYM>(a, qw[u], w[u], acc, rec_of(gi + DEPTH), true, t0, c, lane, magic);
            park_x((gi & 1) ^ 1);
        }
    }
    // drain
#pragma unroll
    for (int u = 0; u < 2 * DEPTH; ++u) {
        const int gi = i + u;
        if (gi < steps) {   // uniform over the workgroup
            __syncthreads();
            const bool more = gi + 1 < mine;
            if (more) load_x(gi + 1);
            if (gi < mine) {
                fetch_a(gi & 1);
                compute_group_lean<MT, TW, false, SYM>(a, qw[u % DEPTH], w[u % DEPTH], acc, rec_of(gi + DEPTH),
                                                  gi + DEPTH < mine, t0, c, lane, magic);
            }
            if (more) park_x((gi & 1) ^ 1);
        }
    }

    // every wavefront parks its accumulators in fragment order; the KS partial sums of a column
    // quarter are then added and leave as row-contiguous quads
    __syncthreads();   // the x tiles are dead: every wavefront has left the group loop
    float *mine_lds = reinterpret_cast<float *>(out4 + wave * E4);
#pragma unroll
    for (int t = 0; t < TW; ++t)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int k4 = 0; k4 < 4; ++k4) mine_lds[((t * MT + mt) * 4 + k4) * 64 + lane] = acc[t][mt][k4];
    __syncthreads();
    const int first_col = nb * kBlockCols + t0 * 16;
    if (S == 1) {
        if (!active) return;
        if (paired_epilogue(y)) {   // uniform
            for (int idx = kset * 64 + lane; idx < E4 / 2; idx += 64 * KS) {
                const int e4 = gate_quad<MT>(idx);
                const PairedPre pre = prefetch_paired<MT>(y, e4, first_col, M, N);
                float4v g = out4[colq * E4 + e4], u = out4[colq * E4 + e4 + 64 * MT];
#pragma unroll
                for (int s = 1; s < KS; ++s) {
                    g += out4[(s * 4 + colq) * E4 + e4];
                    u += out4[(s * 4 + colq) * E4 + e4 + 64 * MT];
                }
                store_paired<MT>(y, g, u, pre, e4, first_col, M, N);
            }
            return;
        }
        constexpr int kMine = (E4 / 64 + KS - 1) / KS;   // quads of this lane: lane + 64 (kset + KS j)
        half4v res[kMine];
#pragma unroll
        for (int j = 0; j < kMine; ++j) {
            const int q = kset + KS * j;
            res[j] = load_residual<MT>(y, lane + 64 * (q < E4 / 64 ? q : E4 / 64 - 1), first_col, M, N);
        }
#pragma unroll
        for (int j = 0; j < kMine; ++j) {
            const int q = kset + KS * j;
            if (q >= E4 / 64) break;   // uniform
            const int e4 = lane + 64 * q;
            float4v v = out4[colq * E4 + e4];
#pragma unroll
            for (int s = 1; s < KS; ++s) v += out4[(s * 4 + colq) * E4 + e4];
            store_quad<MT>(y, v, res[j], e4, first_col, M, N);
        }
        return;
    }
    // K split across workgroups: this workgroup's sums go to the workspace.  Two-kernel mode ends
    // here; otherwise they are published at device scope and the last workgroup of the column unit
    // to take a ticket adds the S partials in split order and stores the result.
    float *mine_part = partial + ((size_t)unit * sstride + ks) * E4 * 4;
    const PartialBuffer all = partial_buffer(partial + (size_t)unit * sstride * E4 * 4);
    if (active) {
        for (int q = kset; q < E4 / 64; q += KS) {
            const int e4 = lane + 64 * q;
            if (quad_row<MT>(e4) >= M) continue;
            float4v v = out4[colq * E4 + e4];
#pragma unroll
            for (int s = 1; s < KS; ++s) v += out4[(s * 4 + colq) * E4 + e4];
            if (fused) store_partial(all, ks * E4 + e4, v);
            else reinterpret_cast<float4v *>(mine_part)[e4] = v;
        }
    }
    if (!fused) return;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this thread's partials have reached device scope
    __syncthreads();
    if (tid == 0) ticket_sh = __hip_atomic_fetch_add(&tickets[wg_unit], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (ticket_sh != (uint32_t)(S - 1)) return;
    if (tid == 0) __hip_atomic_store(&tickets[wg_unit], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (!active) return;
    const auto load = [&](int index) { return load_partial(all, index); };
    if (paired_epilogue(y)) {   // uniform
        for (int idx = kset * 64 + lane; idx < E4 / 2; idx += 64 * KS) {
            const int pair[2] = {gate_quad<MT>(idx), gate_quad<MT>(idx) + 64 * MT};
            const PairedPre pre = prefetch_paired<MT>(y, pair[0], first_col, M, N);
            float4v gu[2];
            sum_partials<2>(gu, pair, S, E4, load);
            store_paired<MT>(y, gu[0], gu[1], pre, pair[0], first_col, M, N);
        }
        return;
    }
    // two quads of the lane at a time: their residuals and a batch of their partials are in flight together
    for (int q = kset; q < E4 / 64; q += 2 * KS) {
        const int q1 = q + KS < E4 / 64 ? q + KS : q;   // uniform; the last round may have one quad only
        const int pair[2] = {lane + 64 * q, lane + 64 * q1};
        const half4v r0 = load_residual<MT>(y, pair[0], first_col, M, N), r1 = load_residual<MT>(y, pair[1], first_col, M, N);
        float4v v[2];
        sum_partials<2>(v, pair, S, E4, load);
        store_quad<MT>(y, v[0], r0, pair[0], first_col, M, N);
        if (q1 != q) store_quad<MT>(y, v[1], r1, pair[1], first_col, M, N);
    }
}

// Two ways to share the work.  Classic (per == 0): grid = (S, workgroup units), workgroup (ks, u) takes
// K split ks of unit u.  Even split (per > 0): the (unit, group) pairs, unit-major, are dealt out in
// runs of `per` to a 1-D grid, so every workgroup gets the same number of groups even when the units
// alone do not fill the chip; a run that crosses a unit boundary is handled as two segments, and a
// unit shared by several runs is summed by its last arriver.
template <int MT, int TW, int KS, int DEPTH, bool SYM>
__global__ __launch_bounds__(256 * KS) void gemm_cs_kernel(
    const _Float16 *__restrict__ x, const uint8_t *__restrict__ packed, const Out y,
    float *__restrict__ partial, uint32_t *__restrict__ tickets, int M, int N, int K, int groups, int S, int fused,
    int gq, int grem, int per, int wg_units)
{
    extern __shared__ float4v lds4[];
    __shared__ uint32_t ticket_sh;
    if (per == 0) {
        const KRange kr = k_range(blockIdx.x, gq, grem);
        cs_segment<MT, TW, KS, DEPTH, SYM>(x, packed, y, partial, tickets, lds4, ticket_sh, M, N, K, groups, blockIdx.y,
                                      kr.begin, kr.end, S, blockIdx.x, S, fused);
        return;
    }
    const int total = wg_units * groups;
    int item = blockIdx.x * per;
    const int end = min(item + per, total);
    bool again = false;
    while (item < end) {   // uniform over the workgroup
        const int u = item / groups, g0 = item - u * groups;
        const int g1 = min(groups, g0 + (end - item));
        const int first = (u * groups) / per, last = ((u + 1) * groups - 1) / per;   // runs that touch unit u
        if (again) __syncthreads();   // the previous segment's epilogue has left LDS
        cs_segment<MT, TW, KS, DEPTH, SYM>(x, packed, y, partial, tickets, lds4, ticket_sh, M, N, K, groups, u, g0, g1,
                                      last - first + 1, (int)blockIdx.x - first, S, 1);
        item += g1 - g0;
        again = true;
    }
}

// second pass of the two-kernel split-K mode: one workgroup per column unit
constexpr int kReduceThreads = 256;
template <int MT, int TW>
__global__ __launch_bounds__(kReduceThreads) void splitk_reduce_kernel(const float *__restrict__ partial,
                                                                       const Out y, int M, int N, int S)
{
    constexpr int E4 = 4 * TW * MT * 16;
    constexpr int Q = (E4 + kReduceThreads - 1) / kReduceThreads;
    constexpr bool kRagged = (E4 % kReduceThreads) != 0;
    const int unit = blockIdx.x, tid = threadIdx.x;
    const int nb = (unit * TW) >> 3, t0 = (unit * TW) & 7;
    const float4v *all = reinterpret_cast<const float4v *>(partial) + (size_t)unit * S * E4;
    const auto load = [&](int index) { return all[index]; };
    const int first_col = nb * kBlockCols + t0 * 16;
    if (paired_epilogue(y)) {   // uniform
        for (int idx = tid; idx < E4 / 2; idx += kReduceThreads) {
            const int pair[2] = {gate_quad<MT>(idx), gate_quad<MT>(idx) + 64 * MT};
            const PairedPre pre = prefetch_paired<MT>(y, pair[0], first_col, M, N);
            float4v gu[2];
            sum_partials<2>(gu, pair, S, E4, load);
            store_paired<MT>(y, gu[0], gu[1], pre, pair[0], first_col, M, N);
        }
        return;
    }
    int quad[Q];
    half4v res[Q];
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        quad[q] = (!kRagged || tid + kReduceThreads * q < E4) ? tid + kReduceThreads * q : E4 - 1;
        res[q] = load_residual<MT>(y, quad[q], first_col, M, N);
    }
    float4v sum[Q];
    sum_partials<Q>(sum, quad, S, E4, load);
#pragma unroll
    for (int q = 0; q < Q; ++q)
        if (!kRagged || tid + kReduceThreads * q < E4) store_quad<MT>(y, sum[q], res[q], tid + kReduceThreads * q, first_col, M, N);
}

// ---- host side ---------------------------------------------------------------------------------

struct Plan {
    int tw;      // column tiles per wavefront (2, 4 or 8); 0 = no compiled variant matches the knobs
    int nw;      // wavefronts per workgroup: 4, 8 or 16 that split K for the same columns, or 1 for the
                 // variant whose four wavefronts split the columns and share x fragments through LDS
    int depth;   // groups of codes in flight per wavefront (1, 2 or 4)
    int S;       // workgroups splitting K for one column unit
    int fused;   // S > 1: 1 = last workgroup of a unit sums the partials, 0 = a second kernel does
    int ks;      // 0, or the number of interleaved K sets of the high-occupancy column-split variant
                 // (4*ks wavefronts per workgroup; nw is then 0)
    int ng;      // 0, or the groups per wavefront of the all-loads-up-front variant (M <= 4 only;
                 // K / 128 == S * nw * ng exactly)
};

// measured rows are keyed by a row bucket: 0 for M <= 8 (plain decoding and sequence verification), else
// the number of 16-row tiles (1 = M 9..16, 2 = 17..32, ...)
static int row_bucket(int M) { return M <= 8 ? 0 : (M + 15) / 16; }
struct TunedRow { int N, K, mt, tw, nw, depth, S, fused, ks; };
static const TunedRow kTuned[] = {
#include "tuned_plans.inc"
};
struct TunedFlatRow { int N, K, m_max, tw, nw, ng, S, fused; };   // consulted first when M <= m_max
static const TunedFlatRow kTunedFlat[] = {
    {0, 0, 0, 0, 0, 0, 0, 0},
#include "tuned_flat.inc"
};

// all-loads-up-front variant: F(TW, NW, NG)
#define W4_FLAT_VARIANTS(F)                                                                         \
    F(2, 8, 8) F(2, 16, 4) F(2, 4, 8) F(2, 8, 4) F(2, 4, 4) F(2, 8, 7) F(2, 4, 7)                                 \
    F(4, 8, 8) F(4, 16, 4) F(4, 4, 8) F(4, 8, 4) F(4, 4, 4) F(4, 8, 7) F(4, 4, 7)                                 \
    F(8, 8, 4) F(8, 4, 4)

static bool flat_variant_exists(int tw, int nw, int ng)
{
#define F(TW_, NW_, NG_) if (tw == TW_ && nw == NW_ && ng == NG_) return true;
    W4_FLAT_VARIANTS(F)
#undef F
    return false;
}

// the kernel variants that are compiled: X(MT, TW, NW, DEPTH)
#define W4_VARIANTS_SMALL(X, MT)                                                                    \
    X(MT, 2, 4, 1) X(MT, 2, 4, 2) X(MT, 2, 4, 4) X(MT, 4, 4, 1) X(MT, 4, 4, 2) X(MT, 8, 4, 1) X(MT, 8, 4, 2)
#define W4_VARIANTS(X)                                                                              \
    W4_VARIANTS_SMALL(X, 1) W4_VARIANTS_SMALL(X, 2) W4_VARIANTS_SMALL(X, 3) W4_VARIANTS_SMALL(X, 4) \
    X(1, 2, 8, 1) X(1, 2, 8, 2) X(1, 2, 8, 4) X(1, 4, 4, 4) X(1, 4, 8, 1) X(1, 4, 8, 2)                         \
    X(1, 8, 8, 1) X(1, 8, 8, 2) X(2, 2, 8, 1) X(2, 2, 8, 2) X(2, 4, 8, 1)

// column-split variant (nw == 0): Y(MT, TW, DEPTH)
#define W4_NS_VARIANTS(Y)                                                                           \
    Y(2, 4, 1) Y(2, 4, 2) Y(2, 8, 1) Y(3, 4, 1) Y(3, 4, 2) Y(3, 8, 1) Y(4, 4, 1) Y(4, 4, 2) Y(4, 8, 1) Y(1, 8, 1) Y(1, 8, 2)

// high-occupancy column-split variant: Z(MT, TW, KS, DEPTH)
#define W4_CS_VARIANTS(Z)                                                                           \
    Z(2, 2, 1, 2) Z(2, 2, 2, 2) Z(2, 4, 1, 2) Z(2, 4, 2, 2) Z(2, 8, 1, 2)                                     \
    Z(3, 2, 1, 2) Z(3, 2, 2, 2) Z(3, 4, 1, 2)                                                         \
    Z(4, 2, 1, 2) Z(4, 2, 2, 2) Z(4, 4, 1, 2)                                                         \
    Z(4, 8, 1, 1) Z(3, 8, 1, 2) Z(3, 8, 1, 1) Z(4, 4, 1, 1) Z(3, 4, 2, 1) Z(2, 4, 2, 1) Z(2, 8, 2, 1) Z(2, 4, 3, 1) Z(4, 4, 2, 1) Z(3, 4, 1, 1) \
    Z(2, 2, 3, 2) Z(3, 2, 3, 1) Z(2, 2, 3, 1) Z(4, 2, 2, 1) Z(3, 2, 2, 1) Z(2, 2, 2, 1)

static bool variant_exists(int mt, int tw, int nw, int depth, int ks = 0)
{
#define Z(MT_, TW_, KS_, D_) if (ks == KS_ && mt == MT_ && tw == TW_ && depth == D_) return true;
    if (ks > 0) {
        W4_CS_VARIANTS(Z)
        return false;
    }
#undef Z
#define Y(MT_, TW_, D_) if (nw == 1 && mt == MT_ && tw == TW_ && depth == D_) return true;
    W4_NS_VARIANTS(Y)
#undef Y
#define X(MT_, TW_, NW_, D_) if (mt == MT_ && tw == TW_ && nw == NW_ && depth == D_) return true;
    W4_VARIANTS(X)
#undef X
    return false;
}

// Launch shape.  Measured winners for the shapes in tuned_plans.inc; otherwise a rule distilled from
// those measurements: about one workgroup per compute unit (more when the tile is small), as few
// K splits across workgroups as that allows (each costs an fp32 partial round trip that grows
// with M), and as many tiles per wavefront as that allows (each x fragment is reused per tile).
// Any knob set through w4a16_set_param overrides the corresponding field.
static Plan choose_plan(int M, int N, int K)
{
    const Params &p = params();
    const int mt = (M + 15) / 16;
    const int groups = K / kGroup, tiles = pad_cols(N) / 16;
    Plan best = {0, 0, 0, 0, 1, 0, 0};
    if (p.flat_groups > 0) {   // forced: the all-loads-up-front variant
        const int tw = p.tiles_per_wave ? p.tiles_per_wave : 2, nw = p.waves_per_wg ? p.waves_per_wg : 8;
        const int s = p.split_k > 0 ? p.split_k : 1;
        if (M <= kFlatMaxRows && flat_variant_exists(tw, nw, p.flat_groups) && groups == s * nw * p.flat_groups)
            best = {tw, nw, 0, s, p.fused_reduce == 2 ? 1 : p.fused_reduce, 0, p.flat_groups};
        return best;
    }
    const bool free_choice = !p.tiles_per_wave && !p.waves_per_wg && !p.prefetch_depth && !p.split_k && !p.k_sets;
    if (free_choice) {
        for (const TunedFlatRow &r : kTunedFlat)
            if (r.N == N && r.K == K && M <= r.m_max && M <= kFlatMaxRows && flat_variant_exists(r.tw, r.nw, r.ng) &&
                groups == r.S * r.nw * r.ng) {
                Plan pl = {r.tw, r.nw, 0, r.S, r.fused, 0, r.ng};
                if (p.fused_reduce != 2) pl.fused = p.fused_reduce;
                return pl;
            }
        for (const TunedRow &r : kTuned)
            if (r.N == N && r.K == K && r.mt == row_bucket(M) && variant_exists(mt, r.tw, r.nw, r.depth, r.ks))
                best = {r.tw, r.nw, r.depth, r.S, r.fused, r.ks, 0};
    }
    if (p.k_sets > 0) {   // forced: the high-occupancy column-split variant
        const int tw = p.tiles_per_wave ? p.tiles_per_wave : 4, depth = p.prefetch_depth ? p.prefetch_depth : 2;
        int s = p.split_k > 0 ? p.split_k : 1;
        if (s > groups) s = groups;
        if (p.even_split) s = 0;
        if (variant_exists(mt, tw, 0, depth, p.k_sets)) best = {tw, 0, depth, s, p.fused_reduce == 1, p.k_sets, 0};
        return best;
    }
    if (best.tw == 0 && free_choice && mt > 1) {
        // no measured row: the high-occupancy variant with two K sets, about one workgroup per
        // compute unit, wide tiles only when the columns alone fill the chip
        const int tw = tiles / 16 >= 200 ? 4 : 2;
        const int units = (tiles / tw + 3) / 4;
        int s = (256 + units / 2) / units;
        if (s > groups / 4) s = groups / 4;   // two groups per K set at least
        if (s < 1) s = 1;
        if (variant_exists(mt, tw, 0, 1, 2)) best = {tw, 0, 1, s, 0, 2, 0};
    }
    if (best.tw == 0) {
        const int forced_s = p.split_k > 0 ? (p.split_k < groups ? p.split_k : groups) : 0;
        double best_cost = 1e30;
        for (int tw = 8; tw >= 2; tw >>= 1) {
            if (p.tiles_per_wave > 0 && tw != p.tiles_per_wave) continue;
            for (int nw = 1; nw <= 16; nw = (nw == 1 ? 4 : nw << 1)) {
                if (p.waves_per_wg > 0 ? nw != p.waves_per_wg : (nw == 16 || nw == 1)) continue;
                for (int depth = 1; depth <= 4; depth <<= 1) {
                    if (p.prefetch_depth > 0 ? depth != p.prefetch_depth : depth != 1) continue;
                    if (!variant_exists(mt, tw, nw, depth)) continue;
                    const int units = nw == 1 ? (tiles / tw + 3) / 4 : tiles / tw;   // workgroups per K split
                    const int kways = nw == 1 ? 1 : nw;                        // wavefronts sharing a K range
                    int cap = groups / (2 * kways) > 0 ? groups / (2 * kways) : 1;   // two groups per wavefront at least
                    if (cap > 16) cap = 16;
                    for (int s = forced_s ? forced_s : 1; s <= (forced_s ? forced_s : cap); ++s) {
                        const double fill = (double)units * s / 256.0;         // workgroups per compute unit
                        double cost = fill >= 1 ? 0.25 * (fill - 1) : 1.5 * (1 / fill - 1);
                        cost += 0.06 * mt * (s - 1);                            // partial-sum round trip
                        cost += 0.05 * mt * (8 / tw - 1);                       // x-fragment reuse
                        cost += (mt > 1 && nw > 4) ? 0.3 : 0.0;                 // registers: big tiles want 4 wavefronts
                        cost += (mt == 1 && nw == 4 && units * s < 384) ? 0.3 : 0.0;
                        if (groups % (s * kways) != 0) cost += 0.2;            // uneven work per wavefront
                        if (cost < best_cost) { best_cost = cost; best = {tw, nw, depth, s, mt == 1, 0, 0}; }
                    }
                }
            }
        }
    }
    if (p.fused_reduce != 2) best.fused = p.fused_reduce;
    return best;   // tw == 0: the knobs name a variant that is not compiled
}

// Even split of the column-split kernel's (workgroup unit, group) pairs over the compute units:
// run length, number of runs (= workgroups) and the largest number of runs that touch one unit.
constexpr int kComputeUnits = 256;
struct EvenSplit { int per, runs, max_slots; };
static EvenSplit even_split(int wg_units, int groups)
{
    const long long total = (long long)wg_units * groups;
    EvenSplit e;
    e.per = (int)((total + kComputeUnits - 1) / kComputeUnits);
    e.runs = (int)((total + e.per - 1) / e.per);
    e.max_slots = 1;
    for (int u = 0; u < wg_units; ++u) {
        const int first = (int)(((long long)u * groups) / e.per), last = (int)((((long long)u + 1) * groups - 1) / e.per);
        if (last - first + 1 > e.max_slots) e.max_slots = last - first + 1;
    }
    return e;
}

// plan.S == 0 asks for that even split (column-split kernels only); otherwise S is the number of K splits
static size_t partial_bytes(int mt, int nblocks, const Plan &pl, int groups)
{
    const size_t units = (size_t)nblocks * kTiles / pl.tw;
    const int slots = pl.S == 0 ? even_split((int)((units + 3) / 4), groups).max_slots : pl.S;
    return slots > 1 ? units * slots * (4 * pl.tw * mt * 64) * sizeof(float) : 0;
}

// symmetric-weight instantiations exist for the K-split and the high-occupancy column-split kernels; the other
// two families (and any call without the caller's word for it) read the zero-points, which is always correct
template <int MT, int TW, int NW, int DEPTH, bool SYM>
static int launch_sym(const void *x, const void *packed, const Out &y, int M, int N, int K, int S, int fused,
                      void *workspace, hipStream_t stream)
{
    static bool lds_ok = false;   // LDS above 64 KB needs an opt-in, once per kernel
    const size_t lds_bytes = (size_t)NW * 4 * TW * MT * 64 * sizeof(float);
    if (lds_bytes > 160 * 1024) return W4A16_EUNSUP;
    if (!lds_ok && lds_bytes > 48 * 1024) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_kernel<MT, TW, NW, DEPTH, SYM>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes) != hipSuccess)
            return W4A16_EHIP;
        lds_ok = true;
    }
    const int groups = K / kGroup, nblocks = pad_cols(N) / kBlockCols;
    const int units = nblocks * kTiles / TW;
    uint32_t *tickets = reinterpret_cast<uint32_t *>(workspace);
    float *partial = reinterpret_cast<float *>(reinterpret_cast<uint8_t *>(workspace) + kTicketBytes);
    hipLaunchKernelGGL((gemm_kernel<MT, TW, NW, DEPTH, SYM>), dim3((unsigned)S, (unsigned)units), dim3(NW * 64), lds_bytes,
                       stream, (const _Float16 *)x, (const uint8_t *)packed, y, partial, tickets, M, N,
                       K, groups, S, fused, groups / S, groups % S);
    if (S > 1 && !fused)
        hipLaunchKernelGGL((splitk_reduce_kernel<MT, TW>), dim3((unsigned)units), dim3(kReduceThreads), 0, stream,
                           (const float *)partial, y, M, N, S);
    return launch_status();
}

template <int MT, int TW, int NW, int DEPTH>
static int launch(const void *x, const void *packed, const Out &y, int M, int N, int K, int S, int fused,
                  void *workspace, hipStream_t stream)
{
    return y.sym ? launch_sym<MT, TW, NW, DEPTH, true>(x, packed, y, M, N, K, S, fused, workspace, stream)
                 : launch_sym<MT, TW, NW, DEPTH, false>(x, packed, y, M, N, K, S, fused, workspace, stream);
}

template <int MT, int TW, int DEPTH>
static int launch_ns(const void *x, const void *packed, const Out &y, int M, int N, int K, int S, void *workspace,
                     hipStream_t stream)
{
    static bool lds_ok = false;
    const size_t lds_bytes = (size_t)TW * MT * 4096;   // four wavefronts' results; the x tiles (MT * 8 KB) fit inside
    if (!lds_ok && lds_bytes > 48 * 1024) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_ns_kernel<MT, TW, DEPTH>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes) != hipSuccess)
            return W4A16_EHIP;
        lds_ok = true;
    }
    const int groups = K / kGroup, units = pad_cols(N) / 16 / TW;
    float *partial = reinterpret_cast<float *>(reinterpret_cast<uint8_t *>(workspace) + kTicketBytes);
    hipLaunchKernelGGL((gemm_ns_kernel<MT, TW, DEPTH>), dim3((unsigned)S, (unsigned)((units + 3) / 4)), dim3(256), lds_bytes, stream,
                       (const _Float16 *)x, (const uint8_t *)packed, y, partial, M, N, K, groups, S, groups / S,
                       groups % S);
    if (S > 1)
        hipLaunchKernelGGL((splitk_reduce_kernel<MT, TW>), dim3((unsigned)units), dim3(kReduceThreads), 0, stream,
                           (const float *)partial, y, M, N, S);
    return launch_status();
}

template <int MT, int TW, int KS, int DEPTH, bool SYM>
static int launch_cs_sym(const void *x, const void *packed, const Out &y, int M, int N, int K, int S, int fused,
                         void *workspace, hipStream_t stream)
{
    static bool lds_ok = false;
    const size_t lds_bytes = (size_t)KS * TW * MT * 4096;   // 4*KS wavefronts' results; the x tiles (KS * MT * 8 KB) fit inside
    if (lds_bytes > 160 * 1024) return W4A16_EUNSUP;
    if (!lds_ok && lds_bytes > 48 * 1024) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_cs_kernel<MT, TW, KS, DEPTH, SYM>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes) != hipSuccess)
            return W4A16_EHIP;
        lds_ok = true;
    }
    const int groups = K / kGroup, units = pad_cols(N) / 16 / TW;
    uint32_t *tickets = reinterpret_cast<uint32_t *>(workspace);
    float *partial = reinterpret_cast<float *>(reinterpret_cast<uint8_t *>(workspace) + kTicketBytes);
    if (S == 0) {   // even split of (unit, group) pairs over the compute units, summed by last arrivers
        const EvenSplit e = even_split((units + 3) / 4, groups);
        hipLaunchKernelGGL((gemm_cs_kernel<MT, TW, KS, DEPTH, SYM>), dim3((unsigned)e.runs), dim3(256 * KS), lds_bytes, stream,
                           (const _Float16 *)x, (const uint8_t *)packed, y, partial, tickets, M, N, K, groups,
                           e.max_slots, 1, 0, 0, e.per, (units + 3) / 4);
        return launch_status();
    }
    hipLaunchKernelGGL((gemm_cs_kernel<MT, TW, KS, DEPTH, SYM>), dim3((unsigned)S, (unsigned)((units + 3) / 4)), dim3(256 * KS),
                       lds_bytes, stream, (const _Float16 *)x, (const uint8_t *)packed, y, partial, tickets, M, N, K,
                       groups, S, fused, groups / S, groups % S, 0, 0);
    if (S > 1 && !fused)
        hipLaunchKernelGGL((splitk_reduce_kernel<MT, TW>), dim3((unsigned)units), dim3(kReduceThreads), 0, stream,
                           (const float *)partial, y, M, N, S);
    return launch_status();
}

template <int MT, int TW, int KS, int DEPTH>
static int launch_cs(const void *x, const void *packed, const Out &y, int M, int N, int K, int S, int fused,
                     void *workspace, hipStream_t stream)
{
    return y.sym ? launch_cs_sym<MT, TW, KS, DEPTH, true>(x, packed, y, M, N, K, S, fused, workspace, stream)
                 : launch_cs_sym<MT, TW, KS, DEPTH, false>(x, packed, y, M, N, K, S, fused, workspace, stream);
}

template <int TW, int NW, int NG>
static int launch_flat(const void *x, const void *packed, const Out &y, int M, int N, int K, int S, int fused,
                       void *workspace, hipStream_t stream)
{
    static bool lds_ok = false;
    const size_t x_bytes = (size_t)M * (NW * NG * 16 + 1) * 16, sum_bytes = (size_t)NW * 4 * TW * 64 * sizeof(float);
    const size_t lds_bytes = x_bytes > sum_bytes ? x_bytes : sum_bytes;
    const size_t lds_max = (size_t)kFlatMaxRows * (NW * NG * 16 + 1) * 16 > sum_bytes
                               ? (size_t)kFlatMaxRows * (NW * NG * 16 + 1) * 16 : sum_bytes;
    if (lds_max > 160 * 1024) return W4A16_EUNSUP;
    if (!lds_ok && lds_max > 48 * 1024) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_flat_kernel<TW, NW, NG>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_max) != hipSuccess)
            return W4A16_EHIP;
        lds_ok = true;
    }
    const int groups = K / kGroup, units = pad_cols(N) / 16 / TW;
    uint32_t *tickets = reinterpret_cast<uint32_t *>(workspace);
    float *partial = reinterpret_cast<float *>(reinterpret_cast<uint8_t *>(workspace) + kTicketBytes);
    hipLaunchKernelGGL((gemm_flat_kernel<TW, NW, NG>), dim3((unsigned)S, (unsigned)units), dim3(NW * 64), lds_bytes,
                       stream, (const _Float16 *)x, (const uint8_t *)packed, y, partial, tickets, M, N,
                       K, groups, S, fused);
    if (S > 1 && !fused)
        hipLaunchKernelGGL((splitk_reduce_kernel<1, TW>), dim3((unsigned)units), dim3(kReduceThreads), 0, stream,
                           (const float *)partial, y, M, N, S);
    return launch_status();
}

static int dispatch(int mt, const Plan &pl, const void *x, const void *packed, const Out &y, int M, int N, int K,
                    void *workspace, hipStream_t stream)
{
#define F(TW_, NW_, NG_)                                                           \
    if (pl.tw == TW_ && pl.nw == NW_ && pl.ng == NG_)                              \
        return launch_flat<TW_, NW_, NG_>(x, packed, y, M, N, K, pl.S, pl.fused, workspace, stream);
    if (pl.ng > 0) {
        W4_FLAT_VARIANTS(F)
        return W4A16_EUNSUP;
    }
#undef F
#define Z(MT_, TW_, KS_, D_)                                                       \
    if (mt == MT_ && pl.ks == KS_ && pl.tw == TW_ && pl.depth == D_)               \
        return launch_cs<MT_, TW_, KS_, D_>(x, packed, y, M, N, K, pl.S, pl.fused, workspace, stream);
    if (pl.ks > 0) {
        W4_CS_VARIANTS(Z)
        return W4A16_EUNSUP;
    }
#undef Z
#define X(MT_, TW_, NW_, D_)                                                       \
    if (mt == MT_ && pl.tw == TW_ && pl.nw == NW_ && pl.depth == D_)               \
        return launch<MT_, TW_, NW_, D_>(x, packed, y, M, N, K, pl.S, pl.fused, workspace, stream);
    W4_VARIANTS(X)
#undef X
#define Y(MT_, TW_, D_)                                                            \
    if (mt == MT_ && pl.nw == 1 && pl.tw == TW_ && pl.depth == D_)                 \
        return launch_ns<MT_, TW_, D_>(x, packed, y, M, N, K, pl.S, workspace, stream);
    W4_NS_VARIANTS(Y)
#undef Y
    return W4A16_EUNSUP;
}

}  // namespace w4

using namespace w4;

extern "C" {

size_t w4a16_workspace_bytes(int M_max, int N, int K, int G)
{
    if (check_weight_shape(N, K, G) != W4A16_OK || M_max < 1 || M_max > W4A16_MAX_M) return 0;
    const int nblocks = pad_cols(N) / kBlockCols;
    size_t need = 0;
    for (int m = 1; m <= M_max; ++m) {   // the plan depends on M only through a few thresholds: cheap enough
        const Plan pl = choose_plan(m, N, K);
        size_t b = pl.tw ? partial_bytes((m + 15) / 16, nblocks, pl, K / kGroup) : 0;
        if (b > need) need = b;
    }
    return kTicketBytes + need;
}

static int gemm_entry(const void *x, const void *packed, const Out &out, int M, int N, int K, int G, void *workspace,
                      size_t workspace_bytes, void *stream)
{
    int rc = check_weight_shape(N, K, G);
    if (rc != W4A16_OK) return rc;
    if (M < 1) return W4A16_EINVAL;
    if (M > W4A16_MAX_M) return W4A16_EUNSUP;
    if (!x || !packed || !out.y) return W4A16_ENULL;
    if (misaligned(x) || misaligned(packed) || misaligned(out.y) || workspace_misaligned(workspace)) return W4A16_EALIGN;
    const int nblocks = pad_cols(N) / kBlockCols;
    const int mt = (M + 15) / 16;
    Plan pl = choose_plan(M, N, K);
    if (pl.tw == 0) return W4A16_EUNSUP;
    // one ticket per column unit: only the last-arriver sums use them
    const bool wants_tickets = pl.S == 0 || (pl.S > 1 && pl.fused && pl.nw != 1);
    if (wants_tickets && nblocks * kTiles / pl.tw > kMaxTickets) {
        if (pl.S == 0) return W4A16_EUNSUP;   // the even split has no two-kernel form
        pl.fused = 0;                         // same K split, summed by the second kernel
    }
    if (pl.S != 1) {
        const size_t need = partial_bytes(mt, nblocks, pl, K / kGroup);
        if (need > 0 && !workspace) return W4A16_EWORKSPACE;
        if (need > 0 && workspace_bytes < kTicketBytes + need) return W4A16_EWORKSPACE;
    }
    return dispatch(mt, pl, x, packed, out, M, N, K, workspace, (hipStream_t)stream);
}

// ---- w4a16_gemm for callers that cannot allocate a workspace ---------------------------------------
// The split-K partial sums and tickets live in a file-scope device array instead of a caller buffer.
// In host code the array's name is only a handle for hipGetSymbolAddress: the device address it yields
// (one per GPU, each GPU holds its own copy) is what kernels and the ticket clear receive.
constexpr size_t kStaticScratchPartials = (size_t)32 << 20;
constexpr size_t kStaticScratchBytes = kTicketBytes + kStaticScratchPartials;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static void *scratch_of_device[kMaxDevices];   // device address of `scratch`, by HIP device ordinal

static int static_scratch(void **ptr)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return W4A16_EHIP;
    if (!scratch_of_device[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return W4A16_EHIP;
        scratch_of_device[dev] = p;
    }
    *ptr = scratch_of_device[dev];
    return W4A16_OK;
}

int w4a16_gemm_static(const void *x, const void *packed, void *y, int M, int N, int K, int G, void *stream)
{
    int rc = check_weight_shape(N, K, G);
    if (rc != W4A16_OK) return rc;
    if (M < 1) return W4A16_EINVAL;
    if (M > W4A16_MAX_M) return W4A16_EUNSUP;
    if (!x || !packed || !y) return W4A16_ENULL;
    if (misaligned(x) || misaligned(packed) || misaligned(y)) return W4A16_EALIGN;
    const Plan pl = choose_plan(M, N, K);
    if (pl.tw == 0) return W4A16_EUNSUP;
    const size_t need = pl.S != 1 ? partial_bytes((M + 15) / 16, pad_cols(N) / kBlockCols, pl, K / kGroup) : 0;
    if (need > kStaticScratchPartials) return W4A16_EWORKSPACE;   // this shape needs more than the built-in scratch holds
    void *ws = nullptr;
    if ((rc = static_scratch(&ws)) != W4A16_OK) return rc;
    // The array keeps what the previous call left.  Partial sums are all written before they are read; the
    // tickets must start at zero, and although a finished call leaves them so, one that was cut short would
    // not: they are cleared here (a fill kernel, so the call can be captured in a graph) whenever they are used.
    if (pl.S == 0 || (pl.S > 1 && pl.fused && pl.nw != 1))
        if ((rc = w4a16_workspace_init(ws, kStaticScratchBytes, stream)) != W4A16_OK) return rc;
    return gemm_entry(x, packed, Out{(_Float16 *)y, nullptr, kEpiNone}, M, N, K, G, ws, kStaticScratchBytes, stream);
}

int w4a16_plan_describe(int M, int N, int K, int G, int *out)
{
    if (!out) return W4A16_ENULL;
    int rc = check_weight_shape(N, K, G);
    if (rc != W4A16_OK) return rc;
    if (M < 1) return W4A16_EINVAL;
    if (M > W4A16_MAX_M) return W4A16_EUNSUP;
    const Plan pl = choose_plan(M, N, K);
    if (pl.tw == 0) return W4A16_EUNSUP;
    const int family = pl.ng > 0 ? 1 : pl.ks > 0 ? 3 : pl.nw == 1 ? 2 : 0;
    const int plan[8] = {family, (M + 15) / 16, pl.tw, family == 3 ? pl.ks : pl.nw, family == 1 ? pl.ng : pl.depth,
                         pl.S, pl.S > 1 ? pl.fused : 0, (family == 0 || family == 3) ? 1 : 0};
    for (int i = 0; i < 8; ++i) out[i] = plan[i];
    return W4A16_OK;
}

int w4a16_gemm(const void *x, const void *packed, void *y, int M, int N, int K, int G,
               void *workspace, size_t workspace_bytes, void *stream)
{
    return gemm_entry(x, packed, Out{(_Float16 *)y, nullptr, kEpiNone}, M, N, K, G, workspace, workspace_bytes, stream);
}

int w4a16_gemm_fused(const void *x, const void *packed, void *y, int M, int N, int K, int G, int epilogue,
                     const void *residual, void *workspace, size_t workspace_bytes, void *stream)
{
    const int sym = (epilogue & W4A16_SYMMETRIC) ? 1 : 0;
    epilogue &= ~W4A16_SYMMETRIC;
    if (epilogue != W4A16_EPI_NONE && epilogue != W4A16_EPI_RESIDUAL && epilogue != W4A16_EPI_SILU_MUL)
        return W4A16_EINVAL;
    if (epilogue == W4A16_EPI_RESIDUAL) {
        if (!residual) return W4A16_ENULL;
        if (misaligned(residual)) return W4A16_EALIGN;
    } else if (residual) {
        return W4A16_EINVAL;
    }
    if (epilogue == W4A16_EPI_SILU_MUL && (N <= 0 || N % 32 != 0)) return W4A16_EINVAL;
    static_assert(W4A16_EPI_NONE == kEpiNone && W4A16_EPI_RESIDUAL == kEpiResidual && W4A16_EPI_SILU_MUL == kEpiSiluMul,
                  "public and internal epilogue codes agree");
    Out out = {(_Float16 *)y, (const _Float16 *)residual, epilogue};
    out.sym = sym;
    return gemm_entry(x, packed, out, M, N, K, G, workspace, workspace_bytes, stream);
}


int w4a16_gemm_rope(const void *x, const void *packed, int M, int K, int G, const int32_t *pos, const float *cos_table,
                    const float *sin_table, int n_pos, void *q, void *k_cache, void *v_cache, int P, int Hq, int Hkv, int D,
                    void *workspace, size_t workspace_bytes, void *stream)
{
    return w4::gemm_rope(x, packed, M, K, G, pos, cos_table, sin_table, n_pos, q, k_cache, v_cache, P, Hq, Hkv, D, workspace,
                         workspace_bytes, stream, 0);
}

}  // extern "C"

int w4::gemm_rope(const void *x, const void *packed, int M, int K, int G, const int32_t *pos, const float *cos_table,
                  const float *sin_table, int n_pos, void *q, void *k_cache, void *v_cache, int P, int Hq, int Hkv, int D,
                  void *workspace, size_t workspace_bytes, void *stream, int symmetric)
{
    if (P < 0 || Hq < 1 || Hkv < 1 || D < 32 || D % 32 != 0 || n_pos < 1) return W4A16_EINVAL;
    if ((long long)(Hq + 2 * Hkv) * D > 0x7fffffff) return W4A16_EUNSUP;
    if (!pos || !cos_table || !sin_table || !q || !k_cache || !v_cache) return W4A16_ENULL;
    if (misaligned(q) || misaligned(k_cache) || misaligned(v_cache) || misaligned(cos_table) || misaligned(sin_table) ||
        (reinterpret_cast<uintptr_t>(pos) & 3u))
        return W4A16_EALIGN;
    Out out = {(_Float16 *)q, nullptr, kEpiRope,
               {pos, cos_table, sin_table, (_Float16 *)q, (_Float16 *)k_cache, (_Float16 *)v_cache, n_pos, P, Hq, Hkv, D}};
    out.sym = symmetric ? 1 : 0;
    return gemm_entry(x, packed, out, M, (Hq + 2 * Hkv) * D, K, G, workspace, workspace_bytes, stream);
}
