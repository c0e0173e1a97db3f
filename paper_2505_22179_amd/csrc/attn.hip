// tree_verify_attn: attention of the tree-verification pass (paper section 2.1) on gfx950.
//
// Scores are computed transposed, S^T = K . Q^T, with 16x16x32 fp16 MFMA steps over the head
// dimension, so that a lane ends up with eight scores of ONE query row: exactly the operand
// fragment the P.V product needs, with no shuffle in between.  The tree mask is applied to the
// draft keys only, softmax runs online in fp32 (base-2 exponentials), and V enters its product
// transposed (the contraction there runs over keys while V is stored with the head dimension
// contiguous).  Key ranges of different workgroups are combined in range order, by the last
// workgroup of a tile to finish or by a second small kernel, so the result does not depend on
// scheduling.  Two kernels: tree_attn_shared_kernel, which every call runs by default (eight
// wavefronts, K and V tiles brought to LDS once per workgroup and shared), and the older
// tree_attn_kernel (every wavefront fetches its own K fragments and V rows), kept selectable.
#include <type_traits>

#include "internal.h"
#include "devscope.h"

namespace w4 {

typedef _Float16 half8v __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kHeadDim = 128;
constexpr int kKeyBlock = 32;
constexpr int kRowsPad = 64;
// LDS of a workgroup of 4 * RG wavefronts with RT row tiles each: one exchange slot per wavefront
// (8 * RT accumulator quads + 2 * RT state values per lane); the slots cover the 8 KB V tiles
constexpr int attn_lds_bytes(int rt, int rg) { return 4 * rg * (8 * rt * 4 + 2 * rt) * 64 * 4; }
constexpr int kMaxSplits = 16;   // key ranges per head (the merge keeps one value per range in registers)

// v_max3_f32 and v_max_f32 as they stand: fmaxf chains are compiled with a canonicalising v_max x, x per
// operand, which doubles the instruction count of a row maximum; no score here is a NaN.
__device__ __forceinline__ float max_of_three(float a, float b, float c)
{
    float d;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
    return d;
}

__device__ __forceinline__ float max_of_two(float a, float b)
{
    float d;
    asm("v_max_f32 %0, %1, %2" : "=v"(d) : "v"(a), "v"(b));
    return d;
}

// Maximum over the four lanes l, l ^ 16, l ^ 32, l ^ 48 (the lanes that share a query row), returned to
// all four.  v_permlane16_swap exchanges the odd 16-lane rows of its first operand with the even rows of
// its second, v_permlane32_swap the upper half of the first with the lower half of the second; applied
// to two copies of a value each leaves the two partners of a pair side by side in the two registers.
// They run on the vector ALU: no LDS round trip as with a cross-lane shuffle.  (Written in assembly:
// the compiler's builtin folded the maximum of the two results into one of them.)
__device__ __forceinline__ float row_group_max(float v)
{
    float a = v, b = v;
    asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1" : "+v"(a), "+v"(b));
    a = max_of_two(a, b);
    b = a;
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
    return max_of_two(a, b);
}

constexpr float kLowest = -1.0e30f;   // "no key seen yet": finite, so differences of two of them are 0, not NaN

// Merge of the key ranges of one tile by the workgroup that finished last (fused mode): NS = compiled
// upper bound of the number of ranges, IT = items a thread handles at once (all their loads are issued
// together).  Loads are device-scope: other workgroups, on other XCDs, wrote the partials in this kernel.
template <int NS, int IT>
__device__ __forceinline__ void merge_ranges(PartialBuffer unit_o, PartialBuffer unit_ml, _Float16 *__restrict__ out,
                                             int tid, int threads, int items, int M, int Hq, int nsplit, int rep,
                                             int unit)
{
    const float NEG_INF = -__builtin_inff();
    for (int base = tid; base < items; base += threads * IT) {
        float ms[IT][NS], ls[IT][NS];
        float4v os[IT][NS];
#pragma unroll
        for (int it = 0; it < IT; ++it) {
            const int idx = base + it * threads;
            const int trow = idx / (kHeadDim / 4), d4 = idx % (kHeadDim / 4);
#pragma unroll
            for (int s = 0; s < NS; ++s) {
                ms[it][s] = NEG_INF;
                ls[it][s] = 0.f;
                os[it][s] = (float4v){0.f, 0.f, 0.f, 0.f};
                if (s < nsplit && idx < items) {
                    ms[it][s] = load_partial_f32(unit_ml, (s * kRowsPad + trow) * 2);
                    ls[it][s] = load_partial_f32(unit_ml, (s * kRowsPad + trow) * 2 + 1);
                    os[it][s] = load_partial(unit_o, (s * kRowsPad + trow) * (kHeadDim / 4) + d4);
                }
            }
        }
#pragma unroll
        for (int it = 0; it < IT; ++it) {
            const int idx = base + it * threads;
            if (idx >= items) break;
            const int trow = idx / (kHeadDim / 4), d4 = idx % (kHeadDim / 4);
            float m_all = NEG_INF;
#pragma unroll
            for (int s = 0; s < NS; ++s) m_all = fmaxf(m_all, ms[it][s]);
            float den = 0.f;
            float4v num = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < NS; ++s) {
                float wgt = (ms[it][s] == NEG_INF) ? 0.f : __builtin_amdgcn_exp2f(ms[it][s] - m_all);
                den += wgt * ls[it][s];
                num += wgt * os[it][s];
            }
            const float inv = 1.f / den;
            // tile row -> (query row, head): see tree_attn_kernel
            const int j = rep ? trow / M : 0;
            const int qrow = trow - j * M, h = rep ? unit * rep + j : unit;
            typedef _Float16 half4v __attribute__((ext_vector_type(4)));
            half4v hv = {(_Float16)(num[0] * inv), (_Float16)(num[1] * inv), (_Float16)(num[2] * inv), (_Float16)(num[3] * inv)};
            *reinterpret_cast<half4v *>(out + ((size_t)qrow * Hq + h) * kHeadDim + d4 * 4) = hv;
        }
    }
}

// One workgroup = one 64-row tile (a query head, or the heads of a KV group) x one contiguous range
// of 32-key steps.  Its 4 * RG wavefronts are RG row groups of four: the four wavefronts of a row
// group split the KEYS -- wavefront kw takes steps kw, kw + 4, ... of the range -- and each carries,
// for the RT * 16 rows of its group, its own online-softmax state -- running maximum, running sum and an
// unnormalised output tile -- so K and V rows are fetched once per workgroup (no wavefront re-reads
// another's keys), the main loop has no workgroup barrier, and the four states meet once, at the
// end, through LDS.  RT = 4, RG = 1: one wavefront per SIMD holds all 64 rows.  RT = 2, RG = 2: two
// wavefronts per SIMD with 32 rows each (half the accumulator and Q registers, K/V fragments fetched
// twice from L2): one wavefront's dependent softmax chain hides behind the other's matrix work.
// RT = 2, RG = 1: tiles of at most 32 rows; two such workgroups fit a compute unit.
//
// Per step a lane's registers hold, for row tile rt (rows 16 rt + c) and lane (r, c):
//   S^T = K . Q^T     sa[rt][i], sb[rt][i]: keys 4r + i of the step's two 16-key tiles, row 16 rt + c
//                     -- eight scores of ONE query row, which after exp2 and fp16 rounding are, as they
//                     stand, the second operand P^T of the next product (contraction slot 8r + p:
//                     p < 4 the first tile's key 4r + p, p >= 4 the second tile's key 4r + p - 4)
//   O^T += V^T . P^T  o[dt][rt][i]: head-dim element 16 dt + 4r + i of row 16 rt + c: the row index
//                     is the lane's c again, so the rescale factor of a row is lane-local
// V^T (first operand: head-dim element 16 dt + c, the eight keys of contraction slots 8r ..) comes
// from a per-wavefront LDS tile vt[d][32 keys in slot order], written as 8-byte units of four keys
// and read as one 16-byte load per dt; 16-byte chunks are XOR-swizzled by bits of d against bank
// conflicts.  The same wavefront writes and reads the tile: LDS keeps its program order.
template <int RT, int RG>
__global__ __launch_bounds__(256 * RG) void tree_attn_kernel(
    const _Float16 *__restrict__ q, const _Float16 *__restrict__ k, const _Float16 *__restrict__ v,
    const uint8_t *__restrict__ mask, _Float16 *__restrict__ out, float *__restrict__ part_o,
    float *__restrict__ part_ml, uint32_t *__restrict__ tickets, int M, int P, int Hq, int Hkv,
    float scale_log2e, int nsplit, int bq, int brem, int rep, int fused)
{
    extern __shared__ float4v smem4[];
    // one batch of scalar loads instead of three dependent ones before the first K/V request goes out
    const unsigned grid = gridDim.x;
    fetch_arguments_together(q, k, v, mask, out, part_o, part_ml, tickets, M, P, Hq, Hkv, scale_log2e, nsplit, bq, brem, rep,
                             fused, grid);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kw = wave & 3, rg = wave >> 2;   // key wavefront inside the row group, row group
    const int r = lane >> 4, c = lane & 15;
    // Workgroups are dealt to the eight XCDs round-robin by index, and each XCD has its own L2.
    // Renumber so that the workgroups of one KV head (consecutive logical ids) share an XCD and
    // its K/V rows are fetched into one L2 instead of all eight.
    int lid = blockIdx.x;
    if ((grid & 7) == 0) lid = (blockIdx.x & 7) * (grid >> 3) + (blockIdx.x >> 3);
    // A workgroup's row tile holds the M rows of one query head (rep == 0), or -- when they fit -- the M rows
    // of rep consecutive query heads that share a KV head (tile row j * M + m = head unit * rep + j, query
    // row m): few-row calls then read K and V once per rep heads instead of once per head.
    const int unit = lid / nsplit, sp = lid % nsplit;
    const int kvh = (rep ? unit * rep : unit) / (Hq / Hkv);
    const int R = rep ? M * rep : M;   // valid rows of the tile
    const int T = P + M;
    // key steps of this split: bq = nblk / nsplit each, the first brem = nblk % nsplit one more (host-computed)
    const int b0 = sp * bq + (sp < brem ? sp : brem), b1 = b0 + bq + (sp < brem ? 1 : 0);
    const size_t kv_stride = (size_t)Hkv * kHeadDim;

    int row[RT], head[RT];   // query row and head of tile row 16 (rg RT + rt) + c; tile rows >= R repeat row R-1 and are never stored
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        const int rho = min((rg * RT + rt) * 16 + c, R - 1);
        const int j = rep ? rho / M : 0;
        row[rt] = rho - j * M;
        head[rt] = rep ? unit * rep + j : unit;
    }
    // Tree mask as one 64-bit word per query row (bit j = draft key j visible), built once by the
    // workgroups whose key range reaches the draft keys: a byte load per key inside the step loop
    // would put some thirty dependent memory round trips on the critical path of the last steps.
    __shared__ uint64_t row_bits[kRowsPad];
    uint64_t mbits[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) mbits[rt] = 0;
    const bool reaches_draft = b1 * kKeyBlock > P;   // uniform over the workgroup
    // Requested first and used after the Q, K and V requests: the oldest loads.  Every lane loads from a
    // clamped, valid address and discards what lies outside the mask afterwards: a load under a per-lane
    // condition would be compiled as a branch with its own wait, sixteen memory round trips in a row.
    uint8_t mask_byte[16];
    const int mcol = min(lane, M - 1);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int mrow = min((wave & 3) * 16 + i, M - 1);   // wavefronts 0..3 cover the 64 rows
        mask_byte[i] = mask[(size_t)mrow * M + mcol];
    }
    // Q^T fragments (second operand of S^T): lane (r, c) holds q[row, h, 32 j + 8 r .. +7]
    half8v qf[RT][4];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            qf[rt][j] = *reinterpret_cast<const half8v *>(q + ((size_t)row[rt] * Hq + head[rt]) * kHeadDim + 32 * j + 8 * r);

    float4v o[8][RT];
#pragma unroll
    for (int dt = 0; dt < 8; ++dt)
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) o[dt][rt] = (float4v){0.f, 0.f, 0.f, 0.f};
    float m_run[RT], l_run[RT];   // l_run: this lane's share (its keys 4r + i) of the row's sum
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        m_run[rt] = kLowest;
        l_run[rt] = 0.f;
    }

    // this wavefront's transposed V tile: 128 rows (d) x 64 B (32 keys in contraction-slot order)
    uint8_t *vt = reinterpret_cast<uint8_t *>(smem4) + wave * (kHeadDim * 64);
    const _Float16 *kbase = k + (size_t)kvh * kHeadDim + 8 * r;
    // V staging: lane (g, ch) = (lane % 8, lane / 8) fetches keys 4g .. 4g+3 of the step, head-dim
    // chunks ch and ch + 8 (eight elements each); key group g sits in 8-byte unit 2 (g % 4) + g / 4
    const int vg = lane & 7, vch = lane >> 3;
    const _Float16 *vbase = v + (size_t)kvh * kHeadDim + vch * 8;
    auto load_k = [&](int step, half8v (&fa)[4], half8v (&fb)[4]) {
        const int key0 = step * kKeyBlock;
        const int ra = key0 + c, rb = key0 + 16 + c;
        const bool ragged = key0 + kKeyBlock > T;   // uniform: only the last step
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            fa[j] = *reinterpret_cast<const half8v *>(kbase + (size_t)(ragged ? min(ra, T - 1) : ra) * kv_stride + 32 * j);
            fb[j] = *reinterpret_cast<const half8v *>(kbase + (size_t)(ragged ? min(rb, T - 1) : rb) * kv_stride + 32 * j);
        }
    };
    auto load_v = [&](int step, u32x4 (&vr)[2][4]) {
        const int key0 = step * kKeyBlock;
        const int rv = key0 + 4 * vg;
        const bool ragged = key0 + kKeyBlock > T;
#pragma unroll
        for (int it = 0; it < 2; ++it)
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
                vr[it][kk] = *reinterpret_cast<const u32x4 *>(vbase + (size_t)(ragged ? min(rv + kk, T - 1) : rv + kk) * kv_stride + it * 64);
    };
    auto park_v = [&](const u32x4 (&vr)[2][4]) {
#pragma unroll
        for (int it = 0; it < 2; ++it)
#pragma unroll
            for (int dd = 0; dd < 8; ++dd) {
                const uint32_t sel = (dd & 1) ? 0x07060302u : 0x05040100u;   // the odd or the even halves of two words
                u32x2 unit;
                unit[0] = __builtin_amdgcn_perm(vr[it][1][dd >> 1], vr[it][0][dd >> 1], sel);
                unit[1] = __builtin_amdgcn_perm(vr[it][3][dd >> 1], vr[it][2][dd >> 1], sel);
                const int d = (vch + 8 * it) * 8 + dd;
                const int chunk = (vg & 3) ^ ((d >> 1) & 3) ^ ((d >> 3) & 3);
                *reinterpret_cast<u32x2 *>(vt + d * 64 + chunk * 16 + (vg >> 2) * 8) = unit;
            }
    };
    // One 32-key step.  The K fragments and the V rows of the wavefront's next step are requested
    // into the very registers this step has just emptied (V after its rows are parked in LDS, K after
    // the score products), so one register set each gives a prefetch distance of most of a step.
    auto step_fn = [&](int step, bool more, half8v (&fa)[4], half8v (&fb)[4], u32x4 (&vr)[2][4]) {
        const int key0 = step * kKeyBlock, next = step + 4;
        park_v(vr);
        if (more) load_v(next, vr);
        __builtin_amdgcn_sched_barrier(0);
        float4v sa[RT], sb[RT];
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            sa[rt] = (float4v){0.f, 0.f, 0.f, 0.f};
            sb[rt] = (float4v){0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) {
                sa[rt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fa[j], qf[rt][j], sa[rt], 0, 0, 0);
                sb[rt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fb[j], qf[rt][j], sb[rt], 0, 0, 0);
            }
        if (more) load_k(next, fa, fb);
        __builtin_amdgcn_sched_barrier(0);
        half8v pb[RT];
        const bool prefix_only = key0 + kKeyBlock <= P;   // uniform: committed keys, all visible
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            float s[8];
            if (prefix_only) {
#pragma unroll
                for (int i = 0; i < 8; ++i) s[i] = ((i < 4) ? sa[rt][i & 3] : sb[rt][i & 3]) * scale_log2e;
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int key = key0 + 4 * r + (i & 3) + (i >> 2) * 16;
                    const int j = key - P;   // draft key index; bits at and beyond M are clear
                    const bool vis = j < 0 || (j < 64 && ((mbits[rt] >> j) & 1));
                    const float raw = (i < 4) ? sa[rt][i & 3] : sb[rt][i & 3];
                    s[i] = vis ? raw * scale_log2e : -__builtin_inff();
                }
            }
            float m_blk = s[0];
#pragma unroll
            for (int i = 1; i < 8; ++i) m_blk = fmaxf(m_blk, s[i]);
            m_blk = row_group_max(m_blk);
            const float m_new = fmaxf(m_run[rt], m_blk);
            const float alpha = __builtin_amdgcn_exp2f(m_run[rt] - m_new);
            float psum = 0.f;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float pv = __builtin_amdgcn_exp2f(s[i] - m_new);
                psum += pv;
                pb[rt][i] = (_Float16)pv;
            }
            l_run[rt] = l_run[rt] * alpha + psum;
            m_run[rt] = m_new;
            if (__any(alpha != 1.0f)) {   // after the first steps a row's maximum rarely moves
#pragma unroll
                for (int dt = 0; dt < 8; ++dt) o[dt][rt] *= alpha;
            }
        }
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
            const int d = dt * 16 + c;
            const int chunk = r ^ ((d >> 1) & 3) ^ ((d >> 3) & 3);
            const half8v va = *reinterpret_cast<const half8v *>(vt + d * 64 + chunk * 16);
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) o[dt][rt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(va, pb[rt], o[dt][rt], 0, 0, 0);
        }
    };

    half8v ka[4], kb[4];
    u32x4 vr[2][4];
    const int first = b0 + kw;
    if (first < b1) {
        load_k(first, ka, kb);
        load_v(first, vr);
    }
    if (reaches_draft) {
        uint64_t mine = 0;   // lane i keeps the word of row 16 wave + i: one LDS write per wavefront instead of sixteen
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const uint64_t bits = __ballot(mask_byte[i] != 0 && wave * 16 + i < M && lane < M);
            mine = lane == i ? bits : mine;
        }
        if (lane < 16 && wave < 4) row_bits[wave * 16 + lane] = mine;
        __syncthreads();
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) mbits[rt] = row_bits[row[rt]];
    }
    for (int step = first; step < b1; step += 4)
        step_fn(step, step + 4 < b1, ka, kb, vr);

    // a row's sum over this wavefront's keys: add the four lanes (r = 0..3) that share the row
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        l_run[rt] += __shfl_xor(l_run[rt], 16, 64);
        l_run[rt] += __shfl_xor(l_run[rt], 32, 64);
    }
    // The wavefronts' states meet in LDS: each parks its whole state (8 * RT accumulator quads and
    // 2 * RT state values per lane, lane-contiguous), and after one barrier wavefront (rg, kw) combines, in
    // wavefront order, the head-dim tiles 2 kw and 2 kw + 1 of the four key wavefronts of its row group.
    constexpr int kQuads = 8 * RT;
    float4v *xq = smem4;                                                             // [slots][8 RT quads][64 lanes]
    float *xs = reinterpret_cast<float *>(smem4 + 4 * RG * kQuads * 64);             // [slots][2 RT values][64 lanes]
    __syncthreads();   // every wavefront has left its V tile: the exchange reuses that LDS
#pragma unroll
    for (int dt = 0; dt < 8; ++dt)
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) xq[(wave * kQuads + dt * RT + rt) * 64 + lane] = o[dt][rt];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        xs[(wave * 2 * RT + rt) * 64 + lane] = m_run[rt];
        xs[(wave * 2 * RT + RT + rt) * 64 + lane] = l_run[rt];
    }
    __syncthreads();
    const bool last = nsplit == 1;
    float *po = part_o + (size_t)lid * kRowsPad * kHeadDim;
    float *pml = part_ml + (size_t)lid * kRowsPad * 2;
    // fused mode: the partials of a tile's key ranges are published with device-scope stores and merged by
    // the last workgroup of the tile to finish (below)
    const PartialBuffer unit_o = partial_buffer(part_o + (size_t)unit * nsplit * kRowsPad * kHeadDim);
    const PartialBuffer unit_ml = partial_buffer(part_ml + (size_t)unit * nsplit * kRowsPad * 2);
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        float ms[4], wgt[4], m_all = kLowest, l_all = 0.f;
#pragma unroll
        for (int w2 = 0; w2 < 4; ++w2) {
            ms[w2] = xs[((rg * 4 + w2) * 2 * RT + rt) * 64 + lane];
            m_all = fmaxf(m_all, ms[w2]);
        }
#pragma unroll
        for (int w2 = 0; w2 < 4; ++w2) {
            wgt[w2] = __builtin_amdgcn_exp2f(ms[w2] - m_all);
            l_all += wgt[w2] * xs[((rg * 4 + w2) * 2 * RT + RT + rt) * 64 + lane];
        }
        const int orow = (rg * RT + rt) * 16 + c;
        const float inv = last ? 1.f / l_all : 1.f;
#pragma unroll
        for (int dd = 0; dd < 2; ++dd) {
            const int dt = 2 * kw + dd;
            float4v val = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int w2 = 0; w2 < 4; ++w2) val += wgt[w2] * xq[((rg * 4 + w2) * kQuads + dt * RT + rt) * 64 + lane];
            val *= inv;
            // tile row orow, head-dim elements 16 dt + 4r .. + 3: four consecutive outputs
            if (orow < R) {
                if (last) {
                    typedef _Float16 half4v __attribute__((ext_vector_type(4)));
                    half4v hv = {(_Float16)val[0], (_Float16)val[1], (_Float16)val[2], (_Float16)val[3]};
                    *reinterpret_cast<half4v *>(out + ((size_t)row[rt] * Hq + head[rt]) * kHeadDim + dt * 16 + 4 * r) = hv;
                } else if (fused) {
                    store_partial(unit_o, (sp * kRowsPad + orow) * (kHeadDim / 4) + dt * 4 + r, val);
                } else {
                    *reinterpret_cast<float4v *>(po + orow * kHeadDim + dt * 16 + 4 * r) = val;
                }
            }
        }
        if (!last && kw == 0 && r == 0 && orow < R) {
            // partial state of this key range
            if (fused) {
                store_partial_f32(unit_ml, (sp * kRowsPad + orow) * 2, m_all);
                store_partial_f32(unit_ml, (sp * kRowsPad + orow) * 2 + 1, l_all);
            } else {   // a second kernel merges the ranges (the kernel boundary makes them visible, at no fence cost)
                pml[orow * 2] = m_all;
                pml[orow * 2 + 1] = l_all;
            }
        }
    }
    if (last || !fused) return;   // uniform over the grid
    // The workgroups of a tile take a ticket each once their partials have reached device scope; the one
    // that draws the last ticket merges the tile's key ranges, in range order, with the arithmetic of
    // tree_attn_merge_kernel, and leaves the ticket at zero for the next call.
    __shared__ uint32_t ticket_sh;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0) ticket_sh = __hip_atomic_fetch_add(&tickets[unit], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (ticket_sh != (uint32_t)(nsplit - 1)) return;
    if (tid == 0) __hip_atomic_store(&tickets[unit], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int items = R * (kHeadDim / 4);   // one item = four consecutive outputs of a tile row
    if (nsplit <= 4)
        merge_ranges<4, 4>(unit_o, unit_ml, out, tid, 256 * RG, items, M, Hq, nsplit, rep, unit);
    else if (nsplit <= 8)
        merge_ranges<8, 2>(unit_o, unit_ml, out, tid, 256 * RG, items, M, Hq, nsplit, rep, unit);
    else
        merge_ranges<kMaxSplits, 1>(unit_o, unit_ml, out, tid, 256 * RG, items, M, Hq, nsplit, rep, unit);
}

// ---- Row tiles of 33..64 rows: K and V tiles shared through LDS -------------------------------------
// The kernel above lets every wavefront fetch its own K fragments and V rows from global memory.  With
// a full tile that costs twice: a K fragment load touches sixteen key rows with 64 bytes each, the
// costliest pattern for the address path of a compute unit (about four times the time of a load of
// whole cache lines), and 64 rows of accumulators and Q fragments fill the register file of a SIMD
// with one wavefront, so nothing overlaps that wavefront's softmax arithmetic, its matrix products
// and its memory waits.  Here a workgroup has eight wavefronts, two per SIMD: wavefront (kw, rh)
// holds tile rows 32 rh .. 32 rh + 31 and takes key step 4 t + kw of the workgroup's range in round t.
// All K and V tiles of a round (four steps of 32 keys, 8 KB each for K and for V) are brought in one
// round ahead by direct global -> LDS loads of whole key rows (one instruction: four rows of 256 B),
// the K tile of a step by wavefront (kw, 0) and the V tile by (kw, 1), double-buffered, one workgroup
// barrier per round.  Both wavefronts of a pair read the same tiles:
//   K fragments   one 16-byte LDS read per fragment; the 16-byte chunks of a key row are stored at
//                 chunk ^ (key % 8), the permutation being applied to the SOURCE address of the
//                 transfer (its destination is fixed: lane l of a transfer fills bytes 16 l ..)
//   V^T fragments the transposing LDS read (ds_read_b64_tr_b16): in each block of 16 lanes, lane s
//                 points at four consecutive head-dim elements 4 (s % 4) .. of key row s / 4, and
//                 lane c receives element c of the four rows -- four keys at one head-dim index,
//                 which is the operand layout, with no pass through registers.  Chunks of a V row
//                 are stored at chunk ^ (2 key % 16).
// Q reaches its fragments the same way (once, through the second round buffer).  The softmax is that
// of the kernel above with the scale folded into the exponent's multiply-add; the states of the four
// key wavefronts of a row half meet in LDS at the end, in a row-major layout (rows padded to 528 B)
// from which thread t then reads, merges and stores whole 512-byte output rows.
constexpr int kSharedWaves = 8;
constexpr int kTileBytes = kKeyBlock * kHeadDim * 2;         // one K or V tile: 32 keys x 256 B
constexpr int kStepBytes = 2 * kTileBytes;                   // K tile, then V tile
constexpr int kRoundBytes = 4 * kStepBytes;                  // the four key steps of a round
constexpr int kExRow = kHeadDim * 4 + 16;                    // exchange row: 128 fp32 + 16 B of padding
constexpr int kExWave = 32 * kExRow;                         // per wavefront: its 32 rows
constexpr int kExState = kSharedWaves * kExWave;             // then [8 wavefronts][32 rows] (max, sum)
constexpr int kSharedLds = kExState + kSharedWaves * 32 * 8 > 2 * kRoundBytes ? kExState + kSharedWaves * 32 * 8 : 2 * kRoundBytes;

typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void global_void;
typedef short short4v __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) short4v lds_short4v;

__device__ __forceinline__ uint32_t lds_address(const void *p)
{
    return (uint32_t)(size_t)(lds_void *)p;
}
// The transposing read of the rows at lds_addr and 16 key rows (4 KB) further on.  Written in assembly: through
// the builtin the compiler waits, before every such read, for ALL outstanding global -> LDS transfers -- the
// next round's, requested a moment earlier precisely so that they overlap this round's arithmetic.  The
// compiler therefore does not know of these reads; wait_lds_reads says when their results may be used.
template <int OFFSET>
__device__ __forceinline__ void read_transposed_pair(short4v &lo, short4v &hi, uint32_t lds_addr)
{
    asm volatile("ds_read_b64_tr_b16 %0, %2 offset:%3\n\tds_read_b64_tr_b16 %1, %2 offset:%4"
                 : "=&v"(lo), "=&v"(hi)
                 : "v"(lds_addr), "n"(OFFSET), "n"(OFFSET + 16 * 256));
}
// returns once at most N LDS operations of this wavefront (the N most recent) are still under way; `first` is
// the first result of the oldest pair still awaited, so that its use cannot be moved above the wait
template <int N>
__device__ __forceinline__ void wait_lds_reads(short4v &first)
{
    asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(first) : "n"(N));
}
// lane l's 16 bytes at src land at lds_base + 16 l (lds_base wavefront-uniform); counted by vmcnt
__device__ __forceinline__ void row_to_lds(const uint8_t *src, uint8_t *lds_base)
{
    __builtin_amdgcn_global_load_lds((global_void *)src, (lds_void *)lds_base, 16, 0, 0);
}

__global__ __launch_bounds__(64 * kSharedWaves) void tree_attn_shared_kernel(
    const _Float16 *__restrict__ q, const _Float16 *__restrict__ k, const _Float16 *__restrict__ v,
    const uint8_t *__restrict__ mask, _Float16 *__restrict__ out, float *__restrict__ part_o,
    float *__restrict__ part_ml, uint32_t *__restrict__ tickets, int M, int P, int Hq, int Hkv,
    float scale_log2e, int nsplit, int bq, int brem, int rep, int fused)
{
    extern __shared__ float4v smem4[];
    uint8_t *lds = reinterpret_cast<uint8_t *>(smem4);
    const unsigned grid = gridDim.x;
    fetch_arguments_together(q, k, v, mask, out, part_o, part_ml, tickets, M, P, Hq, Hkv, scale_log2e, nsplit, bq, brem, rep,
                             fused, grid);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kw = wave >> 1, rh = wave & 1;   // key wavefront, row half
    const int r = lane >> 4, c = lane & 15;
    int lid = blockIdx.x;   // workgroups of one KV head on one XCD (see tree_attn_kernel)
    if ((grid & 7) == 0) lid = (blockIdx.x & 7) * (grid >> 3) + (blockIdx.x >> 3);
    const int unit = lid / nsplit, sp = lid % nsplit;
    const int kvh = (rep ? unit * rep : unit) / (Hq / Hkv);
    const int R = rep ? M * rep : M;   // valid rows of the tile
    const int T = P + M;
    const int b0 = sp * bq + (sp < brem ? sp : brem), b1 = b0 + bq + (sp < brem ? 1 : 0);
    const int rounds = (b1 - b0 + 3) >> 2;
    const size_t kv_row_bytes = (size_t)Hkv * kHeadDim * 2;

    // tile row -> its query row and the element offset of its (query row, head) in q and out; rows >= R repeat
    // row R - 1 and are never stored
    auto locate = [&](int rho, int &qrow) {
        rho = min(rho, R - 1);
        const int j = rep ? rho / M : 0;
        qrow = rho - j * M;
        return (uint32_t)(qrow * Hq + (rep ? unit * rep + j : unit)) * kHeadDim;
    };
    // tree mask of the draft keys, one 64-bit word per query row, in the workgroups that reach them:
    // wavefront w asks for the bytes of rows 8 w .. 8 w + 7 first (lane = column) and turns them into words
    // after the transfers below have been requested
    __shared__ uint64_t row_bits[kRowsPad];
    const bool reaches_draft = b1 * kKeyBlock > P;   // uniform over the workgroup
    uint8_t mask_byte[8];
    if (reaches_draft) {
        const int mcol = min(lane, M - 1);
#pragma unroll
        for (int i = 0; i < 8; ++i) mask_byte[i] = mask[(size_t)min(wave * 8 + i, M - 1) * M + mcol];
    }

    // transfers: lane l of transfer i fills bytes 16 (l % 16) .. of tile row 4 i + l / 16
    const int trow = lane >> 4, tchunk = lane & 15;
    // LDS: per key wavefront pair 32 KB = two buffers of (K tile, V tile); Q sits in pair 0's second buffer until
    // that pair requests the tiles of its second round
    uint8_t *const pair_lds = lds + kw * (2 * kStepBytes);
    uint8_t *const qtile = lds + kStepBytes;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int rho = 4 * (2 * wave + u) + trow;
        int qrow;
        const uint32_t elem = locate(rho, qrow);
        row_to_lds(reinterpret_cast<const uint8_t *>(q) + (size_t)elem * 2 + ((tchunk ^ (rho & 7)) << 4), qtile + (2 * wave + u) * 1024);
    }
    // K (rh = 0) or V (rh = 1) rows of this wavefront's key steps.  Tile row 4 i + trow goes to chunk positions
    // permuted by key % 8 (K) or 2 key % 16 (V), which depends on i through its parity only: two lane offsets,
    // added to a wavefront-uniform address that moves with the step and with i.
    const uint8_t *const kv_src = reinterpret_cast<const uint8_t *>(rh ? v : k) + (size_t)kvh * kHeadDim * 2;
    uint32_t lane_src[2];
#pragma unroll
    for (int par = 0; par < 2; ++par) {
        const int key = 4 * par + trow;
        lane_src[par] = (uint32_t)trow * (uint32_t)kv_row_bytes + (uint32_t)((tchunk ^ (rh ? (2 * key) & 15 : key & 7)) << 4);
    }
    auto request_round = [&](int t, int buf) {
        const int step = b0 + 4 * t + kw;
        if (step >= b1) return;   // uniform over the wavefront
        const int key0 = step * kKeyBlock;
        uint8_t *dst = pair_lds + buf * kStepBytes + rh * kTileBytes;
        if (key0 + kKeyBlock <= T) {
            const uint8_t *from = kv_src + (size_t)key0 * kv_row_bytes;
#pragma unroll
            for (int i = 0; i < 8; ++i) row_to_lds(from + (size_t)(4 * i) * kv_row_bytes + lane_src[i & 1], dst + i * 1024);
        } else {   // the last step of all: rows beyond the last key repeat it (they are masked out below)
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int key = 4 * i + trow;
                const int swz = rh ? (2 * key) & 15 : key & 7;
                row_to_lds(kv_src + (size_t)min(key0 + key, T - 1) * kv_row_bytes + ((tchunk ^ swz) << 4), dst + i * 1024);
            }
        }
    };
    request_round(0, 0);

    if (reaches_draft) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint64_t bits = __ballot(mask_byte[i] != 0 && wave * 8 + i < M && lane < M);
            if (lane == i) row_bits[wave * 8 + i] = bits;
        }
    }
    // Q fragments (second operand of S^T): lane (r, c) holds elements 32 j + 8 r .. + 7 of tile row 32 rh + 16 rt + c
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    half8v qf[2][4];
    uint64_t mbits[2] = {0, 0};
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) {
        const int rho = 32 * rh + 16 * rt + c;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            qf[rt][j] = *reinterpret_cast<const half8v *>(qtile + rho * 256 + (((4 * j + r) ^ (rho & 7)) << 4));
        int qrow;
        locate(rho, qrow);
        if (reaches_draft) mbits[rt] = row_bits[qrow];
    }

    float4v o[8][2];
#pragma unroll
    for (int dt = 0; dt < 8; ++dt)
#pragma unroll
        for (int rt = 0; rt < 2; ++rt) o[dt][rt] = (float4v){0.f, 0.f, 0.f, 0.f};
    float m_run[2] = {kLowest, kLowest}, l_run[2] = {0.f, 0.f};   // l_run: this lane's share (its keys) of the row's sum

    // fragment addresses inside the pair's first buffer (the second lies kStepBytes further on: an immediate offset)
    const uint8_t *kfrag[4];   // K: key c (and 16 + c: + 4 KB), chunk (4 j + r) ^ (c % 8)
#pragma unroll
    for (int j = 0; j < 4; ++j) kfrag[j] = pair_lds + ((c * 256 + ((r ^ (c & 7)) << 4)) ^ (j << 6));
    // V: lane c of block r points at key row 4 r + c / 4 (and 16 + that: + 4 KB), elements 16 dt + 4 (c % 4) ..
    const int vkey = 4 * r + (c >> 2);
    const int voff = vkey * 256 + (((((c >> 1) & 1)) ^ ((2 * vkey) & 15)) << 4) + (c & 1) * 8;
    uint32_t vfrag[8];
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) vfrag[dt] = lds_address(pair_lds + kTileBytes) + (voff ^ (dt << 5));

    // one round, on buffer BUF of the pair (the loop below alternates them, so that BUF is a compile-time offset)
    auto round = [&](auto buf_tag, int t) {
        constexpr int BUF = decltype(buf_tag)::value;
        // this wavefront's transfers of round t have landed; after the barrier everybody's have, and nobody
        // still reads the other buffer
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        __syncthreads();
        if (t + 1 < rounds) request_round(t + 1, BUF ^ 1);
        const int step = b0 + 4 * t + kw;
        const bool active = step < b1;   // uniform over the wavefront; the barriers are outside these branches
        const int key0 = step * kKeyBlock;
        half8v pb[2];
        if (active) {
            float4v sa[2], sb[2];
#pragma unroll
            for (int rt = 0; rt < 2; ++rt) {
                sa[rt] = (float4v){0.f, 0.f, 0.f, 0.f};
                sb[rt] = (float4v){0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const half8v fa = *reinterpret_cast<const half8v *>(kfrag[j] + BUF * kStepBytes);
                const half8v fb = *reinterpret_cast<const half8v *>(kfrag[j] + BUF * kStepBytes + 16 * 256);
#pragma unroll
                for (int rt = 0; rt < 2; ++rt) {
                    sa[rt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fa, qf[rt][j], sa[rt], 0, 0, 0);
                    sb[rt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fb, qf[rt][j], sb[rt], 0, 0, 0);
                }
            }
            const bool prefix_only = key0 + kKeyBlock <= P;   // uniform: committed keys, all visible
#pragma unroll
            for (int rt = 0; rt < 2; ++rt) {
                float s[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) s[i] = (i < 4) ? sa[rt][i & 3] : sb[rt][i & 3];
                if (!prefix_only) {
                    // visibility of the step's 32 keys as one word: the step's first key is draft key `first`
                    // (-31 .. 63; negative: the step begins with committed keys, all visible); mask bits at and
                    // beyond M are clear, so keys past the last one are hidden
                    const int first = key0 - P;
                    const uint64_t window = first >= 0 ? mbits[rt] >> first : (mbits[rt] << -first) | ((1ull << -first) - 1);
                    const uint32_t mine = (uint32_t)window >> (4 * r);   // bit i: key 4 r + i; bit 16 + i: key 16 + 4 r + i
#pragma unroll
                    for (int i = 0; i < 8; ++i) s[i] = ((mine >> ((i & 3) + 16 * (i >> 2))) & 1u) ? s[i] : -__builtin_inff();
                }
                // the scale is positive (checked by the host): the largest raw score is the largest scaled one
                const float m_blk = row_group_max(max_of_three(max_of_three(s[0], s[1], s[2]), max_of_three(s[3], s[4], s[5]), max_of_two(s[6], s[7])));
                const float m_new = max_of_two(m_run[rt], m_blk * scale_log2e);
                const float alpha = __builtin_amdgcn_exp2f(m_run[rt] - m_new);
                float pv[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    pv[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[i], scale_log2e, -m_new));
                    pb[rt][i] = (_Float16)pv[i];
                }
                const float psum = ((pv[0] + pv[1]) + (pv[2] + pv[3])) + ((pv[4] + pv[5]) + (pv[6] + pv[7]));
                l_run[rt] = l_run[rt] * alpha + psum;
                m_run[rt] = m_new;
                if (__any(alpha != 1.0f)) {   // after the first steps a row's maximum rarely moves
#pragma unroll
                    for (int dt = 0; dt < 8; ++dt) o[dt][rt] *= alpha;
                }
            }
        }
        if (!active) return;
        // V^T fragments, two head-dim tiles ahead of the products that use them: contraction slots 8 r .. 8 r + 3
        // are keys 4 r .. of the step's first 16, slots 8 r + 4 .. those of its second 16
        short4v lo[8], hi[8];
        read_transposed_pair<BUF * kStepBytes>(lo[0], hi[0], vfrag[0]);
        read_transposed_pair<BUF * kStepBytes>(lo[1], hi[1], vfrag[1]);
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
            if (dt + 2 < 8) read_transposed_pair<BUF * kStepBytes>(lo[dt + 2], hi[dt + 2], vfrag[dt + 2]);
            if (dt + 2 < 8)
                wait_lds_reads<4>(lo[dt]);
            else if (dt + 1 < 8)
                wait_lds_reads<2>(lo[dt]);
            else
                wait_lds_reads<0>(lo[dt]);
            typedef short short8v __attribute__((ext_vector_type(8)));
            const short8v both = __builtin_shufflevector(lo[dt], hi[dt], 0, 1, 2, 3, 4, 5, 6, 7);
            const half8v va = __builtin_bit_cast(half8v, both);
#pragma unroll
            for (int rt = 0; rt < 2; ++rt) o[dt][rt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(va, pb[rt], o[dt][rt], 0, 0, 0);
        }
    };
    for (int t = 0; t < rounds; t += 2) {
        round(std::integral_constant<int, 0>{}, t);
        if (t + 1 < rounds) round(std::integral_constant<int, 1>{}, t + 1);
    }

    // a row's sum over this wavefront's keys: add the four lanes (r = 0..3) that share the row
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) {
        l_run[rt] += __shfl_xor(l_run[rt], 16, 64);
        l_run[rt] += __shfl_xor(l_run[rt], 32, 64);
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __syncthreads();   // every wavefront has left the K and V tiles: the exchange reuses that LDS
    uint8_t *const mine = lds + wave * kExWave;
    float *const state = reinterpret_cast<float *>(lds + kExState);   // [wavefront][row of its half][max, sum]
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) {
#pragma unroll
        for (int dt = 0; dt < 8; ++dt)
            *reinterpret_cast<float4v *>(mine + (16 * rt + c) * kExRow + (4 * dt + r) * 16) = o[dt][rt];
        if (r == 0) {
            state[(wave * 32 + 16 * rt + c) * 2] = m_run[rt];
            state[(wave * 32 + 16 * rt + c) * 2 + 1] = l_run[rt];
        }
    }
    __syncthreads();
    // thread t merges, in wavefront order, the four key wavefronts' values of four consecutive outputs of a row:
    // 32 threads per row, whole rows per store
    const bool last = nsplit == 1;
    const PartialBuffer unit_o = partial_buffer(part_o + (size_t)unit * nsplit * kRowsPad * kHeadDim);
    const PartialBuffer unit_ml = partial_buffer(part_ml + (size_t)unit * nsplit * kRowsPad * 2);
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int item = tid + it * (64 * kSharedWaves);
        const int rho = item >> 5, quad = item & 31;   // tile row, its outputs 4 quad .. 4 quad + 3
        const int half_ = rho >> 5, hrow = rho & 31;
        float ms[4], wgt[4], m_all = kLowest, l_all = 0.f;
#pragma unroll
        for (int w2 = 0; w2 < 4; ++w2) {
            ms[w2] = state[((2 * w2 + half_) * 32 + hrow) * 2];
            m_all = fmaxf(m_all, ms[w2]);
        }
        float4v val = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int w2 = 0; w2 < 4; ++w2) {
            wgt[w2] = __builtin_amdgcn_exp2f(ms[w2] - m_all);
            l_all += wgt[w2] * state[((2 * w2 + half_) * 32 + hrow) * 2 + 1];
            val += wgt[w2] * *reinterpret_cast<const float4v *>(lds + (2 * w2 + half_) * kExWave + hrow * kExRow + quad * 16);
        }
        if (rho >= R) continue;
        if (last) {
            val *= 1.f / l_all;
            typedef _Float16 half4v __attribute__((ext_vector_type(4)));
            half4v hv = {(_Float16)val[0], (_Float16)val[1], (_Float16)val[2], (_Float16)val[3]};
            int qrow;
            *reinterpret_cast<half4v *>(out + locate(rho, qrow) + quad * 4) = hv;
        } else {
            // written through to memory in either mode: left in the L2 as ordinary stores, the partials of the
            // two-kernel mode would all be written back at the end of the kernel, after the last workgroup
            store_partial(unit_o, (sp * kRowsPad + rho) * (kHeadDim / 4) + quad, val);
            if (quad == 0) {
                store_partial_f32(unit_ml, (sp * kRowsPad + rho) * 2, m_all);
                store_partial_f32(unit_ml, (sp * kRowsPad + rho) * 2 + 1, l_all);
            }
        }
    }
    if (last || !fused) return;   // uniform over the grid
    // last-arriver merge of the tile's key ranges, as in tree_attn_kernel
    __shared__ uint32_t ticket_sh;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0) ticket_sh = __hip_atomic_fetch_add(&tickets[unit], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (ticket_sh != (uint32_t)(nsplit - 1)) return;
    if (tid == 0) __hip_atomic_store(&tickets[unit], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int items = R * (kHeadDim / 4);
    if (nsplit <= 4)
        merge_ranges<4, 4>(unit_o, unit_ml, out, tid, 64 * kSharedWaves, items, M, Hq, nsplit, rep, unit);
    else if (nsplit <= 8)
        merge_ranges<8, 2>(unit_o, unit_ml, out, tid, 64 * kSharedWaves, items, M, Hq, nsplit, rep, unit);
    else
        merge_ranges<kMaxSplits, 1>(unit_o, unit_ml, out, tid, 64 * kSharedWaves, items, M, Hq, nsplit, rep, unit);
}

// merge of the key ranges: one thread per four consecutive output elements, ranges in order;
// NS = compiled upper bound of the number of ranges (all loads of a thread are issued at once)
template <int NS>
__global__ __launch_bounds__(256) void tree_attn_merge_kernel(const float *__restrict__ part_o,
                                                              const float *__restrict__ part_ml,
                                                              _Float16 *__restrict__ out, int M, int Hq, int nsplit,
                                                              int rep)
{
    fetch_arguments_together(part_o, part_ml, out, M, Hq, nsplit, rep);
    const int idx = blockIdx.x * 256 + threadIdx.x;   // over M * Hq * 32 quads
    if (idx >= M * Hq * (kHeadDim / 4)) return;
    const int d4 = idx % (kHeadDim / 4), h = (idx / (kHeadDim / 4)) % Hq, qrow = idx / (kHeadDim / 4) / Hq;
    const float NEG_INF = -__builtin_inff();
    // where the first kernel left this (row, head): tile `unit`, tile row `row` (see tree_attn_kernel)
    const int unit = rep ? h / rep : h, row = rep ? (h % rep) * M + qrow : qrow;
    const float *hml = part_ml + (size_t)unit * nsplit * kRowsPad * 2;
    const float4v *ho = reinterpret_cast<const float4v *>(part_o + (size_t)unit * nsplit * kRowsPad * kHeadDim);
    float ms[NS], ls[NS];
    float4v os[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        ms[s] = NEG_INF;
        ls[s] = 0.f;
        os[s] = (float4v){0.f, 0.f, 0.f, 0.f};
        if (s < nsplit) {
            ms[s] = hml[((size_t)s * kRowsPad + row) * 2];
            ls[s] = hml[((size_t)s * kRowsPad + row) * 2 + 1];
            os[s] = ho[((size_t)s * kRowsPad + row) * (kHeadDim / 4) + d4];
        }
    }
    float m_all = NEG_INF;
#pragma unroll
    for (int s = 0; s < NS; ++s) m_all = fmaxf(m_all, ms[s]);
    float den = 0.f;
    float4v num = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        float wgt = (ms[s] == NEG_INF) ? 0.f : __builtin_amdgcn_exp2f(ms[s] - m_all);   // ranges without a visible key: l = 0
        den += wgt * ls[s];
        num += wgt * os[s];
    }
    const float inv = 1.f / den;
    typedef _Float16 half4v __attribute__((ext_vector_type(4)));
    half4v hv = {(_Float16)(num[0] * inv), (_Float16)(num[1] * inv), (_Float16)(num[2] * inv), (_Float16)(num[3] * inv)};
    *reinterpret_cast<half4v *>(out + ((size_t)qrow * Hq + h) * kHeadDim + d4 * 4) = hv;
}

// Greedy acceptance of a verified draft tree, then compaction of the accepted K/V rows.
// Wavefront 0 walks the tree with lane i = node i: at node cur it broadcasts target[cur], every lane
// tests "my parent is cur and my token is that", and the lowest set bit of the ballot is the next
// node.  cur grows strictly, so the walk ends after at most M rounds whatever the input holds.
// Then all 256 threads move the accepted rows: thread t owns 16-byte column chunk t of every row and
// copies row path[j] to row j for j = 1, 2, ... in this order; path[j] >= j and the path is
// increasing, so a row is never overwritten before it has been read, and threads never share bytes.
__global__ __launch_bounds__(256) void tree_accept_kernel(const int32_t *__restrict__ parent,
                                                          const int32_t *__restrict__ token,
                                                          const int32_t *__restrict__ target, int M,
                                                          int32_t *__restrict__ path, int32_t *__restrict__ result,
                                                          u32x4 *k, u32x4 *v, int P, int row_chunks)
{
    __shared__ int32_t path_sh[kRowsPad];
    __shared__ int32_t n_sh;
    fetch_arguments_together(parent, token, target, M, path, result, k, v, P, row_chunks);
    const int tid = threadIdx.x;
    if (tid < 64) {
        const int lane = tid;
        const bool node = lane < M;
        const int32_t my_parent = node ? parent[lane] : -2;
        const int32_t my_token = node ? token[lane] : 0;
        const int32_t my_target = node ? target[lane] : 0;
        int cur = 0, n = 1;
        int32_t mine = lane == 0 ? 0 : -1;   // path entry of position `lane`
        for (;;) {
            const int32_t want = __shfl(my_target, cur, 64);
            const uint64_t hits = __ballot(node && lane > cur && my_parent == cur && my_token == want);
            if (hits == 0) break;
            cur = __builtin_ctzll(hits);
            if (lane == n) mine = cur;
            ++n;
        }
        const int32_t next_token = __shfl(my_target, cur, 64);   // the target model's own token after the last accepted node
        path_sh[lane] = mine;
        if (node) path[lane] = mine;
        if (lane == 0) {
            n_sh = n;
            result[0] = n;
            result[1] = next_token;
        }
    }
    __syncthreads();
    if (k == nullptr) return;
    const int n = n_sh;
    for (int item = tid; item < 2 * row_chunks; item += 256) {
        u32x4 *base = (item < row_chunks ? k : v) + (size_t)P * row_chunks + (item < row_chunks ? item : item - row_chunks);
        for (int j = 1; j < n; ++j) {
            const int src = path_sh[j];
            if (src != j) base[(size_t)j * row_chunks] = base[(size_t)src * row_chunks];
        }
    }
}

// Query heads per row tile (0 = one head per tile).  The heads of a KV group can share a tile, which reads K
// and V once for all of them; fewer tiles, on the other hand, mean more key ranges per tile to fill the chip,
// and every range costs a partial result that has to be merged.  Measured over M = 1 .. 32 with 64/8 and 32/8
// heads (prefix 2048), the best point is about 32 tiles (eight key ranges each, merged by the last workgroup):
// the smallest pack that leaves at most 32 tiles is taken -- two heads of a group of eight with 64 heads (10.3
// to 12.9 us for M = 1 .. 16, against 12.7 to 13.2 unpacked), none with 32 heads (10.0 to 12.6 us for
// M = 1 .. 32, against 10.7 to 18.6 with two per tile).  Calls of so few rows that a whole group fits eight
// tile rows pack the group (plain decoding: 9.9 against 10.3 us).
static int attn_rep(int M, int Hq, int Hkv)
{
    const int group = Hq / Hkv, knob = params().attn_pack;
    if (knob == 1 || group < 2) return 0;
    if (knob >= 10) {   // 10 + d: exactly d heads per tile, where that is possible
        const int d = knob - 10;
        return (d >= 2 && group % d == 0 && M * d <= kRowsPad) ? d : 0;
    }
    if (knob == 2) return M * group <= kRowsPad ? group : 0;
    if (M * group <= 8) return group;
    int best = 1;
    for (int d = 1; d <= group; ++d) {
        if (group % d != 0 || M * d > kRowsPad) continue;
        best = d;
        if (Hq / d <= 32) break;
    }
    return best >= 2 ? best : 0;
}

static int attn_splits(int M, int P, int units)
{
    int nblk = (P + M + kKeyBlock - 1) / kKeyBlock;
    int want = params().attn_splits > 0 ? params().attn_splits : (256 + units - 1) / units;   // about one workgroup per compute unit
    if (want > nblk) want = nblk;
    if (want > kMaxSplits) want = kMaxSplits;
    return want < 1 ? 1 : want;
}

template <int RT, int RG, typename... Args>
static int launch_attn_variant(int grid, hipStream_t stream, Args... args)
{
    static bool lds_ok = false;   // LDS above 48 KB needs an opt-in, once per variant
    constexpr int lds = attn_lds_bytes(RT, RG);
    if (!lds_ok) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&tree_attn_kernel<RT, RG>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess)
            return W4A16_EHIP;
        lds_ok = true;
    }
    hipLaunchKernelGGL((tree_attn_kernel<RT, RG>), dim3((unsigned)grid), dim3(256 * RG), lds, stream, args...);
    return W4A16_OK;
}

template <typename... Args>
static int launch_attn_shared(int grid, hipStream_t stream, Args... args)
{
    static bool lds_ok = false;
    if (!lds_ok) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&tree_attn_shared_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kSharedLds) != hipSuccess)
            return W4A16_EHIP;
        lds_ok = true;
    }
    hipLaunchKernelGGL(tree_attn_shared_kernel, dim3((unsigned)grid), dim3(64 * kSharedWaves), kSharedLds, stream, args...);
    return W4A16_OK;
}

template <typename... Args>
static int launch_attn(int rt, int rgroups, int grid, hipStream_t stream, Args... args)
{
    if (rt == 0) return launch_attn_shared(grid, stream, args...);
    if (rt == 4) return launch_attn_variant<4, 1>(grid, stream, args...);
    if (rgroups == 2) return launch_attn_variant<2, 2>(grid, stream, args...);
    return launch_attn_variant<2, 1>(grid, stream, args...);
}

static int check_attn(int M, int P, int Hq, int Hkv, int D)
{
    if (M < 1 || P < 0 || Hq < 1 || Hkv < 1 || D < 1) return W4A16_EINVAL;
    if (Hq % Hkv != 0) return W4A16_EINVAL;
    if (D != kHeadDim || M > W4A16_MAX_M || Hq > kMaxTickets || Hq / Hkv > 8) return W4A16_EUNSUP;
    return W4A16_OK;
}

}  // namespace w4

using namespace w4;

extern "C" {

size_t tree_verify_attn_workspace_bytes(int M, int P, int Hq, int Hkv, int D)
{
    if (check_attn(M, P, Hq, Hkv, D) != W4A16_OK) return 0;
    const int nblk = (P + M + kKeyBlock - 1) / kKeyBlock;
    const int ns = nblk < kMaxSplits ? nblk : kMaxSplits;   // the most splits any setting of the knobs can ask for
    return kTicketBytes + (size_t)Hq * ns * kRowsPad * (kHeadDim + 2) * sizeof(float);
}

int tree_verify_attn(const void *q, const void *k, const void *v, const uint8_t *mask, void *out,
                     int M, int P, int Hq, int Hkv, int D, float scale,
                     void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = check_attn(M, P, Hq, Hkv, D);
    if (rc != W4A16_OK) return rc;
    if (!(scale > 0.f) || scale > 3.0e38f) return W4A16_EINVAL;   // the kernels take row maxima before scaling
    if (!q || !k || !v || !mask || !out) return W4A16_ENULL;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(out) || workspace_misaligned(workspace)) return W4A16_EALIGN;
    const int rep = attn_rep(M, Hq, Hkv);
    const int units = rep ? Hq / rep : Hq;
    const int ns = attn_splits(M, P, units);
    const size_t need = kTicketBytes + (size_t)units * ns * kRowsPad * (kHeadDim + 2) * sizeof(float);
    if (ns > 1 && (!workspace || workspace_bytes < need)) return W4A16_EWORKSPACE;
    float *part_o = reinterpret_cast<float *>(reinterpret_cast<uint8_t *>(workspace) + kTicketBytes);
    float *part_ml = part_o + (size_t)units * ns * kRowsPad * kHeadDim;
    const float scale_log2e = scale * 1.4426950408889634f;
    const int nblk = (P + M + kKeyBlock - 1) / kKeyBlock;
    // Every tile runs in the kernel that shares K and V tiles through LDS (rt = 0 below): it is the fastest
    // form at every tile height, with half of its rows padding too (prefix 2048, 64/8 heads: 11.2 against
    // 12.0 us at M = 8, 13.8 against 16.7 at M = 24, 15.7 against 22.3 at M = 64).  The older kernel stays
    // selectable for comparison: one wavefront per SIMD carrying all 64 rows (4), or 32 rows per wavefront,
    // in two row groups for taller tiles (2).
    const int rows = rep ? M * rep : M;
    const int knob = params().attn_row_tiles;
    const int rt = knob == 4 ? 4 : knob == 2 ? 2 : 0, rgroups = (rt == 2 && rows > 32) ? 2 : 1;
    // The key ranges of a tile are merged by the last of its workgroups to finish, or by a second kernel.  Fused
    // saves a launch and the wait for it, but one workgroup then reads all the partials of its tile (rows x
    // ranges x 512 B), which pays while they are few.  Measured break-even points, prefix 2048: about 160 row-
    // ranges with up to four ranges (64 heads, M = 33 .. 64: 14.7 fused against 14.9 us at 132, 16.3 against
    // 15.5 at 256); with five to eight ranges 512 for tiles of one head (32 heads, M = 64: 15.6 against 16.7 us)
    // and 256 for packed ones (64 heads in pairs: 12.9 against 13.1 us at M = 16, 14.4 against 13.6 at M = 24);
    // 256 with more ranges (M = 4 of 32 heads 10.7 against 11.0 us at 256, M = 8 of 64 heads 14.0 against 11.0
    // at 512).
    const int fm = params().attn_fused_merge;
    const int row_ranges = rows * ns;
    const bool few = row_ranges <= (ns <= 4 ? 160 : (ns <= 8 && !rep) ? 512 : 256);
    const int fused = (ns > 1 && fm != 1 && (fm == 2 || few)) ? 1 : 0;
    rc = launch_attn(rt, rgroups, units * ns, (hipStream_t)stream, (const _Float16 *)q, (const _Float16 *)k,
                     (const _Float16 *)v, mask, (_Float16 *)out, part_o, part_ml, reinterpret_cast<uint32_t *>(workspace),
                     M, P, Hq, Hkv, scale_log2e, ns, nblk / ns, nblk % ns, rep, fused);
    if (rc != W4A16_OK) return rc;
    if (ns > 1 && !fused) {
        const int quads = M * Hq * (kHeadDim / 4);
        const dim3 grid((unsigned)((quads + 255) / 256));
        if (ns <= 4)
            hipLaunchKernelGGL(tree_attn_merge_kernel<4>, grid, dim3(256), 0, (hipStream_t)stream, (const float *)part_o,
                               (const float *)part_ml, (_Float16 *)out, M, Hq, ns, rep);
        else if (ns <= 8)
            hipLaunchKernelGGL(tree_attn_merge_kernel<8>, grid, dim3(256), 0, (hipStream_t)stream, (const float *)part_o,
                               (const float *)part_ml, (_Float16 *)out, M, Hq, ns, rep);
        else
            hipLaunchKernelGGL(tree_attn_merge_kernel<kMaxSplits>, grid, dim3(256), 0, (hipStream_t)stream,
                               (const float *)part_o, (const float *)part_ml, (_Float16 *)out, M, Hq, ns, rep);
    }
    return launch_status();
}

int tree_accept(const int32_t *parent, const int32_t *token, const int32_t *target, int M, int32_t *path,
                int32_t *result, void *k, void *v, int P, int Hkv, int D, void *stream)
{
    if (M < 1 || P < 0) return W4A16_EINVAL;
    if (M > W4A16_MAX_M) return W4A16_EUNSUP;
    if (!parent || !token || !target || !path || !result) return W4A16_ENULL;
    if ((k == nullptr) != (v == nullptr)) return W4A16_ENULL;
    int row_chunks = 0;
    if (k) {
        if (Hkv < 1 || D < 1) return W4A16_EINVAL;
        if (((size_t)Hkv * D * 2) % 16 != 0) return W4A16_EUNSUP;
        if (misaligned(k) || misaligned(v)) return W4A16_EALIGN;
        row_chunks = (int)((size_t)Hkv * D * 2 / 16);
    }
    if ((reinterpret_cast<uintptr_t>(parent) | reinterpret_cast<uintptr_t>(token) | reinterpret_cast<uintptr_t>(target) |
         reinterpret_cast<uintptr_t>(path) | reinterpret_cast<uintptr_t>(result)) & 3u)
        return W4A16_EALIGN;
    hipLaunchKernelGGL(tree_accept_kernel, dim3(1), dim3(256), 0, (hipStream_t)stream, parent, token, target, M, path,
                       result, (u32x4 *)k, (u32x4 *)v, P, row_chunks);
    return launch_status();
}

}  // extern "C"
