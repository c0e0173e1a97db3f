// tree_verify_attn: attention of the tree-verification pass (paper section 2.1) on gfx950.
//
// One workgroup handles one query head and one contiguous range of keys; each of its four
// wavefronts owns a 16-row tile of the (at most 64) draft-token query rows.  Scores are computed
// transposed, S^T = K . Q^T, with 16x16x32 fp16 MFMA steps over the head dimension, so that a lane
// ends up with eight scores of ONE query row (keys 4r..4r+3 of two 16-key tiles): exactly the
// first-operand fragment the P.V product needs, with no shuffle in between.  The tree mask is
// applied to the draft keys, softmax runs online in fp32 (base-2 exponentials), and V reaches the
// second MFMA operand through a double-buffered LDS tile shared by the four wavefronts, because
// the contraction there runs over keys while V is stored with the head dimension contiguous.  Key ranges are combined by a second small
// kernel, in range order, so the result does not depend on scheduling.
#include "internal.h"

namespace w4 {

typedef _Float16 half8v __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kHeadDim = 128;
constexpr int kKeyBlock = 32;
constexpr int kVtStride = 36;    // halves per LDS row of the transposed V tile (72 B: 8-byte aligned, 16 rows -> 16 banks)
constexpr int kOStride = 132;    // floats per LDS row of the output staging tile
constexpr int kAttnThreads = 256;
constexpr int kRowsPad = 64;
constexpr int kMaxSplits = 16;   // key ranges per head (the merge keeps one value per range in registers)

__device__ __forceinline__ float xor_max(float v, int lane_mask)
{
    return fmaxf(v, __shfl_xor(v, lane_mask, 64));
}

__global__ __launch_bounds__(kAttnThreads) void tree_attn_kernel(
    const _Float16 *__restrict__ q, const _Float16 *__restrict__ k, const _Float16 *__restrict__ v,
    const uint8_t *__restrict__ mask, _Float16 *__restrict__ out, float *__restrict__ part_o,
    float *__restrict__ part_ml, int M, int P, int Hq, int Hkv,
    float scale_log2e, int nsplit, int bq, int brem)
{
    // V tile of the current and of the next key block, TRANSPOSED: vt[d][key ^ 4*((d>>4)&7)], so a
    // lane's eight keys for one head-dim column are two 8-byte reads
    __shared__ _Float16 vt[2][kHeadDim][kVtStride];
    __shared__ float ot[4][16][kOStride];   // per-wavefront output tile for row-contiguous stores
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane >> 4, c = lane & 15;
    // Workgroups are dealt to the eight XCDs round-robin by index, and each XCD has its own L2.
    // Renumber so that the workgroups of one KV head (consecutive logical ids) share an XCD and
    // its K/V rows are fetched into one L2 instead of all eight.
    int lid = blockIdx.x;
    if ((gridDim.x & 7) == 0) lid = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
    const int h = lid / nsplit, sp = lid % nsplit;
    const int kvh = h / (Hq / Hkv);
    const int T = P + M;
    // key blocks of this split: bq = nblk / nsplit each, the first brem = nblk % nsplit one more (host-computed)
    const int b0 = sp * bq + (sp < brem ? sp : brem), b1 = b0 + bq + (sp < brem ? 1 : 0);
    const int row0 = wave * 16;
    const int my_row = min(row0 + c, M - 1);   // rows >= M repeat row M-1 and are never stored
    const size_t kv_stride = (size_t)Hkv * kHeadDim;
    const float NEG_INF = -__builtin_inff();

    // Q^T fragment (second operand): lane (r, c) holds q[my_row, h, 32 j + 8 r .. +7]
    half8v qf[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
        qf[j] = *reinterpret_cast<const half8v *>(q + ((size_t)my_row * Hq + h) * kHeadDim + 32 * j + 8 * r);

    float4v o[8];
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) o[dt] = (float4v){0.f, 0.f, 0.f, 0.f};

    // the workgroup stages each 32-key V block once (32 B per thread) and all four wavefronts read it
    const int st_key = tid >> 3, st_chunk = (tid & 7) * 2;
    const _Float16 *vbase = v + (size_t)kvh * kHeadDim + st_chunk * 8;
    const _Float16 *kbase = k + (size_t)kvh * kHeadDim + 8 * r;
    auto load_v = [&](int blk, u32x4 (&reg)[2]) {
        int src = blk * kKeyBlock + st_key;
        if (blk * kKeyBlock + kKeyBlock > T) src = min(src, T - 1);   // uniform: only the last block is ragged
        const _Float16 *p = vbase + (size_t)src * kv_stride;
        reg[0] = *reinterpret_cast<const u32x4 *>(p);
        reg[1] = *reinterpret_cast<const u32x4 *>(p + 8);
    };
    auto store_v = [&](int buf, const u32x4 (&reg)[2]) {
        // this thread holds V[st_key][st_chunk*8 .. +15]: scatter it down 16 rows of the transposed tile
        const int col = st_key ^ (4 * ((st_chunk >> 1) & 7));
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            uint32_t word = reg[i >> 3][(i >> 1) & 3];
            uint16_t h16 = (i & 1) ? (uint16_t)(word >> 16) : (uint16_t)(word & 0xFFFFu);
            vt[buf][st_chunk * 8 + i][col] = __builtin_bit_cast(_Float16, h16);
        }
    };
    // K fragments (first operand of S^T): tile a = keys key0 + 0..15, tile b = key0 + 16..31
    auto load_k = [&](int blk, half8v (&fa)[4], half8v (&fb)[4]) {
        const int key0 = blk * kKeyBlock;
        int ra = key0 + c, rb = key0 + 16 + c;
        if (key0 + kKeyBlock > T) {   // uniform: only the last block is ragged
            ra = min(ra, T - 1);
            rb = min(rb, T - 1);
        }
        const _Float16 *ka = kbase + (size_t)ra * kv_stride;
        const _Float16 *kb = kbase + (size_t)rb * kv_stride;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            fa[j] = *reinterpret_cast<const half8v *>(ka + 32 * j);
            fb[j] = *reinterpret_cast<const half8v *>(kb + 32 * j);
        }
    };
    // Two register sets for K fragments and for V rows give a prefetch distance of two key blocks:
    // a set is refilled for block b+2 as soon as block b has consumed it.
    u32x4 vreg0[2], vreg1[2];
    half8v k0a[4], k0b[4], k1a[4], k1b[4];
    float m_run = NEG_INF, l_run = 0.f;
    int cur = 0;
    auto block = [&](int blk, half8v (&kfa)[4], half8v (&kfb)[4], u32x4 (&v_store)[2], u32x4 (&v_load)[2]) {
        const int key0 = blk * kKeyBlock;
        const int ahead = blk + 2 < b1 ? blk + 2 : b1 - 1;   // clamped: loads stay unconditional
        __syncthreads();   // tile `cur` is complete; nobody still reads the other tile
        load_v(ahead, v_load);
        __builtin_amdgcn_sched_barrier(0);
        float4v sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            sa = __builtin_amdgcn_mfma_f32_16x16x32_f16(kfa[j], qf[j], sa, 0, 0, 0);
            sb = __builtin_amdgcn_mfma_f32_16x16x32_f16(kfb[j], qf[j], sb, 0, 0, 0);
        }
        load_k(ahead, kfa, kfb);   // the fragments just consumed make room for block blk + 2
        __builtin_amdgcn_sched_barrier(0);
        // lane (r, c): sa[i] = score of key key0 + 4r + i, sb[i] = key0 + 16 + 4r + i, query row my_row
        float s[8];
        if (key0 + kKeyBlock <= P) {   // uniform: a block of committed prefix keys, all visible
#pragma unroll
            for (int i = 0; i < 8; ++i) s[i] = ((i < 4) ? sa[i & 3] : sb[i & 3]) * scale_log2e;
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                int key = key0 + 4 * r + (i & 3) + (i >> 2) * 16;
                bool vis = key < P;
                if (!vis && key < T) vis = mask[(size_t)my_row * M + (key - P)] != 0;
                float raw = (i < 4) ? sa[i & 3] : sb[i & 3];
                s[i] = vis ? raw * scale_log2e : NEG_INF;
            }
        }
        float m_blk = s[0];
#pragma unroll
        for (int i = 1; i < 8; ++i) m_blk = fmaxf(m_blk, s[i]);
        m_blk = xor_max(m_blk, 16);
        m_blk = xor_max(m_blk, 32);
        float m_new = fmaxf(m_run, m_blk);
        float m_safe = (m_new == NEG_INF) ? 0.f : m_new;
        float alpha = __builtin_amdgcn_exp2f(m_run - m_safe);   // 0 when nothing was seen before
        float psum = 0.f;
        half8v pa;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            float p = __builtin_amdgcn_exp2f(s[i] - m_safe);
            psum += p;
            pa[i] = (_Float16)p;
        }
        psum += __shfl_xor(psum, 16, 64);
        psum += __shfl_xor(psum, 32, 64);
        l_run = l_run * alpha + psum;
        m_run = m_new;
        // accumulator rows are 4r + i: when some row's running maximum moved, fetch the rescale factors
        // from the lanes that own those rows (after the first few blocks this is rare)
        if (__any(alpha != 1.0f)) {
            float a_row[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a_row[i] = __shfl(alpha, 4 * r + i, 64);
#pragma unroll
            for (int dt = 0; dt < 8; ++dt)
#pragma unroll
                for (int i = 0; i < 4; ++i) o[dt][i] *= a_row[i];
        }
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
            // second operand: V[key slot][dt*16 + c], slots = keys 4r+p (tile a) and 16+4r+p (tile b)
            const _Float16 *rowp = &vt[cur][dt * 16 + c][0];
            u32x2 lo = *reinterpret_cast<const u32x2 *>(rowp + 4 * (r ^ dt));
            u32x2 hi = *reinterpret_cast<const u32x2 *>(rowp + 4 * ((4 + r) ^ dt));
            u32x4 both = {lo[0], lo[1], hi[0], hi[1]};
            o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(pa, __builtin_bit_cast(half8v, both), o[dt], 0, 0, 0);
        }
        store_v(cur ^ 1, v_store);   // V rows of block blk + 1, requested two blocks ago
        cur ^= 1;
    };
    if (b0 < b1) {
        load_v(b0, vreg0);
        load_k(b0, k0a, k0b);
        load_v(b0 + 1 < b1 ? b0 + 1 : b0, vreg1);
        load_k(b0 + 1 < b1 ? b0 + 1 : b0, k1a, k1b);
        store_v(0, vreg0);
    }
    for (int blk = b0; blk < b1; blk += 2) {
        block(blk, k0a, k0b, vreg1, vreg0);
        if (blk + 1 < b1) block(blk + 1, k1a, k1b, vreg0, vreg1);
    }

    // o[dt][i] belongs to query row row0 + 4r + i, column dt*16 + c
    float l_row[4], m_row[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        l_row[i] = __shfl(l_run, 4 * r + i, 64);
        m_row[i] = __shfl(m_run, 4 * r + i, 64);
    }
    // turn the fragment-ordered tile into rows: lane (r, c) owns rows 4r+i, columns dt*16+c
    const bool last = nsplit == 1;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float inv = last ? 1.f / l_row[i] : 1.f;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) ot[wave][4 * r + i][dt * 16 + c] = o[dt][i] * inv;
    }
    // (same wavefront writes and reads its own tile: LDS keeps program order, no barrier needed)
    float *po = part_o + (size_t)lid * kRowsPad * kHeadDim;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const int idx = u * 64 + lane, trow = idx >> 5, d4 = idx & 31;
        const int row = row0 + trow;
        if (row < M) {
            const float4v val = *reinterpret_cast<const float4v *>(&ot[wave][trow][d4 * 4]);
            if (last) {
                typedef _Float16 half4v __attribute__((ext_vector_type(4)));
                half4v hv = {(_Float16)val[0], (_Float16)val[1], (_Float16)val[2], (_Float16)val[3]};
                *reinterpret_cast<half4v *>(out + ((size_t)row * Hq + h) * kHeadDim + d4 * 4) = hv;
            } else {
                *reinterpret_cast<float4v *>(po + row * kHeadDim + d4 * 4) = val;
            }
        }
    }
    if (!last && c == 0) {
        // partial state of this key range: a second kernel merges the ranges (the kernel boundary
        // makes them visible, at no fence cost)
        float *pml = part_ml + (size_t)lid * kRowsPad * 2;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            pml[(row0 + 4 * r + i) * 2] = m_row[i];
            pml[(row0 + 4 * r + i) * 2 + 1] = l_row[i];
        }
    }
}

// merge of the key ranges: one thread per four consecutive output elements, ranges in order
__global__ __launch_bounds__(256) void tree_attn_merge_kernel(const float *__restrict__ part_o,
                                                              const float *__restrict__ part_ml,
                                                              _Float16 *__restrict__ out, int M, int Hq, int nsplit)
{
    const int idx = blockIdx.x * 256 + threadIdx.x;   // over M * Hq * 32 quads
    if (idx >= M * Hq * (kHeadDim / 4)) return;
    const int d4 = idx % (kHeadDim / 4), h = (idx / (kHeadDim / 4)) % Hq, row = idx / (kHeadDim / 4) / Hq;
    const float NEG_INF = -__builtin_inff();
    const float *hml = part_ml + (size_t)h * nsplit * kRowsPad * 2;
    const float4v *ho = reinterpret_cast<const float4v *>(part_o + (size_t)h * nsplit * kRowsPad * kHeadDim);
    float ms[kMaxSplits], ls[kMaxSplits];
    float4v os[kMaxSplits];
#pragma unroll
    for (int s = 0; s < kMaxSplits; ++s) {
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
    for (int s = 0; s < kMaxSplits; ++s) m_all = fmaxf(m_all, ms[s]);
    float den = 0.f;
    float4v num = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < kMaxSplits; ++s) {
        float wgt = (ms[s] == NEG_INF) ? 0.f : __builtin_amdgcn_exp2f(ms[s] - m_all);
        den += wgt * ls[s];
        num += wgt * os[s];
    }
    const float inv = 1.f / den;
    typedef _Float16 half4v __attribute__((ext_vector_type(4)));
    half4v hv = {(_Float16)(num[0] * inv), (_Float16)(num[1] * inv), (_Float16)(num[2] * inv), (_Float16)(num[3] * inv)};
    *reinterpret_cast<half4v *>(out + ((size_t)row * Hq + h) * kHeadDim + d4 * 4) = hv;
}

static int attn_splits(int M, int P, int Hq)
{
    int nblk = (P + M + kKeyBlock - 1) / kKeyBlock;
    int want = params().attn_splits > 0 ? params().attn_splits : (256 + Hq - 1) / Hq;   // about one workgroup per compute unit
    if (want > nblk) want = nblk;
    if (want > kMaxSplits) want = kMaxSplits;
    return want < 1 ? 1 : want;
}

static int check_attn(int M, int P, int Hq, int Hkv, int D)
{
    if (M < 1 || P < 0 || Hq < 1 || Hkv < 1 || D < 1) return W4A16_EINVAL;
    if (Hq % Hkv != 0) return W4A16_EINVAL;
    if (D != kHeadDim || M > W4A16_MAX_M || Hq > kMaxTickets) return W4A16_EUNSUP;
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
    if (!q || !k || !v || !mask || !out) return W4A16_ENULL;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(out) || misaligned(workspace)) return W4A16_EALIGN;
    const int ns = attn_splits(M, P, Hq);
    const size_t need = kTicketBytes + (size_t)Hq * ns * kRowsPad * (kHeadDim + 2) * sizeof(float);
    if (ns > 1 && (!workspace || workspace_bytes < need)) return W4A16_EWORKSPACE;
    float *part_o = reinterpret_cast<float *>(reinterpret_cast<uint8_t *>(workspace) + kTicketBytes);
    float *part_ml = part_o + (size_t)Hq * ns * kRowsPad * kHeadDim;
    const float scale_log2e = scale * 1.4426950408889634f;
    const int nblk = (P + M + kKeyBlock - 1) / kKeyBlock;
    hipLaunchKernelGGL(tree_attn_kernel, dim3((unsigned)(Hq * ns)), dim3(kAttnThreads), 0, (hipStream_t)stream,
                       (const _Float16 *)q, (const _Float16 *)k, (const _Float16 *)v, mask, (_Float16 *)out,
                       part_o, part_ml, M, P, Hq, Hkv, scale_log2e, ns, nblk / ns, nblk % ns);
    if (ns > 1) {
        const int quads = M * Hq * (kHeadDim / 4);
        hipLaunchKernelGGL(tree_attn_merge_kernel, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0,
                           (hipStream_t)stream, (const float *)part_o, (const float *)part_ml, (_Float16 *)out, M, Hq, ns);
    }
    return launch_status();
}

}  // extern "C"
