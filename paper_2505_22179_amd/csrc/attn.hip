// tree_verify_attn: attention of the tree-verification pass (paper section 2.1) on gfx950.
//
// One workgroup handles one query head and one contiguous range of keys; each of its four
// wavefronts owns a 16-row tile of the (at most 64) draft-token query rows.  Scores are computed
// transposed, S^T = K . Q^T, with 16x16x32 fp16 MFMA steps over the head dimension, so that a lane
// ends up with eight scores of ONE query row (keys 4r..4r+3 of two 16-key tiles): exactly the
// first-operand fragment the P.V product needs, with no shuffle in between.  The tree mask is
// applied to the draft keys, softmax runs online in fp32 (base-2 exponentials), and V reaches the
// second MFMA operand through a small LDS tile because the contraction there runs over keys while
// V is stored with the head dimension contiguous.  Key ranges are combined by the last workgroup
// of a head to finish, in split order, so the result does not depend on scheduling.
#include "internal.h"

namespace w4 {

typedef _Float16 half8v __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kHeadDim = 128;
constexpr int kKeyBlock = 32;
constexpr int kVStride = 132;   // halves per LDS row of V (264 B): the four 16-lane groups hit disjoint banks
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
    float *__restrict__ part_ml, uint32_t *__restrict__ tickets, int M, int P, int Hq, int Hkv,
    float scale_log2e, int nsplit)
{
    __shared__ _Float16 vs[4][kKeyBlock][kVStride];
    __shared__ uint32_t ticket_sh;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane >> 4, c = lane & 15;
    const int h = blockIdx.x / nsplit, sp = blockIdx.x % nsplit;
    const int kvh = h / (Hq / Hkv);
    const int T = P + M;
    const int nblk = (T + kKeyBlock - 1) / kKeyBlock;
    const int b0 = (int)((long long)nblk * sp / nsplit), b1 = (int)((long long)nblk * (sp + 1) / nsplit);
    const int row0 = wave * 16;
    const int my_row = min(row0 + c, M - 1);   // rows >= M repeat row M-1 and are never stored
    const size_t kv_stride = (size_t)Hkv * kHeadDim;
    const float NEG_INF = -__builtin_inff();

    // Q^T fragment (second operand): lane (r, c) holds q[my_row, h, 32 j + 8 r .. +7]
    half8v qf[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
        qf[j] = *reinterpret_cast<const half8v *>(q + ((size_t)my_row * Hq + h) * kHeadDim + 32 * j + 8 * r);

    float m_run = NEG_INF, l_run = 0.f;
    float4v o[8];
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) o[dt] = (float4v){0.f, 0.f, 0.f, 0.f};

    for (int blk = b0; blk < b1; ++blk) {
        const int key0 = blk * kKeyBlock;
        // stage this block's V rows (32 keys x 256 B) into the wavefront's LDS tile
        __syncthreads();   // previous block's readers are done
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            int idx = u * 64 + lane;
            int key = idx >> 4, chunk = idx & 15;
            int src = min(key0 + key, T - 1);
            u32x4 d = *reinterpret_cast<const u32x4 *>(v + (size_t)src * kv_stride + kvh * kHeadDim + chunk * 8);
            u32x2 *dst = reinterpret_cast<u32x2 *>(&vs[wave][key][chunk * 8]);
            dst[0] = (u32x2){d[0], d[1]};
            dst[1] = (u32x2){d[2], d[3]};
        }
        // S^T tiles: first operand = K rows (tile a: keys key0 + 0..15, tile b: key0 + 16..31)
        float4v sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
        const _Float16 *ka = k + (size_t)min(key0 + c, T - 1) * kv_stride + kvh * kHeadDim + 8 * r;
        const _Float16 *kb = k + (size_t)min(key0 + 16 + c, T - 1) * kv_stride + kvh * kHeadDim + 8 * r;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            half8v fa = *reinterpret_cast<const half8v *>(ka + 32 * j);
            half8v fb = *reinterpret_cast<const half8v *>(kb + 32 * j);
            sa = __builtin_amdgcn_mfma_f32_16x16x32_f16(fa, qf[j], sa, 0, 0, 0);
            sb = __builtin_amdgcn_mfma_f32_16x16x32_f16(fb, qf[j], sb, 0, 0, 0);
        }
        // lane (r, c): sa[i] = score of key key0 + 4r + i, sb[i] = key0 + 16 + 4r + i, query row my_row
        float s[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            int key = key0 + 4 * r + (i & 3) + (i >> 2) * 16;
            bool vis = key < P;
            if (!vis && key < T) vis = mask[(size_t)my_row * M + (key - P)] != 0;
            float raw = (i < 4) ? sa[i & 3] : sb[i & 3];
            s[i] = vis ? raw * scale_log2e : NEG_INF;
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
        // accumulator rows are 4r + i: fetch their rescale factors from the lanes that own those rows
        float a_row[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) a_row[i] = __shfl(alpha, 4 * r + i, 64);
        __syncthreads();   // V tile written
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
            half8v vb;   // second operand: V[key slot][dt*16 + c], slots = keys 4r+p and 16+4r+p
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                vb[p] = vs[wave][4 * r + p][dt * 16 + c];
                vb[4 + p] = vs[wave][16 + 4 * r + p][dt * 16 + c];
            }
            float4v acc = o[dt];
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i] *= a_row[i];
            o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(pa, vb, acc, 0, 0, 0);
        }
    }

    // o[dt][i] belongs to query row row0 + 4r + i, column dt*16 + c
    float l_row[4], m_row[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        l_row[i] = __shfl(l_run, 4 * r + i, 64);
        m_row[i] = __shfl(m_run, 4 * r + i, 64);
    }
    if (nsplit == 1) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int row = row0 + 4 * r + i;
            if (row < M) {
                float inv = 1.f / l_row[i];
#pragma unroll
                for (int dt = 0; dt < 8; ++dt)
                    out[((size_t)row * Hq + h) * kHeadDim + dt * 16 + c] = (_Float16)(o[dt][i] * inv);
            }
        }
        return;
    }
    // partial state of this key range: unnormalised output rows plus (running max, running sum).
    // Stored with device-scope accesses so that the workgroup that merges the ranges, possibly on
    // another XCD, reads them without any whole-cache write-back or invalidate.
    float *po = part_o + (size_t)blockIdx.x * kRowsPad * kHeadDim;
    float *pml = part_ml + (size_t)blockIdx.x * kRowsPad * 2;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int row = row0 + 4 * r + i;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt)
            __hip_atomic_store(po + row * kHeadDim + dt * 16 + c, o[dt][i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (c == 0) {
            __hip_atomic_store(pml + row * 2, m_row[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(pml + row * 2 + 1, l_row[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0) ticket_sh = __hip_atomic_fetch_add(&tickets[h], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (ticket_sh != (uint32_t)(nsplit - 1)) return;
    // last workgroup of this head: merge the ranges in order.  Weights first (through LDS), then rows.
    float *wgt = reinterpret_cast<float *>(&vs[0][0][0]);   // [nsplit][64] merge weights, reuses the V tiles
    const float *hml = part_ml + (size_t)h * nsplit * kRowsPad * 2;
    const float *ho = part_o + (size_t)h * nsplit * kRowsPad * kHeadDim;
    if (tid < kRowsPad) {
        float ms[kMaxSplits], ls[kMaxSplits];
#pragma unroll
        for (int s2 = 0; s2 < kMaxSplits; ++s2) {
            ms[s2] = NEG_INF;
            ls[s2] = 0.f;
            if (s2 < nsplit) {
                ms[s2] = __hip_atomic_load(hml + ((size_t)s2 * kRowsPad + tid) * 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                ls[s2] = __hip_atomic_load(hml + ((size_t)s2 * kRowsPad + tid) * 2 + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        float m_all = NEG_INF;
#pragma unroll
        for (int s2 = 0; s2 < kMaxSplits; ++s2) m_all = fmaxf(m_all, ms[s2]);
        float den = 0.f;
#pragma unroll
        for (int s2 = 0; s2 < kMaxSplits; ++s2) {
            ms[s2] = (ms[s2] == NEG_INF) ? 0.f : __builtin_amdgcn_exp2f(ms[s2] - m_all);
            den += ms[s2] * ls[s2];
        }
        float inv = 1.f / den;
#pragma unroll
        for (int s2 = 0; s2 < kMaxSplits; ++s2)
            if (s2 < nsplit) wgt[s2 * kRowsPad + tid] = ms[s2] * inv;
    }
    __syncthreads();
    for (int e = tid; e < M * kHeadDim; e += kAttnThreads) {
        int row = e / kHeadDim, d = e % kHeadDim;
        float part[kMaxSplits];
#pragma unroll
        for (int s2 = 0; s2 < kMaxSplits; ++s2) {
            part[s2] = 0.f;
            if (s2 < nsplit)
                part[s2] = __hip_atomic_load(ho + ((size_t)s2 * kRowsPad + row) * kHeadDim + d, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        float num = 0.f;
#pragma unroll
        for (int s2 = 0; s2 < kMaxSplits; ++s2)
            if (s2 < nsplit) num += wgt[s2 * kRowsPad + row] * part[s2];
        out[((size_t)row * Hq + h) * kHeadDim + d] = (_Float16)num;
    }
    if (tid == 0) __hip_atomic_store(&tickets[h], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

static int attn_splits(int M, int P, int Hq)
{
    int nblk = (P + M + kKeyBlock - 1) / kKeyBlock;
    int want = params().attn_splits > 0 ? params().attn_splits : (512 + Hq - 1) / Hq;
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
    uint32_t *tickets = reinterpret_cast<uint32_t *>(workspace);
    float *part_o = reinterpret_cast<float *>(reinterpret_cast<uint8_t *>(workspace) + kTicketBytes);
    float *part_ml = part_o + (size_t)Hq * ns * kRowsPad * kHeadDim;
    const float scale_log2e = scale * 1.4426950408889634f;
    hipLaunchKernelGGL(tree_attn_kernel, dim3((unsigned)(Hq * ns)), dim3(kAttnThreads), 0, (hipStream_t)stream,
                       (const _Float16 *)q, (const _Float16 *)k, (const _Float16 *)v, mask, (_Float16 *)out,
                       part_o, part_ml, tickets, M, P, Hq, Hkv, scale_log2e, ns);
    return launch_status();
}

}  // extern "C"
