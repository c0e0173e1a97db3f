// rms_norm and rope_append: the small element-wise steps of a decoder layer that sit between the
// linears and the attention.  Contracts in include/w4a16.h.
#include "internal.h"

namespace w4 {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));

constexpr int kNormThreads = 1024;
constexpr int kNormChunks = 2;   // 16-byte chunks a thread can hold: K <= 1024 * 2 * 8 = 16384

// one workgroup per row: the row stays in registers between the sum of squares and the scaling;
// the norm weights are requested together with the row, so one memory round trip covers both
__global__ __launch_bounds__(kNormThreads) void rms_norm_kernel(const _Float16 *__restrict__ x,
                                                                const _Float16 *__restrict__ gamma,
                                                                _Float16 *__restrict__ y, int K, float eps)
{
    __shared__ float wave_sum[kNormThreads / 64];
    const int tid = threadIdx.x, m = blockIdx.x;
    const int chunks = K >> 3;
    const half8 *xr = reinterpret_cast<const half8 *>(x + (size_t)m * K);
    const half8 *gr = reinterpret_cast<const half8 *>(gamma);
    half8 v[kNormChunks], g[kNormChunks];
#pragma unroll
    for (int i = 0; i < kNormChunks; ++i) {
        const int ch = tid + kNormThreads * i;
        if (ch < chunks) {
            v[i] = xr[ch];
            g[i] = gr[ch];
        }
    }
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < kNormChunks; ++i) {
        if (tid + kNormThreads * i < chunks) {
#pragma unroll
            for (int e = 0; e < 8; ++e) ss = fmaf((float)v[i][e], (float)v[i][e], ss);
        }
    }
    // fixed-order sum: butterfly inside the wavefront, then the wavefront sums in order
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
    if ((tid & 63) == 0) wave_sum[tid >> 6] = ss;
    __syncthreads();
    float total = 0.f;
#pragma unroll
    for (int w = 0; w < kNormThreads / 64; ++w) total += wave_sum[w];
    const float r = 1.0f / sqrtf(total / (float)K + eps);
    half8 *yr = reinterpret_cast<half8 *>(y + (size_t)m * K);
#pragma unroll
    for (int i = 0; i < kNormChunks; ++i) {
        const int ch = tid + kNormThreads * i;
        if (ch < chunks) {
            half8 o;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = (_Float16)((float)v[i][e] * r * (float)g[i][e]);
            yr[ch] = o;
        }
    }
}

// one workgroup per row: thread t owns the element pair (i, i + D/2), i = t % (D/2), of the heads
// t / (D/2), t / (D/2) + heads_per_pass, ...; its table entry is fetched once and serves every head.
// The general form (any even D, tables at any 4-byte alignment).
constexpr int kRopeThreads = 1024;
__global__ __launch_bounds__(kRopeThreads) void rope_append_scalar_kernel(
    const _Float16 *__restrict__ qkv, const int32_t *__restrict__ pos, const float *__restrict__ cos_t,
    const float *__restrict__ sin_t, int n_pos, _Float16 *__restrict__ q, _Float16 *__restrict__ k_cache,
    _Float16 *__restrict__ v_cache, int P, int Hq, int Hkv, int D)
{
    const int m = blockIdx.x, h = D >> 1;
    const int heads_per_pass = kRopeThreads / h;
    const int i = threadIdx.x % h, slot = threadIdx.x / h;
    if (slot >= heads_per_pass) return;
    const int heads = Hq + 2 * Hkv;
    const int p = pos[m];
    const bool in_table = p >= 0 && p < n_pos;   // otherwise this row's q and k are left untouched
    const float c = in_table ? cos_t[(size_t)p * h + i] : 0.f, s = in_table ? sin_t[(size_t)p * h + i] : 0.f;
    for (int head = slot; head < heads; head += heads_per_pass) {
        const _Float16 *src = qkv + ((size_t)m * heads + head) * D;
        if (head >= Hq + Hkv) {   // value head: plain copy into the cache
            _Float16 *dst = v_cache + ((size_t)(P + m) * Hkv + (head - Hq - Hkv)) * D;
            dst[i] = src[i];
            dst[i + h] = src[i + h];
        } else if (in_table) {
            const float lo = (float)src[i], hi = (float)src[i + h];
            _Float16 *dst = head < Hq ? q + ((size_t)m * Hq + head) * D : k_cache + ((size_t)(P + m) * Hkv + (head - Hq)) * D;
            dst[i] = (_Float16)keep_f32(fmaf(lo, c, -hi * s));
            dst[i + h] = (_Float16)keep_f32(fmaf(hi, c, lo * s));
        }
    }
}

// The form for D % 8 == 0 and 16-byte-aligned tables (every model shape): a thread owns four consecutive
// pairs (i .. i+3, i + D/2 ..), so D/8 threads cover a head and the workgroup covers 8192 / D heads per
// pass.  The kernel is a chain of memory round trips and little else, so it is arranged to have as few
// as possible in a row: all arguments in one batch of scalar loads, then the row's position, and -- not
// waiting for it -- the data of up to kRopePasses passes; then the table entry; then the stores.  The
// arithmetic per element is that of the general form.
constexpr int kRopePasses = 4;
__global__ __launch_bounds__(kRopeThreads) void rope_append_kernel(
    const _Float16 *__restrict__ qkv, const int32_t *__restrict__ pos, const float *__restrict__ cos_t,
    const float *__restrict__ sin_t, int n_pos, _Float16 *__restrict__ q, _Float16 *__restrict__ k_cache,
    _Float16 *__restrict__ v_cache, int P, int Hq, int Hkv, int D)
{
    fetch_arguments_together(qkv, pos, cos_t, sin_t, n_pos, q, k_cache, v_cache, P, Hq, Hkv, D);
    typedef _Float16 half4 __attribute__((ext_vector_type(4)));
    typedef float float4 __attribute__((ext_vector_type(4)));
    const int m = blockIdx.x, h = D >> 1;
    const int lanes = h >> 2;   // threads per head
    const int heads_per_pass = kRopeThreads / lanes;
    const int i = (threadIdx.x % lanes) * 4, slot = threadIdx.x / lanes;
    if (slot >= heads_per_pass) return;
    const int heads = Hq + 2 * Hkv;
    const int p = pos[m];
    const bool in_table = p >= 0 && p < n_pos;   // otherwise this row's q and k are left untouched
    float4 c = {0.f, 0.f, 0.f, 0.f}, s = c;
    bool have_table = false;
    for (int head0 = slot; head0 < heads; head0 += heads_per_pass * kRopePasses) {
        half4 lo[kRopePasses], hi[kRopePasses];
#pragma unroll
        for (int u = 0; u < kRopePasses; ++u) {
            const int head = head0 + u * heads_per_pass;
            if (head < heads) {
                const _Float16 *src = qkv + ((size_t)m * heads + head) * D;
                lo[u] = *reinterpret_cast<const half4 *>(src + i);
                hi[u] = *reinterpret_cast<const half4 *>(src + i + h);
            }
        }
        if (in_table && !have_table) {
            c = *reinterpret_cast<const float4 *>(cos_t + (size_t)p * h + i);
            s = *reinterpret_cast<const float4 *>(sin_t + (size_t)p * h + i);
            have_table = true;
        }
#pragma unroll
        for (int u = 0; u < kRopePasses; ++u) {
            const int head = head0 + u * heads_per_pass;
            if (head >= heads) break;
            if (head >= Hq + Hkv) {   // value head: plain copy into the cache
                _Float16 *dst = v_cache + ((size_t)(P + m) * Hkv + (head - Hq - Hkv)) * D;
                *reinterpret_cast<half4 *>(dst + i) = lo[u];
                *reinterpret_cast<half4 *>(dst + i + h) = hi[u];
            } else if (in_table) {
                _Float16 *dst = head < Hq ? q + ((size_t)m * Hq + head) * D : k_cache + ((size_t)(P + m) * Hkv + (head - Hq)) * D;
                half4 olo, ohi;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float a = (float)lo[u][e], b = (float)hi[u][e];
                    olo[e] = (_Float16)keep_f32(fmaf(a, c[e], -b * s[e]));
                    ohi[e] = (_Float16)keep_f32(fmaf(b, c[e], a * s[e]));
                }
                *reinterpret_cast<half4 *>(dst + i) = olo;
                *reinterpret_cast<half4 *>(dst + i + h) = ohi;
            }
        }
    }
}

}  // namespace w4

using namespace w4;

extern "C" {

int rms_norm(const void *x, const void *gamma, void *y, int M, int K, float eps, void *stream)
{
    if (M < 1 || K < 8 || K % 8 != 0 || !(eps >= 0.f)) return W4A16_EINVAL;
    if (M > 65535) return W4A16_EUNSUP;
    if (K > kNormThreads * kNormChunks * 8) return W4A16_EUNSUP;
    if (!x || !gamma || !y) return W4A16_ENULL;
    if (misaligned(x) || misaligned(gamma) || misaligned(y)) return W4A16_EALIGN;
    hipLaunchKernelGGL(rms_norm_kernel, dim3((unsigned)M), dim3(kNormThreads), 0, (hipStream_t)stream,
                       (const _Float16 *)x, (const _Float16 *)gamma, (_Float16 *)y, K, eps);
    return launch_status();
}

int rope_append(const void *qkv, const int32_t *pos, const float *cos_table, const float *sin_table, int n_pos,
                void *q, void *k_cache, void *v_cache, int M, int P, int Hq, int Hkv, int D, void *stream)
{
    if (M < 1 || P < 0 || Hq < 1 || Hkv < 1 || D < 2 || D % 2 != 0 || n_pos < 1) return W4A16_EINVAL;
    if (M > 65535 || D > 2 * kRopeThreads) return W4A16_EUNSUP;
    if (!qkv || !pos || !cos_table || !sin_table || !q || !k_cache || !v_cache) return W4A16_ENULL;
    if (misaligned(qkv) || misaligned(q) || misaligned(k_cache) || misaligned(v_cache)) return W4A16_EALIGN;
    if ((reinterpret_cast<uintptr_t>(pos) & 3u) || (reinterpret_cast<uintptr_t>(cos_table) & 3u) ||
        (reinterpret_cast<uintptr_t>(sin_table) & 3u))
        return W4A16_EALIGN;
    const bool wide = D % 8 == 0 && !misaligned(cos_table) && !misaligned(sin_table);
    hipLaunchKernelGGL(wide ? rope_append_kernel : rope_append_scalar_kernel, dim3((unsigned)M), dim3(kRopeThreads), 0,
                       (hipStream_t)stream, (const _Float16 *)qkv, pos, cos_table, sin_table, n_pos, (_Float16 *)q,
                       (_Float16 *)k_cache, (_Float16 *)v_cache, P, Hq, Hkv, D);
    return launch_status();
}

}  // extern "C"

// ---- one decoder layer as one call: host glue over the entry points above and in the other files ----

extern "C" int w4a16_decoder_layer(const w4a16_layer_weights *w, void *h, int M, int P, const int32_t *pos,
                                   const float *cos_table, const float *sin_table, int n_pos, const uint8_t *mask,
                                   void *k_cache, void *v_cache, const w4a16_layer_scratch *s, void *stream)
{
    if (!w || !s) return W4A16_ENULL;
    const int H = w->hidden, Hq = w->n_q_heads, Hkv = w->n_kv_heads, D = w->head_dim, F = w->ffn;
    if (H < 1 || Hq < 1 || Hkv < 1 || D < 1 || F < 1 || M < 1 || P < 0) return W4A16_EINVAL;
    if (!w->qkv_packed || !w->o_packed || !w->gate_up_packed || !w->down_packed || !w->norm1_gamma || !w->norm2_gamma)
        return W4A16_ENULL;
    if (!h || !s->norm || (!s->qkv && !w->qkv_heads_packed) || !s->q || !s->attn || !s->act) return W4A16_ENULL;
    const int Nqkv = (Hq + 2 * Hkv) * D;
    const float scale = 1.0f / sqrtf((float)D);
    const int sym = w->symmetric ? W4A16_SYMMETRIC : 0;
    int rc;
    // attention block: h += Wo . attn(rope(Wqkv . norm(h)))
    if ((rc = rms_norm(h, w->norm1_gamma, s->norm, M, H, w->eps, stream)) != W4A16_OK) return rc;
    if (w->qkv_heads_packed) {   // projection, rotary embedding and K/V append in one kernel
        if ((rc = w4::gemm_rope(s->norm, w->qkv_packed, M, H, kGroup, pos, cos_table, sin_table, n_pos, s->q, k_cache, v_cache,
                                P, Hq, Hkv, D, s->gemm_workspace, s->gemm_workspace_bytes, stream, w->symmetric)) != W4A16_OK)
            return rc;
    } else {
        if ((rc = w4a16_gemm_fused(s->norm, w->qkv_packed, s->qkv, M, Nqkv, H, kGroup, W4A16_EPI_NONE | sym, nullptr,
                                   s->gemm_workspace, s->gemm_workspace_bytes, stream)) != W4A16_OK)
            return rc;
        if ((rc = rope_append(s->qkv, pos, cos_table, sin_table, n_pos, s->q, k_cache, v_cache, M, P, Hq, Hkv, D, stream)) !=
            W4A16_OK)
            return rc;
    }
    if ((rc = tree_verify_attn(s->q, k_cache, v_cache, mask, s->attn, M, P, Hq, Hkv, D, scale, s->attn_workspace,
                               s->attn_workspace_bytes, stream)) != W4A16_OK)
        return rc;
    if ((rc = w4a16_gemm_fused(s->attn, w->o_packed, h, M, H, Hq * D, kGroup, W4A16_EPI_RESIDUAL | sym, h, s->gemm_workspace,
                               s->gemm_workspace_bytes, stream)) != W4A16_OK)
        return rc;
    // feed-forward block: h += Wdown . (silu(Wgate . n) * (Wup . n)),  n = norm(h)
    if ((rc = rms_norm(h, w->norm2_gamma, s->norm, M, H, w->eps, stream)) != W4A16_OK) return rc;
    if ((rc = w4a16_gemm_fused(s->norm, w->gate_up_packed, s->act, M, 2 * F, H, kGroup, W4A16_EPI_SILU_MUL | sym, nullptr,
                               s->gemm_workspace, s->gemm_workspace_bytes, stream)) != W4A16_OK)
        return rc;
    return w4a16_gemm_fused(s->act, w->down_packed, h, M, H, F, kGroup, W4A16_EPI_RESIDUAL | sym, h, s->gemm_workspace,
                            s->gemm_workspace_bytes, stream);
}
