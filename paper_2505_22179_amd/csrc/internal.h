// Host-side helpers shared by the entry points (argument checks, launch error mapping, knobs).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/w4a16.h"
#include "layout.h"

namespace w4 {

inline bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }
// workspaces: 256 bytes, so that the partial-sum region of one workgroup never shares a cache line with
// another's -- the exchange of partials inside a kernel goes through device-scope accesses line by line
inline bool workspace_misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 255u) != 0; }

// shape checks common to every weight entry point; returns W4A16_OK or an error code
inline int check_weight_shape(int N, int K, int G)
{
    if (N <= 0 || K <= 0 || G <= 0) return W4A16_EINVAL;
    if (K % G != 0 || N % 8 != 0) return W4A16_EINVAL;
    if (G != kGroup) return W4A16_EUNSUP;
    if ((long long)pad_cols(N) / kBlockCols * (K / kGroup) > (1ll << 30)) return W4A16_EUNSUP;
    return W4A16_OK;
}

// Device side: makes the compiler fetch the named kernel arguments (uniform values) in ONE batch of scalar
// loads where this is called -- the top of a kernel.  Left alone it fetches arguments block by block where
// they are first used; in a short kernel that is several dependent round trips to the argument buffer, a
// good part of a microsecond each, ahead of the first useful memory request.
template <typename... T>
__device__ __forceinline__ void fetch_arguments_together(const T &...args)
{
    (..., [](const T &a) { asm volatile("" ::"s"(a)); }(args));
}

// An fp32 value the compiler must materialise as such.  Without it a following conversion to fp16 may or may
// not be folded into the multiply-add that produced the value (one rounding instead of two), kernel by kernel:
// the rotary arithmetic exists in three kernels that have to agree bit for bit.
__device__ __forceinline__ float keep_f32(float v)
{
    asm volatile("" : "+v"(v));
    return v;
}

inline int launch_status()
{
    return hipGetLastError() == hipSuccess ? W4A16_OK : W4A16_EHIP;
}

struct Params {
    int split_k = 0;       // 0 = heuristic
    int fused_reduce = 2;  // 0 = second kernel, 1 = last workgroup, 2 = per-shape choice
    int attn_splits = 0;   // 0 = heuristic
    int attn_row_tiles = 0;   // 0 = the kernel with K/V tiles shared through LDS; the older kernel: 2 = 32 query rows per wavefront (two row groups for taller tiles), 4 = 64 rows
    int lm_tiles = 0;         // 0 = by M, else 1 or 2 vocabulary tiles per wavefront in lm_head_topk
    int attn_pack = 0;     // query heads of a KV group per row tile: 0 = by size, 1 = one, 2 = the whole group when it fits
    int attn_fused_merge = 0;   // 2 = the last workgroup of a tile merges its key ranges, 1 = a second kernel does, 0 = by size
    int tiles_per_wave = 0;   // 0 = heuristic, else 2, 4 or 8
    int waves_per_wg = 0;     // 0 = heuristic, else 4, 8 or 16
    int prefetch_depth = 0;   // 0 = heuristic, else 1, 2, 3 or 4
    int k_sets = 0;           // 0 = heuristic, else 1..3: force the high-occupancy column-split kernel
    int even_split = 0;       // 1 with k_sets: deal (unit, group) pairs evenly to one workgroup per compute unit
    int flat_groups = 0;      // 0 = heuristic, else 4, 7 or 8: force the all-loads-up-front kernel (M <= 4)
};
Params &params();

// w4a16_gemm_rope with the caller's word that the weight is symmetric (the exported entry point passes 0)
int gemm_rope(const void *x, const void *packed, int M, int K, int G, const int32_t *pos, const float *cos_table,
              const float *sin_table, int n_pos, void *q, void *k_cache, void *v_cache, int P, int Hq, int Hkv, int D,
              void *workspace, size_t workspace_bytes, void *stream, int symmetric);

// number of 256-byte-aligned bytes reserved for tickets at the start of a workspace
constexpr size_t kTicketBytes = 16384;   // 4096 tickets
constexpr int kMaxTickets = 4096;

}  // namespace w4
