/*
 * libw4a16 -- C ABI of the MI355X (gfx950) W4A16 small-M linear layer and tree-verify attention.
 *
 * The computation is the group-wise 4-bit-weight / 16-bit-activation linear layer of a quantised
 * target model (paper section 2.2, "W4A16": 4-bit weights, group size 128, fp16 activations) run
 * at the token counts speculative decoding produces (paper section 2.1: M = 1 for plain decoding,
 * M = draft length + 1 for a sequence draft, M = tree size n for a tree draft), plus the attention
 * of the tree-verification pass.
 *
 * Conventions that hold for every entry point unless stated otherwise
 *   - every pointer is a DEVICE pointer owned by the caller; the library never allocates, frees,
 *     retains or synchronises on caller memory;
 *   - fp16 buffers are passed as `const void*` / `void*` (IEEE binary16, row-major);
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream); the work is enqueued
 *     on it and the call returns without waiting;
 *   - the return value is W4A16_OK or a negative W4A16_E* code; arguments are validated before any
 *     GPU call, so an invalid call enqueues nothing; nothing is printed, nothing aborts;
 *   - all pointers must be 16-byte aligned; buffers must not overlap;
 *   - the same inputs give bit-identical outputs on every call (no atomically ordered sums);
 *   - one GPU per process: the library keeps a few process-wide one-time flags (kernel attributes
 *     set on first use) and the ablation knobs; calls may be issued from any one host thread at a
 *     time, on any stream of the current device.
 */
#ifndef W4A16_H
#define W4A16_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define W4A16_OK 0
#define W4A16_EINVAL (-1)     /* bad shape or argument value */
#define W4A16_ENULL (-2)      /* a required pointer is NULL */
#define W4A16_EALIGN (-3)     /* a pointer is not 16-byte aligned */
#define W4A16_EUNSUP (-4)     /* valid but not implemented (group size other than 128, M > 64, ...) */
#define W4A16_EWORKSPACE (-5) /* workspace missing or smaller than the *_workspace_bytes() value (or than the built-in scratch) */
#define W4A16_EHIP (-6)       /* the HIP runtime reported an error while enqueuing */

#define W4A16_MAX_M 64

/* Library version, major*10000 + minor*100 + patch. */
int w4a16_version(void);

/* Static, NUL-terminated description of a return code. */
const char *w4a16_strerror(int code);

/* Size in bytes of the opaque packed weight buffer for an N-column, K-row weight with group size G
 * (it holds the 4-bit codes, the fp16 scales and the 4-bit zero-points; columns are padded up to a
 * multiple of 128 inside the buffer).  0 if the shape is not supported. */
size_t w4a16_packed_bytes(int N, int K, int G);

/* Bytes of scratch w4a16_gemm may need for any 1 <= M <= M_max at this shape (split-K partial sums
 * and their tickets).  Never 0 for a supported shape. */
size_t w4a16_workspace_bytes(int M_max, int N, int K, int G);

/* Zero the ticket area at the start of a workspace.  Must be enqueued once before the first
 * w4a16_gemm / tree_verify_attn that uses the buffer; each of those calls leaves the tickets zero
 * again, so one initialisation serves any number of later calls (of any shape that fits).  Two
 * calls that may run concurrently must not share a workspace.  A workspace must be 256-byte aligned
 * (W4A16_EALIGN otherwise): workgroups exchange partial sums through it inside a kernel, cache line by
 * cache line, and no line may belong to two of them. */
int w4a16_workspace_init(void *workspace, size_t workspace_bytes, void *stream);

/* Re-lay the canonical quantised weight into the streaming layout the GEMM kernels read
 * (paper section 2.2 fixes the scheme -- 4-bit codes, one scale and one zero-point per group of
 * 128 rows per column; the canonical storage is
 *   qweight int32 [K/8, N]   code of row k in bits 4*(k%8)..4*(k%8)+3 of word [k/8, n]
 *   scales  fp16  [K/G, N]
 *   qzeros  int32 [K/G, N/8] zero-point of column n in bits 4*(n%8)..+3 of word [g, n/8]).
 * `packed` receives w4a16_packed_bytes(N, K, G) bytes.  Requires G == 128, K % 128 == 0,
 * N % 8 == 0.  Exactly invertible by w4a16_unpack. */
int w4a16_pack(const int32_t *qweight, const void *scales, const int32_t *qzeros, void *packed,
               int N, int K, int G, void *stream);

/* Exact inverse of w4a16_pack: recovers the three canonical tensors bit for bit. */
int w4a16_unpack(const void *packed, int32_t *qweight, void *scales, int32_t *qzeros,
                 int N, int K, int G, void *stream);

/* Test export: dequantise the packed weight to a dense fp32 matrix W [K, N] row-major,
 * W[k,n] = (float)(q[k,n] - z[k/G,n]) * (float)s[k/G,n].  The product is exact in fp32, so the
 * result is defined bit for bit. */
int w4a16_dequant(const void *packed, float *W, int N, int K, int G, void *stream);

/* y[M,N] (fp16) = x[M,K] (fp16) . dequant(packed)[K,N], accumulated in fp32 and rounded to fp16
 * with round-to-nearest-even (paper section 2.2 for the layer; section 2.1 and the verification
 * analysis of section 3 for the values of M).  1 <= M <= 64; rows >= M of x and y are never
 * touched; y is overwritten.  `workspace` must hold w4a16_workspace_bytes(M, N, K, G) bytes and
 * have been initialised with w4a16_workspace_init.
 * No restriction on the size of the activations: every operand of the matrix instruction is exact in fp16
 * and products and sums are fp32, so rows of tiny or of large entries keep the same relative accuracy. */
int w4a16_gemm(const void *x, const void *packed, void *y, int M, int N, int K, int G,
               void *workspace, size_t workspace_bytes, void *stream);

/* w4a16_gemm for callers that cannot allocate device memory and so cannot provide a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same computation, same kernels,
 * same results bit for bit; the split-K partial sums and tickets live in a scratch array built into the
 * library (16 KB of tickets + 32 MiB of partial sums, held on every GPU the library is loaded on until the
 * process ends).  The call allocates nothing and frees nothing.  W4A16_EWORKSPACE if the launch plan of this
 * (M, N, K) needs more partial-sum space than the array holds (no Llama-3 8B / 70B layer shape does); all
 * other errors as w4a16_gemm.  Every call on a GPU shares that GPU's array: two calls that may run at the same
 * time on one GPU (different streams, different host threads) race and must not be issued; calls ordered on
 * one stream are safe.  The first call on a GPU looks up the array's address and is not thread-safe. */
int w4a16_gemm_static(const void *x, const void *packed, void *y, int M, int N, int K, int G, void *stream);

/* w4a16_gemm with the element-wise step that follows the linear in a Llama-type decoder layer fused
 * into the store (paper section 2.1 counts a whole forward pass of the target model per
 * verification; its layer is h += Wo.attn(..), h += Wdown.(silu(Wgate.n) * Wup.n), so every linear
 * is followed by a residual add or by the gate):
 *   W4A16_EPI_NONE      y[M,N]   = x . W                       (identical to w4a16_gemm)
 *   W4A16_EPI_RESIDUAL  y[M,N]   = residual[M,N] + x . W       residual fp16, 16-byte aligned; it
 *                                  may be y itself (in place), no other overlap is allowed
 *   W4A16_EPI_SILU_MUL  y[M,N/2] = silu(x . Wgate) * (x . Wup), silu(t) = t / (1 + exp(-t)); `packed`
 *                                  must come from w4a16_pack_gate_up, N % 32 == 0
 * The sum, the residual add and the gate are evaluated in fp32 and rounded to fp16 once.
 * `residual` must be NULL unless the epilogue is W4A16_EPI_RESIDUAL.  Everything else as for
 * w4a16_gemm (same workspace size).
 *
 * W4A16_SYMMETRIC may be OR-ed into `epilogue`: the caller vouches that every zero-point of this weight is 8,
 * i.e. that the weight is symmetrically quantised (the scheme of paper section 2.2: GPTQ, symmetric, group size
 * 128).  The kernels then use w = (q - 8) * s without reading the zero-points -- fewer bytes and instructions;
 * for such a weight the result is that of the call without the flag (bit for bit for M > 16; for M <= 16 the
 * fp32 sums are formed in another order, and exact-arithmetic inputs still give identical bits).  Kernel families
 * without a symmetric instantiation ignore the flag, so for a weight that has other zero-points the result is
 * unspecified: either the correct one or that of zero-points 8.  w4a16_weight_is_symmetric tests a packed weight. */
#define W4A16_EPI_NONE 0
#define W4A16_EPI_RESIDUAL 1
#define W4A16_EPI_SILU_MUL 2
#define W4A16_SYMMETRIC 0x100
int w4a16_gemm_fused(const void *x, const void *packed, void *y, int M, int N, int K, int G, int epilogue,
                     const void *residual, void *workspace, size_t workspace_bytes, void *stream);

/* Writes 1 to *flag (device int32, 4-byte aligned) if every zero-point of the N columns of a packed weight is 8,
 * else 0 -- what a loader checks once before it passes W4A16_SYMMETRIC for that weight (padding columns inside
 * the buffer do not count; the paired packings of w4a16_pack_gate_up / w4a16_pack_heads only permute columns).
 * Enqueued on `stream`; read the flag after synchronising. */
int w4a16_weight_is_symmetric(const void *packed, int N, int K, int G, int32_t *flag, void *stream);

/* w4a16_pack for a weight whose columns 0..N/2-1 are a gate projection and N/2..N-1 the matching up
 * projection: the packed buffer holds the 16-column tiles alternately, gate tile j, up tile j, gate
 * tile j+1, ..., i.e. it equals w4a16_pack of the weight with its columns permuted so that
 * permuted column 32*j + c is column 16*j + c (c < 16) or N/2 + 16*j + c - 16 (c >= 16).  This is
 * the layout W4A16_EPI_SILU_MUL needs; every other entry point sees the permuted weight.
 * Requires N % 32 == 0, otherwise as w4a16_pack. */
int w4a16_pack_gate_up(const int32_t *qweight, const void *scales, const int32_t *qzeros, void *packed,
                       int N, int K, int G, void *stream);

/* Scratch needed by tree_verify_attn for these sizes (partial softmax states of the key splits). */
size_t tree_verify_attn_workspace_bytes(int M, int P, int Hq, int Hkv, int D);

/* Attention of the tree-verification pass (paper section 2.1: the target model scores the n
 * draft-tree tokens in one forward pass).  Query row i of head h attends, through KV head
 * h / (Hq/Hkv), to the P committed prefix keys and to the draft keys j with mask[i*M + j] != 0:
 *   out[i,h,:] = sum_j softmax_j(scale * q[i,h,:].k[j,kvh,:]) * v[j,kvh,:]
 * q, out fp16 [M, Hq, D]; k, v fp16 [P+M, Hkv, D] (draft keys at rows P..P+M-1); mask uint8 [M, M]
 * row-major.  Softmax and accumulation in fp32.  Requires D == 128, 1 <= M <= 64, Hq % Hkv == 0,
 * Hq/Hkv <= 8, P >= 0, a finite scale > 0 (W4A16_EINVAL otherwise), and every row must see at least
 * one key.  `workspace` as for w4a16_gemm,
 * sized by tree_verify_attn_workspace_bytes and initialised by w4a16_workspace_init. */
int tree_verify_attn(const void *q, const void *k, const void *v, const uint8_t *mask, void *out,
                     int M, int P, int Hq, int Hkv, int D, float scale,
                     void *workspace, size_t workspace_bytes, void *stream);

/* Greedy acceptance of a verified draft tree and compaction of the accepted K/V rows -- the integer
 * step that follows tree_verify_attn and the target model's remaining layers (paper section 2.1:
 * draft-then-verify, the target accepts some of the n draft-tree tokens; section 4: verifying a tree
 * turns it into a sequence).  Node 0 is the root (the last committed token); parent[i] < i for i > 0
 * and parent[0] < 0.  token[i] is the draft token at node i, target[i] the target model's greedy next
 * token after the sequence that ends in node i.  Starting at the root, a child of the current node is
 * accepted iff its draft token equals the current node's target token (the lowest index among several);
 * the walk stops at the first node without an accepted child.
 *   path   int32 [M], out: accepted node indices, root first; unused entries are -1
 *   result int32 [2], out: [0] = number of accepted nodes (root included), [1] = target[last accepted
 *          node], the token the target model itself contributes
 *   k, v   fp16 [P+M, Hkv, D], both given or both NULL: when given, cache row P + j receives row
 *          P + path[j] for every accepted position j, in place; all other rows are left untouched
 * parent, token, target, path, result: device pointers, 4-byte aligned; k, v: 16-byte aligned,
 * Hkv * D * 2 a multiple of 16.  1 <= M <= 64.  The kernel stays in bounds and terminates for any
 * content of parent (an entry that breaks parent[i] < i merely makes node i unreachable). */
int tree_accept(const int32_t *parent, const int32_t *token, const int32_t *target, int M, int32_t *path,
                int32_t *result, void *k, void *v, int P, int Hkv, int D, void *stream);

/* Root-mean-square layer norm of the Llama-type target model (paper section 2.1 counts one whole
 * forward pass per verification; every linear pair of a layer is fed by this norm):
 *   y[m,k] = x[m,k] * gamma[k] / sqrt(mean_k(x[m,:]^2) + eps),  fp32 arithmetic, one rounding to fp16.
 * x, y fp16 [M, K] (y may be x: in place), gamma fp16 [K].  Requires K % 8 == 0, K <= 16384, eps >= 0. */
int rms_norm(const void *x, const void *gamma, void *y, int M, int K, float eps, void *stream);

/* Rotary position embedding of the q and k parts of a fused qkv projection and the append of the new
 * keys and values to the cache -- the step between the qkv linear and tree_verify_attn.
 *   qkv       fp16 [M, (Hq + 2 Hkv) D]: per row Hq query heads, Hkv key heads, Hkv value heads
 *   pos       int32 [M], 4-byte aligned: position of each row (draft tree: prefix length + node depth)
 *   cos_table, sin_table  fp32 [n_pos, D/2], 4-byte aligned, the caller's tables: entry [p, i] rotates
 *             the element pair (i, i + D/2) of every head at position p:
 *               out[i] = a[i] cos - a[i + D/2] sin,   out[i + D/2] = a[i + D/2] cos + a[i] sin
 *   q         fp16 [M, Hq, D], out
 *   k_cache, v_cache  fp16 [>= P + M, Hkv, D]: rows P..P+M-1 receive the rotated keys and the values;
 *             all other rows are left untouched
 * fp32 arithmetic, one rounding to fp16.  A row whose position lies outside [0, n_pos) gets its
 * values appended but its q and k rows are left untouched.  Requires D even, D <= 2048. */
int rope_append(const void *qkv, const int32_t *pos, const float *cos_table, const float *sin_table, int n_pos,
                void *q, void *k_cache, void *v_cache, int M, int P, int Hq, int Hkv, int D, void *stream);

/* w4a16_pack for a weight whose columns are heads of head_dim columns each (a q/k/v projection): inside
 * every head the 16-column tiles of its two halves alternate -- packed tile 2j of the head is tile j of
 * elements 0..head_dim/2-1, packed tile 2j+1 tile j of elements head_dim/2.. -- so that the element pair
 * (d, d + head_dim/2) the rotary embedding turns lies in neighbouring tiles.  This is the layout
 * w4a16_gemm_rope needs; every other entry point sees the weight with its columns permuted that way.
 * Requires head_dim % 32 == 0 and N % head_dim == 0, otherwise as w4a16_pack. */
int w4a16_pack_heads(const int32_t *qweight, const void *scales, const int32_t *qzeros, void *packed,
                     int N, int K, int G, int head_dim, void *stream);

/* The q/k/v projection of a decoder layer with rope_append fused into its store: one launch and one round
 * trip of the [M, (Hq + 2 Hkv) D] projection less (3 us per layer at these sizes).  Equal, bit for bit, to
 *   w4a16_gemm(x, Wqkv) -> fp16 qkv;  rope_append(qkv, ...)
 * -- the sums are rounded to fp16 first and then rotated with rope_append's own expressions.  `packed` must
 * come from w4a16_pack_heads with head_dim = D; N is (Hq + 2 Hkv) D.  x, workspace, errors: as w4a16_gemm;
 * pos, tables, q, k_cache, v_cache, P: as rope_append, except that the tables must be 16-byte aligned and
 * D % 32 == 0 (W4A16_EALIGN / W4A16_EINVAL otherwise: use the two calls). */
int w4a16_gemm_rope(const void *x, const void *packed, int M, int K, int G, const int32_t *pos, const float *cos_table,
                    const float *sin_table, int n_pos, void *q, void *k_cache, void *v_cache, int P, int Hq, int Hkv, int D,
                    void *workspace, size_t workspace_bytes, void *stream);

/* One decoder layer of a Llama-type target model on M token rows over a P-token prefix, enqueued as one
 * call (paper section 2.1: a verification is one forward pass of the target over the draft tokens):
 *   n = rms_norm(h, norm1_gamma);  qkv = n . Wqkv;  rope_append(qkv) -> q, cache rows P..P+M-1;
 *   a = tree_verify_attn(q, cache, mask, scale 1/sqrt(head_dim));  h += a . Wo;
 *   n = rms_norm(h, norm2_gamma);  h += (silu(n . Wgate) * (n . Wup)) . Wdown
 * i.e. exactly rms_norm, w4a16_gemm, rope_append, tree_verify_attn and w4a16_gemm_fused (residual in
 * place, SiLU gate) in this order on `stream`; arguments mean what they mean there.  h fp16 [M, hidden] is
 * updated in place.  Weights: w4a16_pack outputs for qkv [hidden -> (n_q_heads + 2 n_kv_heads) head_dim],
 * o [n_q_heads head_dim -> hidden] and down [ffn -> hidden]; a w4a16_pack_gate_up output for
 * gate_up [hidden -> 2 ffn]; group size 128.  Scratch, all fp16 and 16-byte aligned, owned by the
 * caller: norm [M, hidden], qkv [M, (n_q_heads + 2 n_kv_heads) head_dim], q and attn [M, n_q_heads,
 * head_dim], act [M, ffn]; gemm_workspace sized for the largest of the four linears
 * (w4a16_workspace_bytes) and attn_workspace (tree_verify_attn_workspace_bytes), both initialised with
 * w4a16_workspace_init.  With qkv_heads_packed set, qkv_packed is a w4a16_pack_heads output and the second
 * and third step are one call of w4a16_gemm_rope (same results bit for bit; the qkv scratch is not used and
 * may be NULL; head_dim % 32 == 0 and 16-byte-aligned tables are then required).  Returns the first error
 * of the calls it makes; validation failures of the first call enqueue nothing, a failure further on leaves
 * the earlier steps enqueued. */
typedef struct {
    const void *qkv_packed, *o_packed, *gate_up_packed, *down_packed;
    const void *norm1_gamma, *norm2_gamma; /* fp16 [hidden] */
    int hidden, n_q_heads, n_kv_heads, head_dim, ffn;
    float eps;
    int qkv_heads_packed; /* nonzero: qkv_packed comes from w4a16_pack_heads and the layer uses w4a16_gemm_rope */
    int symmetric;        /* nonzero: all four weights have zero-points 8 throughout (W4A16_SYMMETRIC on every linear that
                             takes the flag: o, gate_up, down, and qkv when it is not the fused-rotary projection) */
} w4a16_layer_weights;
typedef struct {
    void *norm, *qkv, *q, *attn, *act;
    void *gemm_workspace;
    size_t gemm_workspace_bytes;
    void *attn_workspace;
    size_t attn_workspace_bytes;
} w4a16_layer_scratch;
int w4a16_decoder_layer(const w4a16_layer_weights *w, void *h, int M, int P, const int32_t *pos,
                        const float *cos_table, const float *sin_table, int n_pos, const uint8_t *mask,
                        void *k_cache, void *v_cache, const w4a16_layer_scratch *s, void *stream);

/* Size in bytes of the packed LM-head weight for a V-token vocabulary and hidden size K (the
 * vocabulary is padded to a multiple of 16 inside the buffer).  0 if the shape is not supported. */
size_t lm_head_packed_bytes(int V, int K);

/* Re-lay an fp16 LM-head weight W [V, K] (row-major, one row per token) into the streaming layout
 * lm_head_topk reads: 16-token tiles whose 16x32 blocks are stored in matrix-instruction operand
 * order, one contiguous run per tile.  Offline, once per weight.  Requires K % 128 == 0;
 * `packed` receives lm_head_packed_bytes(V, K) bytes. */
int lm_head_pack(const void *W, void *packed, int V, int K, void *stream);

/* Scratch lm_head_topk needs for these sizes (per-chunk softmax statistics and top-k candidates). */
size_t lm_head_workspace_bytes(int M, int V, int K, int top_k);

/* Draft-side language-model head with log-softmax and top-k (paper section 2.1: the draft model uses
 * the target's LM head and grows its beam-search tree from the softmax output; section 3.1: the draft
 * stays in fp16 because this head and its softmax dominate drafting and cannot be quantised).
 *   x        fp16 [M, K]   hidden states, 1 <= M <= 64 (a draft beam; or the rows of a verification pass,
 *                          whose target tokens are the top-1 of the target model's own head)
 *   packed   the LM-head weight W fp16 [V, K] as laid out by lm_head_pack
 *   logits   fp32 [M, V]   out: logits[m, v] = sum_k x[m, k] W[v, k], fp32 accumulation
 *   top_idx  int32 [M, top_k], top_logprob fp32 [M, top_k]   out: per row the top_k tokens by logit,
 *            largest first, equal logits in ascending token order, with
 *            logprob = logit - log(sum_v exp(logit[m, v]))
 * x, packed, logits, workspace 16-byte aligned; top_idx, top_logprob 4-byte aligned.  Requires
 * K % 128 == 0, 1 <= top_k <= min(V, 64), V <= 262144 and ceil(V / 512) * top_k <= 8192.  `workspace` holds
 * lm_head_workspace_bytes(M, V, K, top_k) bytes and needs no initialisation.  Deterministic. */
int lm_head_topk(const void *x, const void *packed, int M, int V, int K, int top_k, float *logits, int32_t *top_idx,
                 float *top_logprob, void *workspace, size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------------
 * Measurement and ablation aids.  Not part of the method's interface: nothing above needs them, a
 * deployment never calls them.  They exist so that the benchmark and the tests can force a kernel
 * variant, ask which variant a call would run, and time a plain read beside the GEMM.
 * ------------------------------------------------------------------------------------------------- */

/* Ablation knob for benchmarks and tests: overrides an internal launch heuristic process-wide.
 * Names: "split_k" (0 = heuristic, else forced number of K splits), "fused_reduce" (1 = the last
 * workgroup of a column unit sums the split-K partials inside the GEMM kernel, 0 = a second
 * kernel does, 2 = per-shape choice, the default),
 * "tiles_per_wave" (0 = heuristic, else 2, 4 or 8 sixteen-column tiles per wavefront),
 * "waves_per_wg" (0 = heuristic; 4, 8 or 16 wavefronts per workgroup that split K; 1 selects the
 * variant whose four wavefronts split the columns and share x through LDS), "prefetch_depth" (0 =
 * heuristic, else 1, 2 or 4 groups of codes in flight per wavefront), "k_sets" (0 = heuristic, else
 * 1, 2 or 3: forces the M > 16 variant whose workgroup has 4 * k_sets wavefronts, four column
 * quarters times k_sets interleaved sets of quantisation groups; waves_per_wg is then ignored and
 * fused_reduce = 2 means the second kernel), "even_split" (with k_sets: 1 deals the (column unit, group)
 * pairs in equal runs to one workgroup per compute unit instead of splitting K into split_k equal parts
 * per unit; the runs that share a unit are summed by the last to arrive), "flat_groups" (0 = heuristic, else 4, 7 or 8: forces the M <= 4 variant in which a
 * wavefront owns that many quantisation groups and requests all of their weights up front; needs
 * K / 128 == split_k * waves_per_wg * flat_groups); a combination that is not compiled, or that
 * does not fit the shape, makes w4a16_gemm return W4A16_EUNSUP,
 * "attn_splits" (0 = heuristic, else the number of key ranges per row tile in tree_verify_attn),
 * "attn_pack" (how many query heads of a KV group share a row tile of tree_verify_attn: 0 = the measured
 * rule -- the whole group when it fits 8 tile rows, else the fewest heads that leave at most 32 tiles;
 * 1 = one tile per query head always; 2 = the whole group whenever it fits 64 rows; 10 + d = exactly d heads
 * where d divides the group and the tile fits 64 rows, else one), "attn_row_tiles" (which kernel of
 * tree_verify_attn runs: 0 = the one that shares K and V tiles through LDS; the older one, kept for comparison:
 * 2 = a wavefront carries 32 query rows, in two row groups for taller tiles; 4 = 64 rows, one wavefront
 * per SIMD), "attn_fused_merge" (how the key ranges of a
 * row tile are merged: 2 = by the last of its workgroups to finish, 1 = by a second kernel, 0 = the former while
 * rows x ranges of a tile stay small), "lm_tiles" (0 = heuristic, else 1, 2 or
 * -- for more than 16 rows -- 4 vocabulary tiles per wavefront in lm_head_topk).
 * Returns W4A16_EINVAL for an unknown name or an out-of-range value.  Not thread-safe. */
int w4a16_set_param(const char *name, int value);
int w4a16_get_param(const char *name);

/* The launch shape w4a16_gemm (and its fused forms) would use for this call with the current knobs, so
 * that a test can show that every kernel the default plans reach has been compared with the oracle and a
 * benchmark can name what it timed.  out receives 8 ints:
 *   [0] kernel family: 0 = workgroup whose wavefronts split K, 1 = all loads up front (M <= 4),
 *       2 = column-split software-pipelined, 3 = column-split with interleaved K sets
 *   [1] 16-row tiles (ceil(M / 16))            [2] 16-column tiles per wavefront
 *   [3] wavefronts per workgroup (families 0, 1; 1 for family 2) or K sets (family 3)
 *   [4] groups of codes in flight per wavefront, or groups per wavefront (family 1)
 *   [5] K splits across workgroups (0 = even split)   [6] 1 if the last workgroup of a unit sums the splits
 *   [7] 1 if this kernel family has a symmetric instantiation, i.e. W4A16_SYMMETRIC would take effect, else 0
 * Host only: touches no GPU.  Errors as w4a16_gemm's shape checks; W4A16_EUNSUP if the knobs name a
 * variant that is not compiled. */
int w4a16_plan_describe(int M, int N, int K, int G, int *out);

/* Measurement aid, not part of the method: enqueues a kernel that only reads the first
 * bytes - bytes % 16 bytes of `buf` with 16-byte streaming loads (one 32 KB chunk per workgroup)
 * and writes nothing, except -- practically never -- one 32-bit word to `sink` (4-byte aligned, device)
 * so that the loads cannot be dropped.  Timed beside w4a16_gemm on the same packed buffer it
 * gives the read bandwidth this GPU reaches at that size, the ceiling the paper's memory-bound
 * decoding argument (section 2.1) refers to. */
int w4a16_read_probe(const void *buf, size_t bytes, void *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* W4A16_H */
