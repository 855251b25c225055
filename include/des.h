/*
 * des.h - C ABI of the MI355X (gfx950) hot path of Dynamic Expert Sharing (DES):
 * one Mixture-of-Experts layer applied to a whole parallel-decoding block of N
 * tokens, where the block elects a shared expert coreset (Alg. 1 stage 1), each
 * token is re-routed to its top-K experts inside that coreset (Alg. 1 stage 2)
 * and a grouped SwiGLU expert FFN reads every selected expert's weights from
 * HBM once.
 *
 * Conventions that hold for every entry point unless its comment says otherwise
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library
 *     allocates and frees nothing; scratch comes from the caller's `workspace`.
 *   - Calls validate their arguments on the host, enqueue kernels on
 *     `hip_stream` (a hipStream_t passed as void*; NULL = the default stream)
 *     and return without synchronising.  No device-to-host copy happens: the
 *     host never learns which experts were elected, so launches are sized for
 *     the worst case and pick their work list up from device memory.
 *   - Return value: DES_OK (0), or a negative des_status_t.  Argument errors
 *     are detected before anything is launched, so a failing call leaves all
 *     outputs untouched.  des_strerror() names a code.
 *   - Router logits must be finite; behaviour is unspecified otherwise.
 *   - Every TopK breaks ties towards the lowest expert index and compares
 *     values as numbers (+0 equals -0).
 *   - Results are run-to-run bit-identical: no floating-point atomics are used,
 *     unless the caller asks for them with vote_atomic = 1 (see des_shape_t).
 *   - Expert weights are streamed from HBM straight into matrix-core operand
 *     registers, not staged through LDS: a weight element is used by exactly
 *     one matrix instruction of one wavefront, so a stop in LDS would add a hop
 *     and no reuse (measured slower).  LDS holds what IS shared: the router's
 *     partial tiles, the selection state, the token rows of long blocks and the
 *     partial sums that the wavefronts of a workgroup exchange.
 *
 * Tensor layouts ("rows contiguous along the reduction dimension"):
 *   x          [B][N][D]       hidden states, dtype
 *   w_router   [M][D]          row i is expert i's router vector, dtype
 *   router_bias[M]             fp32, or NULL
 *   w_gate     [M][F][D]       row f of expert e produces intermediate unit f
 *   w_up       [M][F][D]
 *   w_down     [M][D][F]       row d of expert e produces output coordinate d
 *   (the mathematical orientation is gate/up: D x F, down: F x D; a loader
 *   transposes once when the model is set up)
 *   With weight_layout == DES_LAYOUT_PACKED (bf16 only) the three expert
 *   tensors hold the same values re-tiled by des_pack_expert_weights() so that
 *   a wavefront's matrix-core operand is one contiguous 1 KiB read.
 */
#ifndef DES_H
#define DES_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  DES_VANILLA = 0, /* Eq. 1: every token takes its own top-K of all M experts   */
  DES_SEQ = 1,     /* Eq. 5 / Alg. 2: coreset = union of per-token top-k_seq     */
  DES_VOTE = 2     /* Eq. 6 / Alg. 3: coreset = top-C of the masked vote vector  */
} des_mode_t;

typedef enum { DES_F32 = 0, DES_BF16 = 1 } des_dtype_t;

typedef enum { DES_LAYOUT_ROWMAJOR = 0, DES_LAYOUT_PACKED = 1 } des_layout_t;

/* The routing function sigma, which Sec. 4.1 leaves to the model: router weight of
 * expert i for a token = softmax over the M logits, or sigmoid of its own logit.  Either
 * way a token's gates are its selected weights divided by their sum (Eq. 1), and every
 * ranking compares logits (both functions are monotone). */
typedef enum { DES_ROUTER_SOFTMAX = 0, DES_ROUTER_SIGMOID = 1 } des_router_act_t;

/* Group-limited routers (another sigma of Sec. 4.1): the M experts form n_group equal
 * groups of consecutive indices; a token scores each group by the best router weight in
 * it, or by the sum of its two best, keeps the topk_group best groups (ties to the lowest
 * group index) and never ranks an expert outside them - not in its own top-K that
 * nominates and votes (Alg. 1 stage 1), not in its choice inside the coreset (stage 2).
 * A token whose groups hold fewer coreset experts than it may use takes only those
 * (index -1, weight 0 in the other slots; none at all: no routed expert). */
typedef enum { DES_GROUP_MAX = 1, DES_GROUP_TOP2SUM = 2 } des_group_score_t;

typedef enum {
  DES_OK = 0,
  DES_ERR_NULL = -1,      /* a required pointer is NULL                          */
  DES_ERR_SHAPE = -2,     /* a size is out of range or not supported             */
  DES_ERR_MODE = -3,      /* mode is not a des_mode_t                            */
  DES_ERR_DTYPE = -4,     /* dtype / weight_layout not supported                 */
  DES_ERR_WORKSPACE = -5, /* workspace smaller than des_workspace_bytes()        */
  DES_ERR_HIP = -6        /* a HIP call failed; des_last_hip_error() has text    */
} des_status_t;

/* Problem shape.  Paper symbol in brackets. */
typedef struct {
  int32_t n_seqs;        /* B: independent sequences; each elects its own coreset  */
  int32_t n_tokens;      /* [N] tokens per sequence (the parallel-decoding block)  */
  int32_t hidden;        /* [D]                                                    */
  int32_t n_experts;     /* [M]                                                    */
  int32_t ffn;           /* F: routed-expert intermediate size                     */
  int32_t ffn_shared;    /* F_s: always-on shared expert, 0 = none                 */
  int32_t top_k;         /* [K] experts per token                                  */
  int32_t coreset;       /* [M_core] C: coreset budget; ignored in vanilla mode    */
  int32_t k_seq;         /* [k] DES-Seq local count; 0 = largest k' <= K whose     */
                         /*     union fits in C (see des_select_coreset)           */
  int32_t mode;          /* des_mode_t                                             */
  int32_t dtype;         /* des_dtype_t of x, w_router, expert weights and y       */
  int32_t weight_layout; /* des_layout_t of w_gate / w_up / w_down (+ shared)      */
  int32_t residual;      /* 1: y = x + MoE(x)  (layer inside a residual stack)     */
  int32_t k_route;       /* experts a token finally uses (Alg. 1 stage 2) while the */
                         /* election still uses K; 0 = K.  Sec. 5.3, "Effect of    */
                         /* active expert count" (same coreset, k = 8 vs k = 4);   */
                         /* in vanilla mode this is the plain top-k baseline       */
  float skip_beta;       /* > 0: after stage 2, a token drops its experts i..k     */
                         /* (rank order) when their gates sum to less than         */
                         /* skip_beta of the sum of all k gates - the largest such */
                         /* tail, never the best expert - and the gates are        */
                         /* re-normalised over the rest (the adapted NAEE rule of  */
                         /* Sec. 5.1, Baselines).  0 = off.  The comparison is in  */
                         /* fp32; a tail within ~1e-6 (relative) of the threshold  */
                         /* may fall either way                                    */
  int32_t router_act;    /* des_router_act_t: weights that are voted with (Eq. 6)  */
                         /* and turned into gates (Alg. 1 stage 2)                 */
  int32_t vote_renorm;   /* 1: a token's K votes are divided by their sum, so each */
                         /* token casts a total weight of one (the other reading   */
                         /* of how Sec. 4.2 adds up the votes); 0: as Alg. 3 is    */
                         /* written (mask, then sum)                               */
  int32_t n_group;       /* > 1: group-limited routing over this many groups;      */
                         /* 0 or 1 = off (topk_group, group_score then ignored)    */
  int32_t topk_group;    /* groups a token keeps, 1..n_group                       */
  int32_t group_score;   /* des_group_score_t.  "max" compares logits (exact);     */
                         /* "top2sum" adds two fp32 router weights per group, and  */
                         /* two groups within ~1e-6 (relative) may swap            */
  int32_t vote_atomic;   /* 1: the votes of Eq. 6 meet in floating-point atomic    */
                         /* adds, in arrival order, as the selection kernels of    */
                         /* Sec. 4.3 do: V may differ in its last bits from run to */
                         /* run (and two experts within ~1e-6 of each other may    */
                         /* swap).  0: fixed-order sum, bit-identical every run    */
} des_shape_t;

/*
 * Limits checked by every entry point (DES_ERR_SHAPE otherwise):
 *   B, N, D, M, F, K >= 1;  K <= M;  K <= 32;  M <= 512;  B*N <= 4096;
 *   M * ceil(B*N/64) <= 4096;  C >= 1 in seq / vote mode;  0 <= k_seq <= K;
 *   0 <= k_route <= K;  0 <= skip_beta < 1;  router_act, vote_renorm, vote_atomic in {0, 1};
 *   n_group > 1: M a multiple of n_group, the group size M/n_group a multiple of 8,
 *   1 <= topk_group <= n_group, topk_group * (M/n_group) >= K (a token can always
 *   nominate K experts), group_score a des_group_score_t (DES_ERR_MODE otherwise);
 *   seq mode with an explicit k_seq needs C >= min(M, N*k_seq) so that the
 *   union of Eq. 5 always fits the coreset_idx buffer;
 *   bf16: D, F, F_s multiples of 32 (matrix-core K step); fp32: multiples of 4.
 */

/* Width of one row of coreset_idx: M in vanilla mode, min(C, M) otherwise. */
int32_t des_coreset_capacity(const des_shape_t* shape);

/* Bytes of device scratch des_moe_forward needs for `shape`.  Host only: does
 * not touch the GPU.  Returns 0 if the shape is invalid. */
size_t des_workspace_bytes(const des_shape_t* shape);

/*
 * Router scores (Background: G: R^D -> R^M) and the router weights made of them
 * (the per-token softmax of Sec. 4.3, or sigmoids if router_act says so):
 *   logits[b][n][i] = sum_d x[b][n][d] * w_router[i][d] (+ router_bias[i]),
 *   probs [b][n][:] = softmax over all M of logits[b][n][:], or sigmoid of each
 *                     logit (if probs != NULL)
 * Inputs are read in `dtype`, accumulated in fp32; outputs are fp32
 * [B][N][M].  Uses no workspace.
 */
int des_route(const des_shape_t* shape, const void* x, const void* w_router,
              const float* router_bias, float* logits, float* probs, void* hip_stream);

/*
 * Stage 1 of Alg. 1, coreset = Phi(logits), for each of the B sequences.
 *   vanilla: all M experts.
 *   seq    : k_seq > 0: union over tokens of TopK(logits[n], k_seq)  (Eq. 5).
 *            k_seq == 0: the largest k' <= K whose union has at most C members;
 *            if even k' = 1 does not fit, the C experts with the most top-1
 *            nominations (ties to the lowest index) and k_seq_used = 0.
 *   vote   : V[i] = sum over tokens n with i in TopK(logits[n], K) of
 *            softmax(logits[n])[i] (fp32, fixed summation order);
 *            coreset = the C experts of largest V among experts nominated by
 *            at least one token (Eq. 6); it is smaller than C when fewer
 *            were nominated.
 * Outputs: coreset_idx [B][des_coreset_capacity] ascending expert ids padded
 * with -1; coreset_size [B]; votes [B][M] (vote mode; may be NULL);
 * k_seq_used [B] (may be NULL).  Uses no workspace.
 */
int des_select_coreset(const des_shape_t* shape, const float* logits, int32_t* coreset_idx,
                       int32_t* coreset_size, float* votes, int32_t* k_seq_used,
                       void* hip_stream);

/*
 * The whole layer, Alg. 1 (Eq. 1 when mode == DES_VANILLA):
 *   logits as des_route; coreset as des_select_coreset;
 *   S_n   = first k_eff = min(K, |coreset|) experts of the coreset in the order
 *           (logit descending, index ascending)                 -> topk_idx
 *   g_n   = softmax of logits[n] over S_n                        -> topk_w
 *   y_n   = sum_j g_n[j] * E_{S_n[j]}(x_n)  (+ E_shared(x_n))  (+ x_n if residual)
 *   E(x)  = Wd (silu(Wg x) * (Wu x)),  silu(z) = z / (1 + exp(-z))
 * Outputs (all device): y [B][N][D] dtype; logits [B][N][M] fp32;
 * topk_idx [B][N][K] int32 in rank order, unused slots -1; topk_w [B][N][K]
 * fp32, unused slots 0; expert_counts [M] int32 = pairs routed to each expert
 * summed over sequences (cnt_i of Eq. 2); n_unique [1] int32 = experts with a
 * non-zero count (|union S_n|); coreset_idx / coreset_size as above.
 * n_unique = -1 reports that a bounded wait between the stages of a launch ran
 * out.  The routing stages hand their results to each other inside one launch
 * and wait for each other there; that is only safe while every workgroup of
 * the launch is on the chip at once (checked against the device's compute-unit
 * count), so the call assumes that NO OTHER KERNEL occupies the device while it
 * runs.  If a wait does run out - another stream's kernel kept a producer off
 * the chip, or the workspace was shared with an overlapping call - every kernel
 * still exits normally: a routing stage that gives up leaves an empty work list
 * (expert_counts all zero; the expert FFN then reads no weights and y holds
 * only the shared expert's output, plus x under `residual`), an FFN stage that
 * gives up leaves y undefined but touches nothing outside the caller's buffers.
 * ws_gate / ws_up / ws_down: the shared expert ([Fs][D], [Fs][D], [D][Fs], same
 * dtype and layout rule), required iff ffn_shared > 0.
 * y must not alias x.  workspace: >= des_workspace_bytes(shape), 256-byte
 * aligned, contents irrelevant on entry.
 */
int des_moe_forward(const des_shape_t* shape, const void* x, const void* w_router,
                    const float* router_bias, const void* w_gate, const void* w_up,
                    const void* w_down, const void* ws_gate, const void* ws_up,
                    const void* ws_down, void* y, float* logits, int32_t* topk_idx,
                    float* topk_w, int32_t* expert_counts, int32_t* n_unique,
                    int32_t* coreset_idx, int32_t* coreset_size, void* workspace,
                    size_t workspace_bytes, void* hip_stream);

/*
 * des_moe_forward for callers that cannot allocate device memory or have none to
 * hand over: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, results and errors as des_moe_forward,
 * except that the scratch is a buffer built into the library (one copy of
 * DES_BUILTIN_WORKSPACE_BYTES per GPU, held until the process ends) instead of
 * the caller's workspace.  The call allocates and frees nothing.  A shape whose
 * des_workspace_bytes() exceeds DES_BUILTIN_WORKSPACE_BYTES is refused with
 * DES_ERR_WORKSPACE before anything is launched (the 128- and 256-expert
 * single-layer benchmark shapes need about 3 MiB).  All calls on one GPU share
 * that GPU's buffer: calls that overlap in time (different streams or threads,
 * or an overlapping des_moe_forward that was handed the same memory) race.
 * Nothing in the buffer has to survive between calls and nothing has to be
 * cleared.  The first call on a device looks the buffer's address up
 * (hipGetSymbolAddress); make that call outside graph capture.
 */
#define DES_BUILTIN_WORKSPACE_BYTES (8u << 20)
int des_moe_forward_builtin_ws(const des_shape_t* shape, const void* x, const void* w_router,
                               const float* router_bias, const void* w_gate, const void* w_up,
                               const void* w_down, const void* ws_gate, const void* ws_up,
                               const void* ws_down, void* y, float* logits, int32_t* topk_idx,
                               float* topk_w, int32_t* expert_counts, int32_t* n_unique,
                               int32_t* coreset_idx, int32_t* coreset_size, void* hip_stream);

/*
 * A residual stack of n_layers such layers, x_{l+1} = x_l + MoE_l(x_l)
 * (shape->residual is taken as 1).  Layer l's tensors start at
 * base + l * stride elements: w_router [L][M][D], router_bias [L][M] (or NULL),
 * w_gate / w_up [L][M][F][D], w_down [L][M][D][F], shared likewise.
 * Outputs: y [B][N][D] = x_L; n_unique [L]; expert_counts [L][M].
 * workspace: >= des_stack_workspace_bytes(shape).
 */
size_t des_stack_workspace_bytes(const des_shape_t* shape);
int des_moe_stack_forward(const des_shape_t* shape, int32_t n_layers, const void* x,
                          const void* w_router, const float* router_bias, const void* w_gate,
                          const void* w_up, const void* w_down, const void* ws_gate,
                          const void* ws_up, const void* ws_down, void* y,
                          int32_t* expert_counts, int32_t* n_unique, void* workspace,
                          size_t workspace_bytes, void* hip_stream);

/*
 * The attention sub-layer around the MoE layers of a decoding step (the wider step of
 * Fig. 2 left, where attention is the other large share of the latency; Sec. 5.1: a
 * block of N tokens with cached prefix and suffix positions).  The paper does not define
 * it; this is plain multi-head scaled-dot-product attention: every block token attends
 * to every cached position and to every token of its own block (no causal mask - the
 * block is decoded together), no positional encoding, no bias.
 *   q = Wq x, k = Wk x, v = Wv x for the block's tokens; query head h reads key/value head
 *   h / (n_heads / n_kv_heads);  p = softmax(<q, key_j> / sqrt(head_dim)) over the
 *   n_prefix + n_suffix cached and the N block positions;  o = sum_j p_j value_j;
 *   y = Wo [o over heads] (+ x if shape->residual).
 * bf16 only (DES_ERR_DTYPE otherwise).  Layouts: wq [H*dh][D], wk, wv [Hkv*dh][D],
 * wo [D][H*dh] (rows along the reduction dimension, row-major); k_cache, v_cache
 * [B][Hkv][n_prefix + n_suffix][dh] (prefix positions first; may be NULL if both are 0);
 * x, y [B][N][D].  Limits (DES_ERR_SHAPE): D and H*dh multiples of 128; Hkv*dh a
 * multiple of 32; dh a multiple of 8, at most 128; n_heads a multiple of n_kv_heads; one
 * head's values fit 160 KB of LDS ((dh rounded up to 16) x (P + N rounded up to 32, + 4)
 * bf16: up to 600 positions at dh = 128).
 * Of `shape` only n_seqs, n_tokens, hidden, dtype and residual are read.  y must not alias x.
 * workspace: >= des_attention_workspace_bytes(), 256-byte aligned, contents irrelevant.
 */
typedef struct {
  int32_t n_heads;     /* H: query heads                                         */
  int32_t n_kv_heads;  /* Hkv: key / value heads (grouped queries when < H)      */
  int32_t head_dim;    /* dh                                                     */
  int32_t n_prefix;    /* cached positions before the block (Sec. 5.1 uses 16)   */
  int32_t n_suffix;    /* cached positions after the block  (Sec. 5.1 uses 16)   */
} des_attn_shape_t;

size_t des_attention_workspace_bytes(const des_shape_t* shape, const des_attn_shape_t* attn);
int des_block_attention(const des_shape_t* shape, const des_attn_shape_t* attn, const void* x,
                        const void* wq, const void* wk, const void* wv, const void* wo,
                        const void* k_cache, const void* v_cache, void* y, void* workspace,
                        size_t workspace_bytes, void* hip_stream);

/*
 * A stack of decoder layers, each the attention sub-layer above followed by the MoE
 * layer, both with a residual connection:  a = x_l + Attn_l(x_l);  x_{l+1} = a + MoE_l(a).
 * Layer l's tensors start at base + l * (their size): wq [L][H*dh][D], wk, wv, wo,
 * k_cache / v_cache [L][B][Hkv][P][dh], and the MoE tensors as in des_moe_stack_forward.
 * Outputs as des_moe_stack_forward.  workspace: >= des_decoder_workspace_bytes().
 */
size_t des_decoder_workspace_bytes(const des_shape_t* shape, const des_attn_shape_t* attn);
int des_decoder_stack_forward(const des_shape_t* shape, const des_attn_shape_t* attn, int32_t n_layers,
                              const void* x, const void* wq, const void* wk, const void* wv,
                              const void* wo, const void* k_cache, const void* v_cache,
                              const void* w_router, const float* router_bias, const void* w_gate,
                              const void* w_up, const void* w_down, const void* ws_gate,
                              const void* ws_up, const void* ws_down, void* y,
                              int32_t* expert_counts, int32_t* n_unique, void* workspace,
                              size_t workspace_bytes, void* hip_stream);

/*
 * Re-tile bf16 expert weights for DES_LAYOUT_PACKED.  `src` is n_mats
 * row-major matrices [rows][cols] (cols = reduction dimension; rows a
 * multiple of 16, cols a multiple of 32); `dst` (same size, must not alias)
 * receives, per matrix, tiles of 16 rows x 32 columns ordered
 * [row tile][column tile], each tile stored as 64 groups of 8 values:
 *   dst[((rt*(cols/32) + ct)*64 + l)*8 + j] = src[rt*16 + l%16][ct*32 + 8*(l/16) + j].
 * One-time set-up work, not part of the hot path.
 */
int des_pack_expert_weights(const void* src, void* dst, int64_t n_mats, int32_t rows,
                            int32_t cols, void* hip_stream);

/*
 * Coreset size for a budget given as a fraction of the experts, M_core = beta * M
 * (Sec. 5.1), rounded down as the sizes printed in Table 1 imply (0.15 * 256 -> 38,
 * 0.6 * 64 -> 38).  Host only.  Returns 0 for beta outside (0, 1] or n_experts < 1;
 * at least 1 otherwise.
 */
int32_t des_coreset_from_beta(double beta, int32_t n_experts);

/* ------------------------------------------------------------------------
 * Measurement and test aids.  None of them is part of the hot path.
 * ------------------------------------------------------------------------ */

/*
 * Measurement aid: one launch that reads `bytes`
 * bytes at `src` from HBM once (each wavefront streams one contiguous 64 KB
 * chunk) and computes nothing.  Its duration is the practical ceiling of a
 * weight scan of that size on this machine, against which the expert FFN of
 * Alg. 1 (whose cost is the fetch of the selected experts' weights, Eq. 2) is
 * quoted.  `bytes` must be a positive multiple of 65536, `src` and `sink`
 * 16-byte aligned; `sink` is 16 bytes of device memory that are never written
 * for real data.
 */
int des_hbm_read_probe(const void* src, size_t bytes, void* sink, void* hip_stream);

/*
 * Measurement aid, off by default and not part of the hot path: while enabled,
 * every kernel launch of this library carries a pair of HIP events that take
 * the dispatch's own begin and end timestamps (the events are created on the
 * host at launch time, so do not enable it under graph capture).  des_kernel_timing_read() waits for the
 * recorded events and returns the accumulated duration and launch count of one
 * kernel id in [0, des_kernel_timing_count()); des_kernel_timing_name() names
 * it (router, softmax, select, permute, gateup, down, combine, pack, routing,
 * ffn, read_probe, attn_proj, attn_core, attn_out).
 * des_kernel_timing_enable() also clears the accumulators.  Not thread-safe.
 */
int des_kernel_timing_enable(int enable);
int des_kernel_timing_count(void);
const char* des_kernel_timing_name(int kernel_id);
int des_kernel_timing_read(int kernel_id, double* total_ms, int64_t* launches);

/*
 * Test aid: forces the give-up path of the bounded waits from the host, so that a
 * test can check it without faulting or hanging anything.  skip_router = 1: the
 * fused routing launch runs without its router workgroups (nobody produces the
 * logits the selectors wait for); skip_router = 2: the same for the next such
 * launch only, after which both hooks reset themselves (one layer of a stack);
 * max_wait_iters > 0: a wait gives up after that many polls instead of after
 * seconds.  (0, 0) restores normal operation.
 * Process-wide, not thread-safe.
 */
int des_test_hooks(int skip_router, int max_wait_iters);

const char* des_strerror(int code);
/* Text of the last HIP error seen by this thread's DES_ERR_HIP ("" if none). */
const char* des_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* DES_H */
