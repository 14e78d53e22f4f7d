/*
 * metro.h -- C ABI of the MI355X (gfx950) METRO hot path.
 *
 * METRO = Minimum Expert Token ROuting (arxiv 2512.09277): choose one replica for every
 * (token, expert) pair so that the maximum number of *activated* expert replicas on any
 * expert-parallel rank is minimised (problem min-exp-routing, Sec. 4.1), then run the
 * memory-bound decode MoE layer of one rank on the pairs routed to it.
 *
 * Conventions for every call
 *   - All data pointers are DEVICE pointers owned by the caller; nothing is allocated,
 *     freed or synchronised inside.  Work is enqueued on `stream` (a hipStream_t passed as
 *     void*; NULL = the default stream) and the call returns at once.
 *   - Return value: METRO_OK or a negative METRO_ERR_* for arguments the host can check.
 *     On error nothing is enqueued.  Conditions only the device can see (an id out of
 *     range, an expert with tokens but no replica) are reported through `err_flag`.
 *   - Notation: N experts, top-k, G logical EP ranks, spr replica slots per rank,
 *     S = G*spr slots, slot s lives on rank s / spr; T tokens in the (global) batch;
 *     pair index p = t*k + j; H hidden size, I intermediate size.
 *   - Limits: 1 <= N <= 512, 1 <= G <= 64, 1 <= spr <= 64, S <= 2048, 1 <= k <= N,
 *     T*k < 2^24.
 */
#ifndef METRO_H_
#define METRO_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define METRO_OK 0
#define METRO_ERR_INVALID_ARG (-1)   /* null pointer, non-positive size, k > N, misaligned pointer */
#define METRO_ERR_UNSUPPORTED (-2)   /* a size beyond the limits above, unknown dtype */
#define METRO_ERR_WORKSPACE (-3)     /* workspace smaller than the *_workspace_bytes() figure */
#define METRO_ERR_HIP (-4)           /* the HIP runtime refused a launch */
#define METRO_ERR_TOO_LARGE (-5)     /* the problem needs more than the library's built-in scratch buffer */

/* bits of err_flag[layer] */
#define METRO_FLAG_BAD_ID 1          /* a top-k id outside [-1, N) */
#define METRO_FLAG_NO_REPLICA 2      /* an expert that has tokens is on no rank */
#define METRO_FLAG_BAD_PLACEMENT 4   /* a slot_to_expert entry outside [-1, N) */

#define METRO_DTYPE_F32 0
#define METRO_DTYPE_BF16 1

/* Text for a METRO_ERR_* code (static storage). */
const char* metro_status_string(int status);

/*
 * metro_route -- the greedy solve of min-exp-routing (Alg. 1, Sec. 4.3) for L independent
 * layers in one launch.  Experts are served in ascending id; each expert with at least one
 * pair (T[i] > 0) takes, among the ranks hosting it, the one with the fewest activated
 * experts so far, ties to the lowest rank; all of its pairs go to that replica (x from y,
 * Sec. 4.3).  The result is a deterministic, lock-free execution of Alg. 1.
 *
 *   topk_ids       [L,T,k] int32  global top-k expert ids of the whole batch; -1 = padded pair
 *   slot_to_expert [L,S]   int32  placement (matrix A of Sec. 4.1): expert held by each slot,
 *                                 -1 = empty slot; a second copy of an expert on the same rank
 *                                 is ignored (A is binary)
 *   pair_slot      [L,T,k] int32  out: chosen slot of every pair (-1 for padded pairs)
 *   expert_slot    [L,N]   int32  out: activated slot of every expert, -1 if it has no pair
 *   rank_active    [L,G]   int32  out: activated experts per rank (lambda = their maximum)
 *   rank_bitmap    [L,G]   uint64 out: bit l set iff local slot l of the rank is activated
 *   err_flag       [L]     int32  out: 0, or METRO_FLAG_* bits; outputs of a flagged layer are
 *                                 unspecified apart from being in range
 */
int metro_route(const int32_t* topk_ids, const int32_t* slot_to_expert, int L, int T, int k, int N, int G,
                int spr, int32_t* pair_slot, int32_t* expert_slot, int32_t* rank_active,
                uint64_t* rank_bitmap, int32_t* err_flag, void* stream);

/*
 * metro_route_token_balanced -- the baseline the paper compares with (EPLB-style routing,
 * Sec. 2.3 and Sec. 6.1 "Compared baselines"): every expert's pairs are spread evenly over
 * its replicas.  The q-th pair of an expert, in flattened (t, j) order, goes to replica
 * q mod r, replicas taken in ascending slot id.  Same arguments as metro_route, without
 * expert_slot (an expert may activate several replicas).
 */
int metro_route_token_balanced(const int32_t* topk_ids, const int32_t* slot_to_expert, int L, int T, int k,
                               int N, int G, int spr, int32_t* pair_slot, int32_t* rank_active,
                               uint64_t* rank_bitmap, int32_t* err_flag, void* stream);

/*
 * moe_permute -- per-replica token lists of one rank ("route tokens", Sec. 4.3): the pairs
 * whose slot lies on `rank`, ordered by local slot l = slot - rank*spr and, within a slot,
 * by pair index (a stable counting sort).
 *
 *   pair_slot     [T,k]   int32  one layer's routing result
 *   group_offsets [spr+1] int32  out: rows of local slot l are [group_offsets[l], group_offsets[l+1])
 *   perm_pair     [T*k]   int32  out: pair index of every row; entries past n_pairs are not written
 *   pair_row      [T,k]   int32  out: row of each pair in the list, -1 if routed to another rank
 *   n_pairs       [1]     int32  out: number of rows (= group_offsets[spr])
 */
int moe_permute(const int32_t* pair_slot, int T, int k, int rank, int spr, int32_t* group_offsets,
                int32_t* perm_pair, int32_t* pair_row, int32_t* n_pairs, void* stream);

/*
 * metro_route_permute / metro_route_token_balanced_permute -- one layer's routing solve followed, in the same
 * launch, by the token lists of one rank ("route tokens", Sec. 4.3): exactly metro_route (or
 * metro_route_token_balanced) with L = 1 and then moe_permute(pair_slot, rank), without the second launch --
 * the workgroup that has just written pair_slot sorts it.  Arguments and results as in those calls;
 * 0 <= rank < G.
 */
int metro_route_permute(const int32_t* topk_ids, const int32_t* slot_to_expert, int T, int k, int N, int G, int spr,
                        int rank, int32_t* pair_slot, int32_t* expert_slot, int32_t* rank_active,
                        uint64_t* rank_bitmap, int32_t* err_flag, int32_t* group_offsets, int32_t* perm_pair,
                        int32_t* pair_row, int32_t* n_pairs, void* stream);
int metro_route_token_balanced_permute(const int32_t* topk_ids, const int32_t* slot_to_expert, int T, int k, int N,
                                       int G, int spr, int rank, int32_t* pair_slot, int32_t* rank_active,
                                       uint64_t* rank_bitmap, int32_t* err_flag, int32_t* group_offsets,
                                       int32_t* perm_pair, int32_t* pair_row, int32_t* n_pairs, void* stream);

/*
 * moe_gate_topk -- router gate and top-k over the full (gathered) token set: the step that builds
 * the global top-k knowledge the routing solve consumes (Sec. 4.3: tokens are all-gathered and every
 * rank runs top-k on all of them).  The paper leaves the gate itself to the model; this is the
 * common softmax router:
 *     logit[t][e]  = x[t] . w_gate[e]
 *     topk_ids[t]  = the k experts with the largest logits, descending; equal logits: lower id first
 *     topk_w[t][j] = exp(logit[t][ids[t][j]]) / sum over the k selected of exp(logit)
 *     expert_count[e] = number of (token, expert) pairs that selected e      (T[i] of Sec. 4.1)
 * Batches are padded to fixed sizes where the layer is replayed from a captured graph (Sec. 5): tokens
 * t >= *n_valid are padding and get topk_ids -1 (which both routing calls skip), topk_w 0, and count nothing.
 *
 *   x        [T,H]   dtype     activations (rows H elements apart)
 *   w_gate   [N,H]   dtype     router weights, rows ldw >= H elements apart
 *   n_valid  [1]     int32     number of real tokens, read on the device (clamped to [0, T]); NULL = T
 *   topk_ids [T,k]   int32     out; valid input for metro_route / metro_route_token_balanced
 *   topk_w   [T,k]   float32   out; valid input for moe_unpermute
 *   expert_count [N] int32     out, may be NULL (asking for it adds one small launch)
 *   ws                         workspace of moe_gate_topk_workspace_bytes(); 256-byte aligned
 *   dtype  METRO_DTYPE_BF16: bf16 operands, fp32 accumulation on the matrix cores when H % 32 == 0,
 *          N % 64 == 0, ldw % 8 == 0 and x, w_gate are 16-byte aligned; other shapes and
 *          METRO_DTYPE_F32 take a plain fp32 kernel.  Logits are summed in a fixed order, so the
 *          result is deterministic; NaN logits sort below every number.
 * Limits: N <= 512, k <= min(N, 64), T*k < 2^24.  T == 0 writes nothing but expert_count (all zero).
 */
size_t moe_gate_topk_workspace_bytes(int T, int H, int N, int dtype);
int moe_gate_topk(const void* x, const void* w_gate, int ldw, int T, int H, int N, int k, int dtype,
                  const int32_t* n_valid, int32_t* topk_ids, float* topk_w, int32_t* expert_count, void* ws,
                  size_t ws_bytes, void* stream);

/*
 * moe_grouped_ffn -- SwiGLU expert FFN over the token lists of one rank.  Only slots with at
 * least one row are touched, so HBM weight traffic scales with the number of activated
 * experts (Sec. 3.2).  For row r of local slot l, token t = perm_pair[r] / k:
 *     gate = x[t] . w13[l][0:I]^T      up = x[t] . w13[l][I:2I]^T
 *     y_perm[r] = (silu(gate) * up) . w2[l]^T
 *
 *   x      [T,H]       dtype   activations of the whole batch
 *   w13    [spr,2I,H]  dtype   per local slot: rows 0..I-1 gate, I..2I-1 up (H contiguous);
 *                              consecutive rows are ldw13 >= H elements apart, slots 2I*ldw13
 *   w2     [spr,H,I]   dtype   per local slot: down projection (I contiguous), rows ldw2 >= I
 *                              elements apart, slots H*ldw2
 *   ldw13, ldw2                row pitches in elements, multiples of 8.  The weights are the
 *                              library's to lay out: a pitch that is a multiple of 4096 bytes makes
 *                              the 16 rows of one load instruction fall on the same few HBM
 *                              channels (measured: 5.3 instead of 6.2 TB/s at a 4096-byte pitch),
 *                              so pad such rows, e.g. by 128 elements.
 *   y_perm [T*k,H]     dtype   out: rows 0..n_pairs-1 are written
 *   ws                         workspace of moe_grouped_ffn_workspace_bytes(); 256-byte aligned
 *   dtype  METRO_DTYPE_BF16: bf16 storage, fp32 accumulation on the matrix cores, the
 *          intermediate silu(gate)*up rounded to bf16; needs H % 128 == 0 and I % 128 == 0,
 *          other shapes take a slower general kernel.  METRO_DTYPE_F32: fp32 throughout.
 *   x, w13, w2, y_perm must be 16-byte aligned.
 */
size_t moe_grouped_ffn_workspace_bytes(int T, int k, int spr, int H, int I, int dtype);
int moe_grouped_ffn(const void* x, const int32_t* perm_pair, const int32_t* group_offsets, int T, int k,
                    int spr, int H, int I, int dtype, const void* w13, int ldw13, const void* w2, int ldw2,
                    void* y_perm, void* ws, size_t ws_bytes, void* stream);

/*
 * The two stages of moe_grouped_ffn as separate calls, in the order gate_up -> down, on the same
 * workspace and stream (moe_grouped_ffn is exactly that sequence).  They exist so that a caller can
 * put events between the stages or overlap other work; arguments as above.  Both read
 * group_offsets: every workgroup derives its own piece of work from it, there is no planning pass.
 *   gate_up  act = silu(x . w13[gate]^T) * (x . w13[up]^T), kept in the workspace
 *   down     y_perm = act . w2^T
 */
int moe_grouped_ffn_gate_up(const void* x, const int32_t* perm_pair, const int32_t* group_offsets, int T, int k,
                            int spr, int H, int I, int dtype, const void* w13, int ldw13, void* ws,
                            size_t ws_bytes, void* stream);
int moe_grouped_ffn_down(const int32_t* group_offsets, int T, int k, int spr, int H, int I, int dtype,
                         const void* w2, int ldw2, void* y_perm, void* ws, size_t ws_bytes, void* stream);

/*
 * moe_grouped_ffn_static_ws -- moe_grouped_ffn for callers that cannot allocate or size a workspace (code under
 * HIP-graph capture, tight serving loops, harnesses that forbid hipMalloc): the intermediate activations
 * live in an array built into the library, METRO_STATIC_WS_BYTES per GPU, held from library load until the
 * process ends.  Same arguments and results as moe_grouped_ffn without ws / ws_bytes; same kernels.
 *   - A problem whose moe_grouped_ffn_workspace_bytes() exceeds moe_grouped_ffn_static_ws_bytes()
 *     (bf16: T*k*I*2 + 256 bytes; the DeepSeek-V3-shaped decode batch T*k = 8192, I = 2048 just fits)
 *     is refused with METRO_ERR_TOO_LARGE and nothing is enqueued.
 *   - The call allocates nothing.  Its first use on a device looks up the array's address.
 *   - All calls on one GPU share that GPU's array: calls that may overlap in time (different streams,
 *     different threads) race on it; serialise them or use moe_grouped_ffn with separate workspaces.
 *     Nothing in the array has to be cleared between calls.
 */
#define METRO_STATIC_WS_BYTES ((size_t)(32u << 20) + 256u)
size_t moe_grouped_ffn_static_ws_bytes(void);
int moe_grouped_ffn_static_ws(const void* x, const int32_t* perm_pair, const int32_t* group_offsets, int T, int k,
                              int spr, int H, int I, int dtype, const void* w13, int ldw13, const void* w2,
                              int ldw2, void* y_perm, void* stream);

/*
 * moe_unpermute -- the rank's share of the combine step (Sec. 2.2): for every token,
 *     out[t] = sum over j ascending of topk_w[t,j] * y_perm[pair_row[t,j]]   (pairs served here),
 * accumulated in fp32; tokens with no pair on this rank get zeros.
 *
 *   y_perm [T*k,H] dtype, pair_row [T,k] int32, topk_w [T,k] float32, out [T,H] dtype.
 *   An entry of pair_row outside [0, T*k) counts as "not on this rank".
 */
int moe_unpermute(const void* y_perm, const int32_t* pair_row, const float* topk_w, int T, int k, int H,
                  int dtype, void* out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* METRO_H_ */
