/*
 * vsprefill.h - C ABI of the MI355X (gfx950) vertical-slash sparse-prefill library.
 *
 * The library implements the inference hot path of VSPrefill: VSIndexer scoring, the
 * cumulative-threshold budget with TopK, and causal vertical-slash sparse attention with the
 * per-query-tile index merge done inside the attention kernel, plus a dense causal attention
 * kernel on the same layout and the vertical-slash aggregation of the dense attention map (the
 * indexer's distillation target and the Attention Recall metric).
 *
 * Conventions shared by every call
 *   - Every tensor pointer is a DEVICE pointer owned by the caller, contiguous, 16-byte
 *     aligned.  The library never allocates or frees device memory: scratch space is a caller
 *     workspace whose size comes from the matching *_workspace() query (0 bytes is possible;
 *     then ws may be NULL).  Structs (vs_indexer_t, vs_budget_t) live in HOST memory and are
 *     read during the call; the float arrays a vs_indexer_t points to are device memory.
 *   - bf16 tensors are [heads, n, 128] row-major (head_dim is fixed at 128).
 *   - GQA: query head h reads KV head h / (q_heads / kv_heads).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls enqueue
 *     work and return without synchronising; outputs are valid once the stream has run.
 *   - Return value: VS_OK (0) or a negative vs_status.  Argument checks happen on the host
 *     before anything is launched.  Data-dependent conditions (selection larger than the
 *     capacity, NaN scores) never abort: they are flagged in a device status word.
 *   - Calls on the same workspace must not overlap in time.
 */
#ifndef VSPREFILL_H
#define VSPREFILL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    VS_OK = 0,
    VS_ERR_INVALID_ARG = -1, /* null / misaligned pointer, non-positive size, tau outside [0,1] ... */
    VS_ERR_UNSUPPORTED = -2, /* q_heads % kv_heads != 0, d_h not a multiple of 64 or > 1024, n > 2^20 ... */
    VS_ERR_WORKSPACE = -3,   /* ws_bytes smaller than the *_workspace() answer, or ws NULL when bytes are needed */
    VS_ERR_CAPACITY = -4,    /* forced entries alone exceed cap_v / cap_s, or caps <= 0 */
    VS_ERR_HIP = -5,         /* a HIP call failed; vs_last_hip_error() has the hipError_t */
    VS_ERR_STATIC_LIMIT = -6 /* vs_sparse_prefill_static: the call needs more scratch than the library's fixed array holds */
} vs_status;

#define VS_HEAD_DIM 128
#define VS_MAX_SEQ (1 << 20)

/* bits of the per-head device status word written by vs_select_budget */
#define VS_STATUS_OVERFLOW 1  /* selection exceeded the capacity and was truncated by rank */
#define VS_STATUS_BAD_SCORE 2 /* a NaN or negative score was treated as 0 */
#define VS_STATUS_SATURATED 4 /* a score above 1 was given the mass of 1 */

/*
 * Rotary embedding, in place (Appendix, "RoPE Matrix Representation": block-diagonal 2x2
 * rotations, plane p turns by position * theta_base^(-2p/128)).  Input preparation for Q and K.
 *   x        [heads, n, 128] bf16, rotated in place; row r is position pos0 + r
 *   pairing  0: plane p couples elements (2p, 2p+1) (the appendix matrix); 1: (p, p+64)
 * Angles and the rotation are evaluated in fp64 and rounded once to bf16 (nearest even).
 */
int vs_rope_apply(void* x_bf16, int heads, int64_t n, int64_t pos0, double theta_base, int pairing,
                  void* stream);

/*
 * VSIndexer weights (Sec. "VSIndexer Design": Z = act(concat(K, V) W_U + b_U), one logit per
 * direction from W_V / W_S).  One set per layer, shared by all KV heads.  The struct is host
 * memory; the arrays are fp32 device memory.
 */
typedef struct {
    const float* W_U; /* [256, d_h] row-major: rows 0..127 multiply K, rows 128..255 multiply V */
    const float* b_U; /* [d_h] */
    const float* W_V; /* [d_h] vertical down-projection */
    const float* W_S; /* [d_h] slash down-projection */
    float b_V, b_S;   /* scalar output biases (they cancel in the softmax over positions) */
    int d_h;          /* hidden width: multiple of 64, 64..1024 */
    int act;          /* 0 = SiLU, 1 = GELU (erf form) */
} vs_indexer_t;

size_t vs_index_score_workspace(int kv_heads, int64_t n, int d_h);

/*
 * VSIndexer forward (Sec. "VSIndexer Design", Eqs. X, Z, A_v, A_s).
 *   k, v      [kv_heads, n, 128] bf16; k already carries RoPE
 *   a_v, a_s  [kv_heads, n] fp32 out: softmax over the n positions of each head.  a_v[g, j] is
 *             the score of key column j; a_s[g, t] is the score of slash offset o = t.
 * Arithmetic: bf16 inputs times W_U split into two bf16 terms on the matrix cores, fp32
 * accumulation, fp32 activation / down-projection / softmax.
 */
int vs_index_score(const void* k_bf16, const void* v_bf16, int kv_heads, int64_t n, const vs_indexer_t* w,
                   float* a_v, float* a_s, void* ws, size_t ws_bytes, void* stream);

/*
 * Budget rule (Sec. "Adaptive Sparse Index Selection", Eqs. k_d and I_d), host struct.
 *   mode 0  cumulative threshold: per head and direction, the fewest top-ranked scores whose
 *           mass reaches tau_d of the total mass.  Masses are integers, floor(score * 2^40), so
 *           the result does not depend on summation order; rank is (score descending, index
 *           ascending).  The threshold is ceil(tau * total) evaluated in fp64.
 *   mode 1  fixed k_v / k_s with the same ranking.
 * After the rule, columns 0..n_sink-1 and offsets 0..max(n_local,1)-1 are added (offset 0, the
 * diagonal, is always present) and each list is emitted in ascending order.  If a list would
 * exceed its capacity the forced entries stay, the best-ranked others fill the rest and
 * VS_STATUS_OVERFLOW is set for that head.
 */
typedef struct {
    int mode;
    double tau_v, tau_s;
    int k_v, k_s;
    int n_sink;
    int n_local;
    int cap_v, cap_s;
} vs_budget_t;

/* Bytes of device workspace with which vs_select_budget spreads every (head, direction) problem over many
 * workgroups; 0 for lengths short enough for one workgroup per problem.  Contents need no initialisation. */
size_t vs_select_budget_workspace(int heads, int64_t n);

/*
 *   a_v, a_s      [heads, n] fp32 scores (finite, in [0,1] expected; see status bits)
 *   idx_v, idx_s  [heads, cap_v] / [heads, cap_s] int32 out, ascending, first cnt entries valid
 *   cnt_v, cnt_s  [heads] int32 out
 *   status        [heads] int32 out (bit-or of VS_STATUS_* over both directions) or NULL
 *   ws, ws_bytes  device workspace of at least vs_select_budget_workspace() bytes (16-byte aligned), or NULL / 0: the
 *                 call then uses one workgroup per problem (same results; about three times slower at 128k).  A
 *                 non-NULL workspace that is too small is VS_ERR_WORKSPACE.
 */
int vs_select_budget(const float* a_v, const float* a_s, int heads, int64_t n, const vs_budget_t* b,
                     int32_t* idx_v, int32_t* cnt_v, int32_t* idx_s, int32_t* cnt_s, int32_t* status,
                     void* ws, size_t ws_bytes, void* stream);

size_t vs_sparse_prefill_workspace(int q_heads, int kv_heads, int index_heads, int64_t n);

/*
 * Causal vertical-slash sparse attention (Sec. "Sparse Attention Formulation", Eqs. M_S and
 * A-hat, with the mask of Sec. "Linear-Complexity Mask Construction"; kernel behaviour of Sec.
 * "Fused attention kernel implementation": indices are read per query tile, merged on the fly,
 * keys fetched on demand).  Row i of query head h attends to
 *     { j : 0 <= j <= i  and  ( j in I_v  or  i - j in I_s ) },   each key once,
 * with softmax(scale * q.k) renormalised over that set.  A row with no key gives zeros and
 * lse = -inf.
 *   q            [q_heads, n, 128] bf16;  k, v  [kv_heads, n, 128] bf16
 *   idx_v/cnt_v  [index_heads, cap_v] / [index_heads] selected key columns
 *   idx_s/cnt_s  [index_heads, cap_s] / [index_heads] selected diagonal offsets (0 = diagonal)
 *                Lists must be strictly ascending with entries in [0, n); out-of-range entries
 *                are ignored, other violations are undefined.
 *   index_heads  kv_heads (one mask per KV group, the paper's setting) or q_heads
 *   o            [q_heads, n, 128] bf16 out;  lse [q_heads, n] fp32 out or NULL
 * Arithmetic: bf16 MFMA for QK^T and PV, fp32 accumulation and softmax, P rounded to bf16.
 */
int vs_sparse_prefill(const void* q, const void* k, const void* v, int q_heads, int kv_heads, int64_t n,
                      float scale, const int32_t* idx_v, const int32_t* cnt_v, int cap_v,
                      const int32_t* idx_s, const int32_t* cnt_s, int cap_s, int index_heads,
                      void* o_bf16, float* lse, void* ws, size_t ws_bytes, void* stream);

/*
 * Tile-granular slash variant of vs_sparse_prefill (Sec. "Fused attention kernel implementation": the merged index
 * set is built per query block).  slash_granularity g groups the query rows in aligned blocks of g rows; row i keeps
 *     { j : 0 <= j <= i  and  ( j in I_v  or  i' - j in I_s for SOME row i' of the block of i ) },
 * a superset of the element-exact mask (g = 1, identical to vs_sparse_prefill).  Supported: g = 1 and g = 32.
 * All other arguments, the workspace and the error behaviour are those of vs_sparse_prefill; an unsupported g
 * returns VS_ERR_UNSUPPORTED.
 */
int vs_sparse_prefill_tiled(const void* q, const void* k, const void* v, int q_heads, int kv_heads, int64_t n,
                            float scale, const int32_t* idx_v, const int32_t* cnt_v, int cap_v,
                            const int32_t* idx_s, const int32_t* cnt_s, int cap_s, int index_heads,
                            int slash_granularity, void* o_bf16, float* lse, void* ws, size_t ws_bytes, void* stream);

/*
 * Chunked prefill (Sec. "Efficient VS Sparse Attention Inference": the same per-layer pipeline, applied to a block of
 * new query positions against all keys so far).  vs_sparse_prefill_tiled for n_q query rows that are the positions
 * pos0 .. pos0 + n_q - 1 of a sequence whose keys 0 .. n_kv - 1 are present:
 *   q, o   [q_heads, n_q, 128];  k, v  [kv_heads, n_kv, 128];  lse [q_heads, n_q];  pos0 + n_q <= n_kv
 * The mask speaks of absolute positions: the query at position i keeps key j iff j <= i and (j in I_v or i - j in I_s);
 * lists hold columns and offsets in [0, n_kv).  Running the chunks of a sequence one after the other gives, row for
 * row, the results of one call on the whole sequence (up to the order of summation).  pos0 may be any position for
 * slash_granularity 1; granularity 32 groups positions in aligned blocks of 32 and needs pos0 % 32 == 0
 * (VS_ERR_UNSUPPORTED otherwise).  Workspace: vs_sparse_prefill_workspace(q_heads, kv_heads, index_heads, n_kv).
 *
 * Batches: a batch of B sequences of equal length is B * q_heads query heads and B * kv_heads KV heads in the same
 * layout ([B, heads, n, 128] contiguous), with one index list per (sequence, index head); every call of this library
 * accepts that directly because head h always reads KV head h / (q_heads / kv_heads).
 */
int vs_sparse_prefill_chunk(const void* q, const void* k, const void* v, int q_heads, int kv_heads, int64_t n_q,
                            int64_t n_kv, int64_t pos0, float scale, const int32_t* idx_v, const int32_t* cnt_v,
                            int cap_v, const int32_t* idx_s, const int32_t* cnt_s, int cap_s, int index_heads,
                            int slash_granularity, void* o_bf16, float* lse, void* ws, size_t ws_bytes, void* stream);

/*
 * Debug check of index lists before they are given to vs_sparse_prefill / vs_aggregate (whose behaviour is undefined for
 * lists that are not strictly ascending).  One report word per head, written on the device:
 * 0 = usable, else a bit-or of the VS_LIST_* flags.  Out-of-range entries alone are legal input (they are ignored).
 *   idx [heads, cap] int32, cnt [heads] int32, report [heads] int32 out (all device memory)
 */
#define VS_LIST_BAD_COUNT 1     /* cnt < 0 or cnt > cap */
#define VS_LIST_OUT_OF_RANGE 2  /* an entry < 0 or >= n */
#define VS_LIST_NOT_ASCENDING 4 /* an entry not larger than its predecessor (unsorted or duplicate) */
int vs_validate_lists(const int32_t* idx, const int32_t* cnt, int cap, int heads, int64_t n, int32_t* report, void* stream);

/*
 * vs_sparse_prefill for callers that cannot allocate or pass a workspace: code under HIP graph capture, tight serving
 * loops, harnesses that forbid allocation.  Same arguments, results and error behaviour as vs_sparse_prefill, but the
 * scratch (bitmaps, diagonal lists, counters) lives in an array of VS_STATIC_SCRATCH_BYTES that the library holds on
 * every GPU it runs on until the process ends; the call allocates nothing and frees nothing.
 *   - A call whose vs_sparse_prefill_workspace() exceeds VS_STATIC_SCRATCH_BYTES returns VS_ERR_STATIC_LIMIT before
 *     anything is launched (32 / 8 heads with one mask per KV head fit up to n = 262144; n = 2^20 fits with one or two
 *     index heads).
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two streams, two threads)
 *     race.  Calls that follow each other on one stream are safe; every call rewrites what it reads.
 */
#define VS_STATIC_SCRATCH_BYTES (4u << 20)
int vs_sparse_prefill_static(const void* q, const void* k, const void* v, int q_heads, int kv_heads, int64_t n,
                             float scale, const int32_t* idx_v, const int32_t* cnt_v, int cap_v,
                             const int32_t* idx_s, const int32_t* cnt_s, int cap_s, int index_heads,
                             void* o_bf16, float* lse, void* stream);

/*
 * Dense causal attention on the same layout (Sec. "Attention Computation", Eqs. P, A, O, with
 * j <= i): the in-library full-attention baseline.  Same kernel pipeline as the sparse call.
 */
int vs_dense_prefill(const void* q, const void* k, const void* v, int q_heads, int kv_heads, int64_t n,
                     float scale, void* o_bf16, float* lse, void* stream);

/* The same for a chunk of n_q query rows at positions pos0 .. pos0 + n_q - 1 against n_kv keys (layouts as for
 * vs_sparse_prefill_chunk). */
int vs_dense_prefill_chunk(const void* q, const void* k, const void* v, int q_heads, int kv_heads, int64_t n_q,
                           int64_t n_kv, int64_t pos0, float scale, void* o_bf16, float* lse, void* stream);

size_t vs_aggregate_workspace(int q_heads, int kv_heads, int index_heads, int64_t n);

/*
 * Vertical-slash aggregation of the dense causal attention map (Sec. "Vertical-Slash Aggregation for Distillation
 * Training", paragraph "Obtaining Ground Truth": A = softmax(Q K^T / sqrt(d)) summed along columns and along diagonals,
 * both divided by n) and, optionally, the Attention Recall of a vertical-slash mask (Sec. "Sparse Attention
 * Formulation", Eq. R(S)).  A is never stored: it is recomputed tile by tile from Q, K and the row normalisers.
 *   q           [q_heads, n, 128] bf16;  k  [kv_heads, n, 128] bf16 (both already carry RoPE)
 *   lse         [q_heads, n] fp32 natural-log row normalisers as written by vs_dense_prefill for the same q, k and
 *               scale, or NULL: then a first sweep over the scores computes them into the workspace
 *   out_heads   q_heads: one pair of vectors per query head;  kv_heads: the mean over the query heads of each KV group
 *   a_v, a_s    [out_heads, n] fp32 out.  a_v[., j] = (1/n) sum_i A[i, j];  a_s[., o] = (1/n) sum_i A[i, i - o].
 *               Each row sums to 1.  Accumulated with float atomics: the last bits depend on the order of execution.
 *   recall      [out_heads] fp32 out or NULL.  When given, idx_v / cnt_v / cap_v / idx_s / cnt_s / cap_s / index_heads
 *               describe the mask as for vs_sparse_prefill (element-exact rule) and
 *               recall[.] = (1/n) sum over kept (i, j), j <= i, of A[i, j].  When NULL the list arguments are ignored.
 * Arithmetic: bf16 MFMA for Q K^T with fp32 accumulation, fp32 exponentials and sums.
 * Workspace from vs_aggregate_workspace (index_heads = 0 when no recall is wanted); errors as for the other calls.
 */
int vs_aggregate(const void* q, const void* k, int q_heads, int kv_heads, int64_t n, float scale, const float* lse,
                 int out_heads, float* a_v, float* a_s, const int32_t* idx_v, const int32_t* cnt_v, int cap_v,
                 const int32_t* idx_s, const int32_t* cnt_s, int cap_s, int index_heads, float* recall, void* ws,
                 size_t ws_bytes, void* stream);

size_t vs_index_train_workspace(int kv_heads, int64_t n, int d_h);

/*
 * One distillation step of the VSIndexer without the optimizer (Sec. "Vertical-Slash Aggregation for Distillation
 * Training", paragraph "Loss function design"): forward as vs_index_score, then
 *     L = (1 / kv_heads) * sum over heads of [ KL(A^_v || A_v) + KL(A^_s || A_s) ],
 *     KL(P || Q) = sum_t P_t (ln P_t - ln max(Q_t, eps))            (prediction first, as the paper prints it)
 * and the gradient of L with respect to W_U, b_U, W_V, W_S (the scalar output biases cancel in the softmax: their
 * gradient is zero).  Only the indexer is differentiated; K, V and the targets are constants (frozen backbone).
 *   k, v        [kv_heads, n, 128] bf16 as for vs_index_score
 *   t_v, t_s    [kv_heads, n] fp32 target distributions, e.g. vs_aggregate's a_v / a_s with out_heads = kv_heads
 *   eps         floor of the targets inside the logarithm (> 0)
 *   loss        [1] fp32 out (device);  dW_U [256, d_h], db_U, dW_V, dW_S [d_h] fp32 out (device, overwritten)
 * Arithmetic: the inference kernels for the forward; fp64 sums for the loss; the hidden activations are recomputed on
 * the matrix cores (W_U as two bf16 terms), pre-activation gradients enter the second contraction as two bf16 terms,
 * fp32 accumulation per workgroup and a fixed-order fp64 reduction over workgroups: the step is deterministic.
 */
int vs_index_train_step(const void* k_bf16, const void* v_bf16, int kv_heads, int64_t n, const vs_indexer_t* w,
                        const float* t_v, const float* t_s, float eps, float* loss, float* dW_U, float* db_U,
                        float* dW_V, float* dW_S, void* ws, size_t ws_bytes, void* stream);

/*
 * Number of MFMA tiles the last vs_sparse_prefill that used this workspace executed.  One tile is
 * (32 query rows of one head) x (32 keys): 1024 score elements, 4 * 128 * 1024 flop.  The kernel
 * counts them itself (tiles it skipped as fully masked are not counted).  Synchronises `stream`,
 * then copies the counter to the HOST integer `executed_tiles_host`.
 */
int vs_sparse_prefill_tiles(const void* ws, size_t ws_bytes, void* stream, int64_t* executed_tiles_host);

/*
 * The three counters of the last vs_sparse_prefill that used this workspace, copied to the HOST array counters_host[3]
 * after synchronising `stream`: [0] executed MFMA tiles (as vs_sparse_prefill_tiles), [1] 32-key tiles staged in LDS by
 * row gathers of selected columns (each is 32 rows of K and of V, 256 bytes per row: 16 KiB), [2] 32-key tiles staged
 * as contiguous key blocks of the slash part.
 */
int vs_sparse_prefill_counters(const void* ws, size_t ws_bytes, void* stream, int64_t* counters_host);

const char* vs_strerror(int status);
int vs_last_hip_error(void);
const char* vs_version(void);

#ifdef __cplusplus
}
#endif
#endif /* VSPREFILL_H */
