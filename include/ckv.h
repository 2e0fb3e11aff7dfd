/*
 * ckv.h -- C ABI of the CompilerKV prefill-end retention step for AMD MI355X (gfx950).
 *
 * The library implements the online pass of CompilerKV (paper Sec. 4, Alg. 1) for ONE layer per call
 * sequence, cut into four asynchronous calls that are queued back-to-back on one HIP stream:
 *
 *   ckv_window_scores -> ckv_apply_tables -> ckv_select_topk -> ckv_compact_kv
 *
 * Further entry points, each documented where it is declared: ckv_window_lse (the scan's first half),
 * ckv_window_utility (the first two calls as one, without the per-head masses in memory), the calls of
 * the paper's layer-shared mode (ckv_alpha_accumulate, ckv_risk_struct, ckv_shared_utility,
 * ckv_compact_kv_shared), the depth mapping of compiled tables (ckv_map_table_depth) and a decode-side consumer of the compact cache (ckv_decode_attention,
 * ckv_discarded_mass).
 *
 * Notation (paper Sec. 3-4): T = prompt length (keys/values cached at the end of prefill, the
 * observation window included), W = |Omega| = observation window (the last W query positions),
 * P = T - W = prefix length that competes for the budget, Hq / Hkv = query / key-value heads,
 * G = Hq / Hkv (query heads [g*G, (g+1)*G) share KV head g), d = head_dim, B = token budget per KV
 * head (the W window slots included), B_tot = B * Hkv = the layer's total.
 *
 * Conventions that hold for every entry point unless a comment says otherwise:
 *   - every data pointer is a DEVICE pointer owned by the caller; the library never allocates, frees
 *     or keeps device memory, keeps no state between calls and never synchronises;
 *   - `params` is a HOST pointer, read during the call only;
 *   - every call only enqueues work on `hip_stream` (a hipStream_t passed as void*; NULL = the
 *     default stream) and returns; outputs are valid once the stream reaches that point;
 *   - inputs are never written; outputs must not alias inputs or each other;
 *   - calls may be queued on different streams (and from different host threads) and overlap on the
 *     GPU as long as they share no output and no workspace: give every stream a workspace of its own
 *     (ckv_window_lse_static, whose scratch is the library's, is the exception: see there);
 *   - arguments are validated on the host BEFORE anything is launched: on any error nothing has
 *     been enqueued and the status says why (ckv_status_string gives text);
 *   - tensors are dense row-major in the order written in their comment, except Q/K/V which carry
 *     explicit (batch, head, token) strides in ELEMENTS with the head_dim axis contiguous.
 */
#ifndef CKV_H_
#define CKV_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  CKV_OK = 0,
  CKV_EINVAL = 1,       /* a null pointer, a size or a flag outside the documented domain          */
  CKV_EUNSUPPORTED = 2, /* valid, but not built (e.g. head_dim other than 64 / 128, W > 128)       */
  CKV_EWORKSPACE = 3,   /* workspace missing, misaligned (256 B) or smaller than ckv_workspace_bytes */
  CKV_EHIP = 4          /* the HIP runtime refused a launch; see hipGetLastError                   */
} ckv_status;

typedef enum { CKV_F32 = 0, CKV_BF16 = 1 } ckv_dtype;              /* element type of Q, K, V      */
typedef enum { CKV_POOL_NONE = 0, CKV_POOL_AVG = 1, CKV_POOL_MAX = 2 } ckv_pool;

/* flags */
enum {
  CKV_FLAG_VALUE_NORM = 1u, /* multiply the window mass by the value-norm ratio rho (paper Eq. 4)  */
  /* Layer-shared mode only (paper Eq. 4: alpha is a mean over heads): ckv_window_scores writes, instead
   * of every query head's mass, the SUM over the query heads of each KV head, scores [Bz,Hkv,T], and
   * ckv_alpha_accumulate reads that layout -- a quarter of the bytes for groups of four. Exists for
   * bf16 with W <= 32 and G <= 4 (CKV_EUNSUPPORTED otherwise); rejected by
   * the calls that need per-head masses (ckv_apply_tables, ckv_window_utility).                      */
  CKV_FLAG_GROUP_MASS = 8u
};

/* Problem description shared by all calls. Plain data; the caller may reuse or free it after a call. */
typedef struct {
  int32_t batch;          /* Bz >= 1                                                               */
  int32_t n_q_heads;      /* Hq, a multiple of n_kv_heads                                          */
  int32_t n_kv_heads;     /* Hkv >= 1                                                              */
  int32_t head_dim;       /* d: 64 or 128                                                          */
  int32_t seq_len;        /* T, window included; 1 <= W <= T                                       */
  int32_t window;         /* W                                                                     */
  int32_t layer;          /* row of the compiled tables used by this call, 0 <= layer < n_layers   */
  int32_t n_layers;       /* rows in w_head / head_share / t_gate                                  */
  int32_t dtype;          /* ckv_dtype of q_win, k, v, k_out, v_out                                */
  float softmax_scale;    /* logit scale; 0 selects 1/sqrt(head_dim) (paper Sec. 3)                */
  int64_t q_stride[3];    /* element strides of q_win over (batch, q head, window row)             */
  int64_t k_stride[3];    /* element strides of k over (batch, kv head, token)                     */
  int64_t v_stride[3];    /* element strides of v over (batch, kv head, token)                     */
  int32_t pool;           /* ckv_pool: 1-D pooling of the window mass along the token axis         */
  int32_t pool_kernel;    /* odd, 1..63; ignored for CKV_POOL_NONE                                 */
  int32_t budget_per_kv_head; /* B, W <= B (window slots included)                                 */
  int32_t cap;            /* rows per (batch, kv head) in idx / k_out / v_out;
                             cap >= min(T, B_tot - (Hkv-1)*W), the largest budget one head can get */
  uint32_t flags;         /* CKV_FLAG_*                                                            */
} ckv_params;

/* Bytes of scratch that ckv_window_scores and ckv_select_topk need for `params` (the larger of the
 * two; the calls of one layer may share one buffer because they run in stream order).
 * Returns 0 if `params` is NULL or invalid. The buffer must be 256-byte aligned. */
size_t ckv_workspace_bytes(const ckv_params *params);

/*
 * Observation-window scan (paper Sec. 3 attention definition, Eq. 3 "the O(LHTW) scan", Eq. 4's
 * alpha_t taken per query head, Alg. 1 step (A)).
 *
 * For every batch element b, query head h and key position t in [0, T):
 *     z[j,t]      = softmax_scale * <q_win[b,h,j,:], k[b,g(h),t,:]>            j in [0, W)
 *     A[j,t]      = exp(z[j,t] - LSE_j),  LSE_j = log sum_{t' <= P+j} exp z[j,t']   (causal: window
 *                   row j sits at absolute position P+j and sees keys t' <= P+j; A[j,t] = 0 beyond)
 *     scores[b,h,t] = (T / W) * sum_j A[j,t]
 * so that sum_t scores[b,h,t] = T (mean one, the paper's scale normalisation).
 *
 *   q_win        in   [Bz,Hq,W,d]  via q_stride; the last W query rows of the prompt
 *   k            in   [Bz,Hkv,T,d] via k_stride
 *   v            in   [Bz,Hkv,T,d] via v_stride; read only with CKV_FLAG_VALUE_NORM, else may be NULL
 *   lse          in   optional [Bz,Hq,W] fp32 natural-log LSE_j as defined above (for callers whose
 *                     prefill attention kernel already produced it); NULL = computed here with one
 *                     extra pass over K
 *   scores       out  [Bz,Hq,T] fp32
 *   vnorm_ratio  out  [Bz,Hkv,T] fp32, rho[t] = ||v_t||_2 / (mean_{t'<T} ||v_t'||_2 + 1e-6)
 *                     (paper Eq. 4, Alg. 1 Stage 1); required with CKV_FLAG_VALUE_NORM, else ignored
 *   workspace         ckv_workspace_bytes(params) bytes, contents undefined before and after
 * Accumulation is fp32 (bf16 inputs go through bf16 MFMA with fp32 accumulators).
 */
ckv_status ckv_window_scores(const ckv_params *params, const void *q_win, const void *k,
                             const void *v, const float *lse, float *scores, float *vnorm_ratio,
                             void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * First half of the scan on its own: LSE_j of every window row, as defined above (the softmax
 * normaliser of the paper's attention definition, Sec. 3), for callers that want to keep it or to
 * overlap the two passes themselves. ckv_window_scores(lse = NULL) runs exactly this internally.
 *
 *   q_win, k   in   as for ckv_window_scores
 *   lse        out  [Bz,Hq,W] fp32, natural log
 *   workspace       ckv_workspace_bytes(params) bytes
 */
ckv_status ckv_window_lse(const ckv_params *params, const void *q_win, const void *k, float *lse,
                          void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * ckv_window_lse for callers that cannot allocate device memory or hand over a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid allocation. Same arguments, same
 * kernels and bit-identical results as ckv_window_lse; the row partials of the pass live in a device
 * array inside the library (CKV_STATIC_SCRATCH_BYTES per GPU the library runs on, held until the process
 * ends) instead of a workspace. Neither this call nor anything it calls allocates or frees memory. The
 * first call on a device looks the array's address up (once per device).
 *
 * Returns CKV_EWORKSPACE, before anything is launched, when the shape needs more than the array holds:
 * ckv_window_lse_static_bytes(params) gives the need (0 for invalid params); it is
 * 8 bytes * batch * Hkv * (query rows of a KV head, padded to whole 32-row tiles) * (workgroups along
 * the key axis), e.g. 256 KiB for batch 16, 8 KV heads, 4 x 32 query rows at T = 32768.
 * Every call on one GPU uses that GPU's one array, whose contents are undefined between calls: calls
 * that overlap on one GPU (two streams, two threads) race; calls in stream order on one stream do not.
 */
#define CKV_STATIC_SCRATCH_BYTES (4u << 20)
size_t ckv_window_lse_static_bytes(const ckv_params *params);
ckv_status ckv_window_lse_static(const ckv_params *params, const void *q_win, const void *k, float *lse,
                                 void *hip_stream);

/*
 * Pooling, compiled-table lookups and budgets (paper Eq. 6 weighted max over heads, Sec. 4.3 gate
 * lookup, Alg. 1 Stages 2-3 up to the threshold; the 1-D pooling and the per-head budget split are
 * the build's workload definition, not the paper's).
 *
 * For every b, kv head g and prefix position t in [0, P):
 *     c[h,t]  = pool_k(scores[b,h,0:P])[t]   centred, stride 1, same length; AVG divides by
 *               pool_kernel with zeros outside [0,P); MAX ignores positions outside [0,P)
 *     u[h,t]  = c[h,t] * vnorm_ratio[b,g,t]  (with CKV_FLAG_VALUE_NORM, else u = c)
 *     utility[b,g,t] = max_{h in group g} fp32(w_head[layer,h] * u[h,t])
 * and
 *     tau[b]  = t_gate[layer, risk_bins[b,0], risk_bins[b,1]]       (0 if t_gate is NULL: gate off)
 *     budget[b,g]: NULL head_share => min(B, T). Else b_g = floor(head_share[layer,g] * B_tot) evaluated in
 *               fp64, clamped to [W, T]; while sum_g b_g > B_tot the largest b_g that is > W (lowest
 *               g on ties) is decremented by one.
 *
 *   scores       in   [Bz,Hq,T] fp32 (from ckv_window_scores)
 *   vnorm_ratio  in   [Bz,Hkv,T] fp32, required with CKV_FLAG_VALUE_NORM
 *   w_head       in   [n_layers,Hq] fp32, finite and > 0 (paper grid: [0.8,1.5])
 *   head_share   in   [n_layers,Hkv] fp32 >= 0, or NULL
 *   t_gate       in   [n_layers,n_ent,n_ppl] fp32 >= 0 (paper grid: 20 x 4, values in [0.8,1.0]), or NULL
 *   risk_bins    in   [Bz,2] int32 (b_ent, b_ppl), required with t_gate; out-of-range bins are
 *                     clamped into the table on the device (they cannot be checked on the host)
 *   utility      out  [Bz,Hkv,P] fp32
 *   budget       out  [Bz,Hkv] int32
 *   tau          out  [Bz] fp32
 */
ckv_status ckv_apply_tables(const ckv_params *params, const float *scores, const float *vnorm_ratio,
                            const float *w_head, const float *head_share, const float *t_gate,
                            int32_t n_ent, int32_t n_ppl, const int32_t *risk_bins, float *utility,
                            int32_t *budget, float *tau, void *hip_stream);

/*
 * ckv_window_scores followed by ckv_apply_tables as ONE call that does not materialise the per-head
 * window mass: same definitions, same utility / budget / tau (within fp32 rounding of the pooled sum),
 * for callers that only need what the selection consumes (paper Alg. 1 from the window scan up to the
 * threshold). Where the shape allows it (bf16, W <= 64, G*ceil(W/32) <= 8, pooling kernel <= 7, T and
 * P multiples of four) the scan's second pass pools, weights and maximises over the group's heads on
 * chip and writes [Bz,Hkv,P] instead of [Bz,Hq,T] (with CKV_FLAG_VALUE_NORM the ratio, common to a
 * group's heads, then multiplies the group maximum); otherwise the two steps run one after the other
 * through `scores_scratch`.
 *
 *   q_win, k, v, lse                                   as for ckv_window_scores
 *   w_head, head_share, t_gate, n_ent, n_ppl, risk_bins as for ckv_apply_tables
 *   scores_scratch  scratch  [Bz,Hq,T] fp32; contents undefined on return (the fused pass leaves raw
 *                            column sums in parts of it only)
 *   vnorm_ratio     out      as for ckv_window_scores (required with CKV_FLAG_VALUE_NORM, else ignored)
 *   utility, budget, tau  out  as for ckv_apply_tables
 *   workspace                ckv_workspace_bytes(params) bytes
 */
ckv_status ckv_window_utility(const ckv_params *params, const void *q_win, const void *k, const void *v,
                              const float *lse, const float *w_head, const float *head_share,
                              const float *t_gate, int32_t n_ent, int32_t n_ppl, const int32_t *risk_bins,
                              float *scores_scratch, float *vnorm_ratio, float *utility, int32_t *budget,
                              float *tau, void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Elastic candidate pool with budget clamp (paper Eq. 8, Alg. 1 Select), per (b, kv head g):
 *     cand = { t < P : utility[b,g,t] >= tau[b] },  kp = budget[b,g] - W
 *     Sp   = cand                                         if |cand| <= kp
 *          = the kp members of cand that come first under (utility descending, t ascending) otherwise
 *     idx[b,g,:] = Sp in ascending t, then the window P..T-1;   count[b,g] = |Sp| + W
 * Utilities must be non-negative and not NaN (they are sums of softmax weights times positive
 * weights); the order of equal utilities is by position, so the result is unique.
 *
 *   utility  in   [Bz,Hkv,P] fp32      budget in [Bz,Hkv] int32 (values are clamped to [W, min(cap,T)]
 *   tau      in   [Bz] fp32                       on the device)
 *   idx      out  [Bz,Hkv,cap] int32; entries at and beyond count[b,g] are not written
 *   count    out  [Bz,Hkv] int32
 *   workspace     optional (NULL allowed). Up to 32768 prefix positions it is not used. Beyond that,
 *                 with ckv_workspace_bytes(params) bytes (256-byte aligned; CKV_EWORKSPACE if
 *                 misaligned or smaller) a unit's positions are split over several workgroups, which is
 *                 several times faster for long contexts with few (batch, head) units; the result is
 *                 the same either way. Contents on entry are ignored.
 */
ckv_status ckv_select_topk(const ckv_params *params, const float *utility, const int32_t *budget,
                           const float *tau, int32_t *idx, int32_t *count, void *workspace,
                           size_t workspace_bytes, void *hip_stream);

/*
 * Token-axis gather (paper Sec. 3 "K~ = K[S], V~ = V[S]", Alg. 1 Gather_tok): for r < count[b,g]
 *     k_out[b,g,r,:] = k[b,g,idx[b,g,r],:]    v_out[b,g,r,:] = v[b,g,idx[b,g,r],:]     (bit copies)
 *
 *   k, v          in   via k_stride / v_stride
 *   idx, count    in   from ckv_select_topk; indices outside [0,T) are skipped on the device
 *   k_out, v_out  out  [Bz,Hkv,cap,d] dense, same dtype; rows at and beyond count are not written
 */
ckv_status ckv_compact_kv(const ckv_params *params, const void *k, const void *v, const int32_t *idx,
                          const int32_t *count, void *k_out, void *v_out, void *hip_stream);

/*
 * Layer-shared mode: the paper's Alg. 1 as printed, where ONE window mass alpha serves every layer and
 * head and every layer keeps ONE index set for all its heads. Order of calls for a prompt:
 *   for each layer: ckv_window_scores (with CKV_FLAG_VALUE_NORM: rho of that layer) and
 *                   ckv_alpha_accumulate(weight = 1 / (n_layers * Hq))                  -- Alg. 1 (A)
 *   once:           ckv_risk_struct                                                     -- Alg. 1 (A)
 *   for each layer: ckv_shared_utility, ckv_select_topk with a one-head ckv_params (batch, 1 query head,
 *                   1 KV head, budget = B_l; utility [Bz,1,P], budget [Bz,1]), ckv_compact_kv_shared.
 *
 * ckv_alpha_accumulate: alpha[b,t] += weight * sum_h scores[b,h,t] (with CKV_FLAG_GROUP_MASS: the sum
 * over the Hkv rows of the group-mass layout). With weight = 1/(L*Hq) over all
 * layers this is alpha = (T/W) sum_{j in Omega} Abar[j,:] for Abar the mean of A over layers and heads
 * (paper Eq. 4, Alg. 1 (A)); sum_t alpha = T.
 *   scores  in      [Bz,Hq,T] fp32 of one layer (from ckv_window_scores)
 *   alpha   in/out  [Bz,T] fp32; the caller clears it before the first layer
 */
ckv_status ckv_alpha_accumulate(const ckv_params *params, const float *scores, float weight, float *alpha,
                                void *hip_stream);

/*
 * Structural risk coordinate (paper Eq. 7, Alg. 1 (A)): risk[b] = -sum_t A'_t ln A'_t with
 * A' = alpha[b,:] / ||alpha[b,:]||_1 (terms with A'_t = 0 count as 0), and its bin
 * bin[b] = number of ent_edges <= risk[b] (ascending edges chosen by whoever compiled T_gate; the
 * paper does not fix them). Sums are formed in fp64 in a fixed order.
 *   alpha      in   [Bz,T] fp32, non-negative
 *   ent_edges  in   [n_edges] fp32 ascending (device), may be NULL when bin is NULL or n_edges = 0
 *   risk       out  [Bz] fp32           bin  out  [Bz] int32, or NULL
 */
ckv_status ckv_risk_struct(const ckv_params *params, const float *alpha, const float *ent_edges,
                           int32_t n_edges, float *risk, int32_t *bin, void *hip_stream);

/*
 * One utility vector per layer (paper Eq. 4 u = alpha * rho, Eq. 6, Alg. 1 (B)-(C)) and the gate
 * lookup (Sec. 4.3): for t in [0, P)
 *     utility[b,t] = max over ALL query heads h of fp32(w_head[layer,h] * (alpha[b,t] * vnorm_ratio[b,g(h),t]))
 *     tau[b]       = t_gate[layer, risk_bins[b,0], risk_bins[b,1]]      (0 if t_gate is NULL)
 * (the pooling fields of params are not used: the paper has no pooling).
 *   alpha        in   [Bz,T] fp32          vnorm_ratio  in  [Bz,Hkv,T] fp32 of this layer
 *   w_head, t_gate, n_ent, n_ppl, risk_bins   as for ckv_apply_tables
 *   utility      out  [Bz,P] fp32          tau  out  [Bz] fp32
 */
ckv_status ckv_shared_utility(const ckv_params *params, const float *alpha, const float *vnorm_ratio,
                              const float *w_head, const float *t_gate, int32_t n_ent, int32_t n_ppl,
                              const int32_t *risk_bins, float *utility, float *tau, void *hip_stream);

/*
 * Gather with one index set per batch element, shared by all KV heads of the layer (paper Alg. 1,
 * Gather_tok: one index set per layer serves every head): for r < count[b], every g
 *     k_out[b,g,r,:] = k[b,g,idx[b,r],:]    v_out[b,g,r,:] = v[b,g,idx[b,r],:]     (bit copies)
 *   idx  in  [Bz,cap] int32      count  in  [Bz] int32      k_out, v_out  out  [Bz,Hkv,cap,d]
 */
ckv_status ckv_compact_kv_shared(const ckv_params *params, const void *k, const void *v, const int32_t *idx,
                                 const int32_t *count, void *k_out, void *v_out, void *hip_stream);

/*
 * Depth mapping of a compiled table (paper App. "Model choice and cross-architecture applicability": tables
 * are compiled on a 32-layer backbone; models of another depth use a monotonic depth mapping, relative-
 * depth interpolation). mapped[l,:] is the linear interpolation of the two rows of `table` next to the
 * source coordinate x = l * (n_layers_src - 1) / (n_layers_dst - 1) (row 0 for n_layers_dst = 1). Works
 * for w_head ([L,Hq]: row_elems = Hq), head_share ([L,Hkv]) and t_gate ([L,n_ent,n_ppl]: row_elems =
 * n_ent * n_ppl). Table preparation, run once per model.
 *   table  in  [n_layers_src,row_elems] fp32      mapped  out  [n_layers_dst,row_elems] fp32
 */
ckv_status ckv_map_table_depth(const float *table, int32_t n_layers_src, int32_t row_elems, float *mapped,
                               int32_t n_layers_dst, void *hip_stream);

/*
 * Decode-side consumer of the compact cache (paper Sec. 4.5, Proposition 1; proof in App. A).
 *
 * ckv_decode_attention: attention of decoding queries over a ragged KV set. A decoding query sits after
 * the prompt and sees every row. For batch element b, query head h (KV head g = h / G), query i < n_q:
 *     z[j]   = softmax_scale * <q_dec[b,h,i,:], k_rows[b,g,j,:]>          j < n_valid(b,g)
 *     lse    = log sum_j exp z[j]
 *     out    = sum_j exp(z[j] - lse) * v_rows[b,g,j,:]
 * with n_valid(b,g) = count[b,g] clamped to [0, n_rows] (n_rows if count is NULL). Over the compact
 * cache written by ckv_compact_kv (strides {Hkv*cap*d, cap*d, d}, n_rows = cap, the call's count) this
 * is the compressed row of Proposition 1, p~ = p restricted to the retained set and renormalised,
 * applied to V; over the full cache (params' k_stride / v_stride, n_rows = T, count = NULL) it is the
 * uncompressed attention and its lse is the full row's normaliser.
 *
 *   q_dec     in   [Bz,Hq,n_q,d] contiguous, params->dtype, 16-byte aligned
 *   k_rows, v_rows in  rows of (batch, kv head) at element strides k_stride / v_stride over
 *                  (batch, kv head, row); multiples of 16 bytes, row stride >= d; 16-byte aligned
 *   count     in   [Bz,Hkv] int32 or NULL
 *   out       out  [Bz,Hq,n_q,d] fp32 (zeros where no row is valid)
 *   lse       out  [Bz,Hq,n_q] fp32, natural log (-inf where no row is valid)
 *   workspace      ckv_decode_workspace_bytes(params, n_q, n_rows) bytes, 256-byte aligned. That
 *                  function returns 0 for arguments this call rejects, and also for short KV sets
 *                  (n_rows <= 4096), which one launch finishes without scratch: workspace may then
 *                  be NULL.
 *
 * ckv_discarded_mass: m[b,h,i] = 1 - exp(lse_kept - lse_full), the mass the full attention row had
 * outside the retained set (Proposition 1; the row's l1 error is exactly 2m), clamped to [0,1], and
 * eps_tail[b,h] = sqrt(mean_i m^2) (may be NULL).
 *   lse_full, lse_kept  in  [Bz,Hq,n_q] fp32     mass out [Bz,Hq,n_q] fp32     eps_tail out [Bz,Hq] fp32
 */
size_t ckv_decode_workspace_bytes(const ckv_params *params, int32_t n_q, int32_t n_rows);
ckv_status ckv_decode_attention(const ckv_params *params, const void *q_dec, int32_t n_q, const void *k_rows,
                                const void *v_rows, const int64_t *k_stride, const int64_t *v_stride,
                                int32_t n_rows, const int32_t *count, float *out, float *lse, void *workspace,
                                size_t workspace_bytes, void *hip_stream);
ckv_status ckv_discarded_mass(const ckv_params *params, int32_t n_q, const float *lse_full, const float *lse_kept,
                              float *mass, float *eps_tail, void *hip_stream);

/* Static text for a status code; never NULL. */
const char *ckv_status_string(ckv_status status);

#ifdef __cplusplus
}
#endif
#endif /* CKV_H_ */
