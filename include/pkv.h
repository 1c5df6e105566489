/*
 * pkv.h -- C ABI of libpkv: PyramidKV prefill-time KV-cache compression
 * (arXiv 2406.02069) for AMD MI355X (gfx950).
 *
 * For every transformer layer l the library keeps k^l of the n cached tokens
 * of each KV head: the last alpha "instruction" tokens, plus the k^l - alpha
 * prefix tokens that receive the most softmax attention from the instruction
 * queries (Sec. 4.2.2).  The per-layer budgets k^l follow the paper's
 * arithmetic "pyramid" (Sec. 4.2.1).  The kept K/V rows are copied, in
 * ascending position order, into a new smaller cache (appendix "Details of
 * Proposed Method": eviction by gather; appendix on rotary embeddings: kept
 * rows are not re-rotated and positions stay ascending).
 *
 * Conventions
 *  - Plain C, no C++/torch types.  Every function returns a pkv_status
 *    (0 = ok) except the pure size/string helpers.
 *  - Pointers marked DEVICE must be device memory owned by the caller and
 *    stay valid until the work queued on `stream` has finished.  Pointers
 *    marked HOST are read/written synchronously during the call.
 *  - Argument errors are detected on the host before anything is launched
 *    and leave all outputs untouched.
 *  - Launching calls are asynchronous on `stream` (a hipStream_t passed as
 *    void*; NULL = the default stream).  They never synchronise and never
 *    allocate or free memory.  Results are deterministic: the same inputs
 *    give bit-identical outputs.
 *  - Inputs are never modified.
 *  - The library keeps no state between calls and reads no environment
 *    variables.  (The per-device attributes of its kernels are set on first
 *    use; pkv_compress_layer_noalloc has a built-in scratch buffer per device,
 *    see there.)
 *  - Exclusive use of the device.  Whenever a device with at least 256
 *    compute units is given a shape the register-resident scoring kernel
 *    serves (G*alpha <= 512, N <= 262144) without supplied softmax
 *    denominators, that kernel's 512 workgroups exchange softmax statistics
 *    with each other and must all be resident on the device at the same
 *    time; they fill it completely (registers and LDS of every compute
 *    unit).  The caller must therefore not run other kernels on the device
 *    while such a call executes: no second compress call on another stream,
 *    no other tenant.  Work queued behind it on the same stream is fine.
 *    If the workgroups cannot all be resident, the waits between them are
 *    given up after about 50 ms of wall-clock time each, the call completes,
 *    and every count_out of the call reads -1 (see pkv_compress_layer); it
 *    never hangs.  The variants with supplied denominators
 *    (pkv_compress_layers_lse) have no such waits and share the device
 *    freely.
 */
#ifndef PKV_H_
#define PKV_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  PKV_OK = 0,
  PKV_ERR_INVALID_ARG = 1, /* NULL pointer, bad size, bad stride, bad enum   */
  PKV_ERR_UNSUPPORTED = 2, /* valid in the paper's terms, not built here     */
  PKV_ERR_WORKSPACE = 3,   /* workspace NULL, misaligned or too small        */
  PKV_ERR_HIP = 4,         /* a kernel launch was rejected by the runtime    */
  PKV_ERR_SCRATCH = 5      /* shape needs more than the built-in scratch
                              buffer of pkv_compress_layer_noalloc holds     */
} pkv_status;

typedef enum {
  PKV_POOL_NONE = 0,
  PKV_POOL_MAX = 1,
  PKV_POOL_AVG = 2
} pkv_pool;

/*
 * Per-layer budgets (Sec. 4.2.1, Eq. budget).  HOST only, pure.
 *
 * The alpha instruction tokens are kept in every layer; the pyramid is laid
 * over the remaining A = avg_budget - alpha entries per layer
 * (k_total = L*A): top layer A/beta, bottom layer 2A - A/beta, arithmetic
 * sequence in between.  The real-valued sequence is made integer by flooring
 * and handing the missing units to the layers with the largest fractional
 * parts (ties to the lower layer), so that
 *     sum_l k_out[l] == L * avg_budget   and   k_out[l] >= k_out[l+1].
 * k_out[l] INCLUDES the alpha instruction tokens.  L == 1 gives avg_budget;
 * beta == 1 gives a uniform budget.
 *
 * k_out: HOST, int32[L], written.
 * Errors: L < 1, beta < 1, alpha < 0, avg_budget < alpha, k_out NULL
 *         -> PKV_ERR_INVALID_ARG.
 */
int pkv_budgets(int32_t L, int32_t avg_budget, int32_t beta, int32_t alpha,
                int32_t* k_out);

/*
 * Other allocation strategies of the paper's ablation (appendix "Allocation
 * Strategies", which names a geometric and an exponential decay beside the
 * linear one without a formula; written in the layer index both are
 * r_l = C * q^l, so one schedule stands for the two).
 *   PKV_SCHEDULE_LINEAR     pkv_budgets
 *   PKV_SCHEDULE_GEOMETRIC  r_l = C * q^l over A = avg_budget - alpha, with the
 *                           linear pyramid's ratio of top to bottom layer,
 *                           q^(L-1) = 1/(2 beta - 1), and sum_l r_l = L*A
 *   PKV_SCHEDULE_UNIFORM    k_out[l] = avg_budget (SnapKV-style selection)
 * Integerisation, k_out, ownership and errors as pkv_budgets; an unknown
 * schedule -> PKV_ERR_INVALID_ARG.
 */
typedef enum {
  PKV_SCHEDULE_LINEAR = 0,
  PKV_SCHEDULE_GEOMETRIC = 1,
  PKV_SCHEDULE_UNIFORM = 2
} pkv_schedule;

int pkv_budgets_schedule(int32_t L, int32_t avg_budget, int32_t beta,
                         int32_t alpha, int32_t schedule, int32_t* k_out);

/*
 * Shape of one layer's compression problem.  Strides are in ELEMENTS (bf16);
 * the head dimension is always contiguous.
 */
typedef struct {
  int32_t B;      /* sequences in the batch, >= 1                            */
  int32_t Hq;     /* query heads; Hq % Hkv == 0                              */
  int32_t Hkv;    /* key/value heads                                         */
  int32_t d;      /* head dimension d_k: 64 or 128                           */
  int32_t N;      /* (padded) cached length of K and V, >= 1                 */
  int32_t alpha;  /* instruction-token window, 1 <= alpha <= 64              */
  int32_t k_l;    /* this layer's budget including the window, >= alpha      */
  int32_t pool;   /* pkv_pool                                                */
  int32_t pool_w; /* pooling width, odd, 1..63 (1 == no pooling)             */
  int32_t flags;  /* 0.  (Test and measurement switches, pkv_measure.h:
                     bits outside PKV_FLAG_ALL -> PKV_ERR_INVALID_ARG)       */
  int64_t q_sb, q_sh, q_st;    /* strides of Q_win [B, Hq, alpha, d]         */
  int64_t kv_sb, kv_sh, kv_st; /* strides of K and of V [B, Hkv, N, d]       */
  int64_t o_sb, o_sh, o_st;    /* strides of K_out and V_out
                                  [B, Hkv, k_cap, d], k_cap = min(k_l, N)    */
} pkv_layer_desc;

/*
 * Bytes of DEVICE workspace needed to compress L layers of this shape in one
 * call (L = 1 for pkv_compress_layer), whatever their budgets k_l.
 * HOST only, pure.  Returns 0 if the descriptor is invalid or L is not in
 * 1..1024.
 */
size_t pkv_workspace_bytes(const pkv_layer_desc* desc, int32_t L);

/*
 * Compress one layer (Sec. 4.2.2; gather per the appendix "Details of
 * Proposed Method").
 *
 * For each sequence b with n = seq_lens[b] valid tokens and each KV head g
 * (G = Hq/Hkv query heads h = g*G .. g*G+G-1 share it):
 *   1. if k_l >= n every token is kept;
 *   2. otherwise each window query t (absolute position n-alpha+t) attends
 *      causally: A = softmax over keys 0..n-alpha+t of q.k / sqrt(d)
 *      (Eq. Al), window keys included;
 *   3. s^h_i = sum_t A^{(h,t)}_i for prefix keys i < n-alpha (Eq. att_score),
 *      averaged over the G heads of the group;
 *   4. the scores are pooled along the sequence (stride 1, same length; max
 *      ignores out-of-range neighbours, avg counts them as zero and divides
 *      by pool_w);
 *   5. the k_l-alpha prefix positions with the largest pooled score are
 *      kept (equal scores: the lower position wins), in ascending order,
 *      followed by the window positions n-alpha .. n-1;
 *   6. K_out/V_out rows are bit copies of the kept K/V rows.
 * Arithmetic: bf16 inputs, fp32 accumulation and scores.
 *
 * desc       HOST.
 * Q_win      DEVICE bf16 [B,Hq,alpha,d]: queries of the LAST alpha valid
 *            tokens of each sequence (positions n_b-alpha .. n_b-1), as used
 *            by attention (after any rotary embedding).
 * K, V       DEVICE bf16 [B,Hkv,N,d], same strides.  Rows >= n_b are never
 *            read.  V is read only at the kept rows.
 * seq_lens   DEVICE int32[B] with 0 <= n_b <= N, or NULL (all n_b == N).
 *            Values outside the range are clamped on the device.
 *            If n_b <= k_l all n_b tokens are kept (this covers n_b < alpha).
 * K_out,V_out DEVICE bf16 [B,Hkv,k_cap,d], written.  Rows >= count are zero.
 * idx_out    DEVICE int32 [B,Hkv,k_cap] contiguous, written: kept positions,
 *            ascending; the last min(alpha,n_b) valid entries are the window;
 *            entries >= count are -1.
 * count_out  DEVICE int32 [B], written: min(k_l, n_b); or -1 for every
 *            sequence if the scoring kernel had to give up a wait between
 *            its workgroups (they exchange softmax statistics and rely on
 *            being resident on the device together; another tenant of the
 *            device can prevent that).  Every wait is bounded, so the call
 *            always completes; with count -1 the other outputs of the call
 *            are in range but meaningless and the call should be repeated.
 * scores_out DEVICE fp32 [B,Hkv,N] contiguous, or NULL: pooled scores before
 *            selection, defined for i < n_b-alpha when k_l < n_b; other
 *            entries are left untouched.
 * workspace  DEVICE, 256-byte aligned, >= pkv_workspace_bytes(desc, 1) bytes;
 *            contents on entry are irrelevant, contents on exit undefined
 *            (except as pkv_attention_recall uses them).
 *            Calls that may overlap in time need distinct workspaces (and
 *            see "Exclusive use of the device" above).
 * stream     hipStream_t.
 *
 * Errors: PKV_ERR_INVALID_ARG (NULL required pointer, shape/stride rules
 * above violated, unknown flags), PKV_ERR_UNSUPPORTED (d not 64/128,
 * alpha > 64, pool_w > 63), PKV_ERR_WORKSPACE, PKV_ERR_HIP.
 */
int pkv_compress_layer(const pkv_layer_desc* desc, const void* Q_win,
                       const void* K, const void* V, const int32_t* seq_lens,
                       void* K_out, void* V_out, int32_t* idx_out,
                       int32_t* count_out, float* scores_out, void* workspace,
                       size_t workspace_bytes, void* stream);

/*
 * pkv_compress_layer for callers that cannot hand over a workspace and must
 * not cause an allocation: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, results and errors as
 * pkv_compress_layer, without the workspace: the kernels use a scratch
 * buffer of PKV_NOALLOC_SCRATCH_BYTES that is part of the library's device
 * image (every device the library runs on holds one until the process ends).
 * The call allocates and frees nothing, on the host or on the device.
 *
 * A shape whose pkv_workspace_bytes(desc, 1) exceeds
 * PKV_NOALLOC_SCRATCH_BYTES -> PKV_ERR_SCRATCH, nothing launched.  (32 MiB
 * serve, e.g., B*Hkv = 8 heads of 262144 keys, or 64 heads of 32768.)
 * All calls on one device share that device's buffer: calls that may overlap
 * in time on one device race and give undefined results; serialise them (one
 * stream, or events).  The buffer keeps the last call's contents; the call
 * clears what it needs cleared itself.
 */
#define PKV_NOALLOC_SCRATCH_BYTES ((size_t)32 << 20)

int pkv_compress_layer_noalloc(const pkv_layer_desc* desc, const void* Q_win,
                               const void* K, const void* V,
                               const int32_t* seq_lens, void* K_out,
                               void* V_out, int32_t* idx_out,
                               int32_t* count_out, float* scores_out,
                               void* stream);

/*
 * Compress L layers of one request batch (the whole prefill-time step: every
 * layer has its own Q_win/K/V and its own budget descs[l].k_l, Sec. 4.2.1).
 * Same results as L calls of pkv_compress_layer, queued so that independent
 * stages of neighbouring layers can overlap on the device.
 *
 * descs      HOST, L descriptors.  All fields except k_l and the output
 *            strides must be equal across layers.
 * Q_win, K, V, K_out, V_out, idx_out, count_out, scores_out
 *            HOST arrays of L DEVICE pointers, each as in
 *            pkv_compress_layer (scores_out may be NULL, or hold NULLs).
 * seq_lens   DEVICE int32[B] or NULL; shared by all layers.
 * workspace  DEVICE, >= pkv_workspace_bytes(&descs[0], L) bytes.
 * Errors: as pkv_compress_layer; additionally L outside 1..1024 or differing
 * layer shapes -> PKV_ERR_INVALID_ARG.
 */
int pkv_compress_layers(int32_t L, const pkv_layer_desc* descs,
                        const void* const* Q_win, const void* const* K,
                        const void* const* V, const int32_t* seq_lens,
                        void* const* K_out, void* const* V_out,
                        int32_t* const* idx_out, int32_t* const* count_out,
                        float* const* scores_out, void* workspace,
                        size_t workspace_bytes, void* stream);

/*
 * pkv_compress_layers with the softmax denominators of the window queries
 * supplied by the caller.  The scores of Sec. 4.2.2 are taken from the
 * attention of the instruction tokens, which prefill has already computed;
 * an attention kernel that keeps its per-row log-sum-exp hands it over here,
 * and the keys are then swept once instead of twice (no statistics sweep, no
 * exchange between workgroups).
 *
 * lse        HOST array of L DEVICE pointers, each fp32 [B,Hq,alpha]
 *            contiguous: lse[b][h][t] = ln sum_{i <= n_b-alpha+t}
 *            exp(q_{b,h,t} . k_{b,g(h),i} / sqrt(d)), the natural log of the
 *            denominator of window query t's causal softmax (Eq. Al), window
 *            keys included.  The attention of step 2 becomes
 *            exp(q.k/sqrt(d) - lse) and is not renormalised: results equal
 *            pkv_compress_layers' to the accuracy of the supplied values.
 *            Entries of sequences with n_b <= k_l are not read.  Non-finite
 *            entries give meaningless (but in-range) selections.
 * Everything else, and the errors, as pkv_compress_layers; a NULL lse or a
 * NULL or misaligned lse[l] -> PKV_ERR_INVALID_ARG.  count_out is never -1
 * here (nothing waits).
 */
int pkv_compress_layers_lse(int32_t L, const pkv_layer_desc* descs,
                            const void* const* Q_win, const void* const* K,
                            const void* const* V, const float* const* lse,
                            const int32_t* seq_lens, void* const* K_out,
                            void* const* V_out, int32_t* const* idx_out,
                            int32_t* const* count_out,
                            float* const* scores_out, void* workspace,
                            size_t workspace_bytes, void* stream);

/*
 * Per-layer paged output (appendix "PyramidKV Implementation at vLLM": every
 * layer keeps a different number of tokens, so every layer gets its own
 * block table and page pool instead of a share of one uniform paged cache).
 * As pkv_compress_layers (lse NULL) or pkv_compress_layers_lse (lse given),
 * except that the kept rows go straight into pages:
 *   kept row j (0 <= j < count_b) of sequence b, KV head g, layer l
 *     -> K_pages[l] / V_pages[l], page block_tables[l][b][j / page_size],
 *        head g, slot j % page_size.
 * Nothing else in the pools is written (a partly filled last page keeps its
 * old content behind the kept rows); descs[l].o_* are checked as usual but
 * not used.
 */
typedef struct {
  int32_t page_size; /* tokens per page, >= 1                                */
  int32_t num_pages; /* pages in each layer's pool                           */
  int32_t max_pages; /* entries per sequence in each block table,
                        >= ceil(min(k_l, N) / page_size) for every layer     */
  int32_t reserved;  /* must be 0                                            */
} pkv_paged_desc;

/*
 * paged        HOST.
 * K_pages, V_pages
 *              HOST arrays of L DEVICE pointers, each bf16
 *              [num_pages, Hkv, page_size, d] contiguous, 16-byte aligned.
 * block_tables HOST array of L DEVICE pointers, each int32 [B, max_pages]
 *              contiguous: page numbers in [0, num_pages).  Entries beyond
 *              ceil(count_b / page_size) are not read.  A page number out of
 *              range is never written through: the row is dropped and
 *              count_out[l][b] is set to -2.
 * idx_out, count_out, scores_out, seq_lens, workspace, stream: as
 * pkv_compress_layers.
 * Errors: as pkv_compress_layers(_lse); paged NULL or inconsistent (sizes
 * < 1, reserved != 0, max_pages too small for a layer's budget), a NULL or
 * misaligned table -> PKV_ERR_INVALID_ARG.
 */
int pkv_compress_layers_paged(int32_t L, const pkv_layer_desc* descs,
                              const void* const* Q_win, const void* const* K,
                              const void* const* V, const float* const* lse,
                              const int32_t* seq_lens,
                              const pkv_paged_desc* paged,
                              void* const* K_pages, void* const* V_pages,
                              const int32_t* const* block_tables,
                              int32_t* const* idx_out,
                              int32_t* const* count_out,
                              float* const* scores_out, void* workspace,
                              size_t workspace_bytes, void* stream);

/*
 * Attention recall rate of the kept sets (appendix, "Attention Recall Rate
 * Experiment"): the share of the window queries' attention over all keys
 * that falls on the kept keys, averaged over the G*alpha window queries of
 * a KV head: 1 - (window score mass on the dropped prefix keys) / alpha.
 *
 * Call it right after a pkv_compress_layers / _lse / _paged call, with the
 * same L, descs, seq_lens and workspace, on the same stream and before
 * anything else uses the workspace: it reads the un-pooled window scores
 * that the call left there, and the call's idx_out.
 *
 * lse_supplied 1 if the call was given lse, else 0.
 * idx_out      HOST array of L DEVICE pointers: the call's idx_out.
 * recall_out   HOST array of L DEVICE pointers, each fp32 [B,Hkv], written:
 *              1 for sequences that keep everything.
 * Errors: as pkv_compress_layers for descs, pointers and workspace.
 */
int pkv_attention_recall(int32_t L, const pkv_layer_desc* descs,
                         int32_t lse_supplied, const int32_t* seq_lens,
                         const int32_t* const* idx_out,
                         float* const* recall_out, const void* workspace,
                         size_t workspace_bytes, void* stream);

/*
 * The step after the path: decoding attention of one new query per sequence
 * over a layer's compacted cache (Sec. 3: after compression the model attends
 * over the kept keys and values only).  The kept rows carry the rotary phases
 * of their original positions, so q is taken as given (rotated at its own
 * position by the caller) and nothing is re-rotated.
 *   out[b][h] = sum_{j < count_b} softmax_j(q_bh . K_bgj / sqrt(d)) V_bgj,
 *   g = h / (Hq/Hkv);  fp32 accumulation and output.
 * The cache is what pkv_compress_layer(s) wrote (page_size 0: compact
 * [B,Hkv,k_cap,d] with strides c_*) or what pkv_compress_layers_paged wrote
 * (page_size > 0: pool [num_pages,Hkv,page_size,d] with this layer's block
 * table; a page number out of range makes its rows count as absent).
 */
typedef struct {
  int32_t B, Hq, Hkv; /* Hq % Hkv == 0, Hq/Hkv <= 8                          */
  int32_t d;          /* 64 or 128                                           */
  int32_t k_cap;      /* rows per sequence the cache can hold, <= 4096       */
  int32_t page_size;  /* 0: compact cache; > 0: paged                        */
  int32_t num_pages;  /* paged: pages in the pool                            */
  int32_t max_pages;  /* paged: entries per sequence in the block table,
                         >= ceil(k_cap / page_size)                          */
  int32_t reserved;   /* must be 0                                           */
  int32_t reserved2;  /* padding, ignored                                    */
  int64_t c_sb, c_sh, c_st; /* compact: element strides of K_cache/V_cache   */
} pkv_decode_desc;

/*
 * Bytes of DEVICE workspace pkv_decode_attention needs for this shape (0 for
 * shapes it serves with one workgroup per sequence and head; 0 as well if
 * the descriptor is invalid).  HOST only, pure.
 */
size_t pkv_decode_workspace_bytes(const pkv_decode_desc* desc);

/*
 * desc        HOST.
 * q           DEVICE bf16 [B,Hq,d] contiguous, 16-byte aligned.
 * K_cache, V_cache  DEVICE bf16, layouts above, 16-byte aligned.
 * block_table DEVICE int32 [B,max_pages] (paged) or NULL (compact).
 * count       DEVICE int32 [B]: valid rows per sequence (count_out of the
 *             compression call); values outside [0, k_cap] are clamped, so
 *             the error codes -1 / -2 read as an empty cache.
 * out         DEVICE fp32 [B,Hq,d] contiguous, written (zero rows for an
 *             empty cache).
 * lse_out     DEVICE fp32 [B,Hq] or NULL: natural log of the softmax
 *             denominator (-inf for an empty cache).
 * workspace   DEVICE, 256-byte aligned, >= pkv_decode_workspace_bytes(desc)
 *             bytes (may be NULL when that is 0); contents irrelevant on
 *             entry, undefined on exit; concurrent calls need distinct ones.
 * stream      hipStream_t.  Asynchronous, never allocates.
 * Errors: PKV_ERR_INVALID_ARG (NULL / misaligned pointers, shape or stride
 * rules violated), PKV_ERR_UNSUPPORTED (d, Hq/Hkv > 8, k_cap > 4096),
 * PKV_ERR_WORKSPACE, PKV_ERR_HIP.
 */
int pkv_decode_attention(const pkv_decode_desc* desc, const void* q,
                         const void* K_cache, const void* V_cache,
                         const int32_t* block_table, const int32_t* count,
                         float* out, float* lse_out, void* workspace,
                         size_t workspace_bytes, void* stream);

/*
 * pkv_decode_attention over the caches of L layers in one call (Sec. 3; the
 * per-layer budgets of Sec. 4.2.1 make the layers' caches unequal and, at
 * small batch, small: a launch per layer costs more than the rows it reads).
 * For callers that hold the queries of several layers at once; a decoder
 * that computes layer l+1's query from layer l's output calls
 * pkv_decode_attention per layer.
 *   descs[l]  HOST, L descriptors.  B, Hq, Hkv, d and page_size must be the
 *             same for all layers; k_cap, num_pages, max_pages and the c_*
 *             strides are per layer.
 *   q, K_cache, V_cache, block_tables, count, out, lse_out
 *             HOST arrays of L DEVICE pointers, each as in
 *             pkv_decode_attention.  block_tables may be NULL for compact
 *             caches; lse_out may be NULL (no log-sum-exp output), else all
 *             L entries are written through.
 *   workspace DEVICE, 256-byte aligned,
 *             >= pkv_decode_layers_workspace_bytes(L, descs) bytes (may be
 *             NULL when that is 0); contents irrelevant on entry, undefined
 *             on exit; concurrent calls need distinct ones.
 * Every layer's result is what pkv_decode_attention gives for it, up to the
 * order of the fp32 additions (the key ranges are cut differently).
 * Asynchronous on `stream`, never allocates.  Errors as for
 * pkv_decode_attention; layers that differ in B, Hq, Hkv, d or page_size ->
 * PKV_ERR_INVALID_ARG.
 */
size_t pkv_decode_layers_workspace_bytes(int32_t L,
                                         const pkv_decode_desc* descs);
int pkv_decode_attention_layers(int32_t L, const pkv_decode_desc* descs,
                                const void* const* q,
                                const void* const* K_cache,
                                const void* const* V_cache,
                                const int32_t* const* block_tables,
                                const int32_t* const* count,
                                float* const* out, float* const* lse_out,
                                void* workspace, size_t workspace_bytes,
                                void* stream);

/* Static, NUL-terminated description of a pkv_status value.  HOST only. */
const char* pkv_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* PKV_H_ */
