/*
 * kvm.h — C ABI of the per-decode-step KV-cache management pass.
 *
 * The pass manages a paged KV cache whose eviction granularity is one
 * (layer, KV-head, token-block) slice, called a *unit* here (head-granular
 * eviction, paper section 3.4).  Per decode step it
 *   1. folds observed reuse events into the 16 Beta posteriors  (section 3.3, Eq. 5)
 *   2. scores every resident unit by the softmax attention mass it receives
 *      from the step's queries                                   (Eq. 1, section 3.4)
 *   3. folds the masses into an exponential moving average and forms an
 *      eviction priority = head weight x EMA x posterior reuse probability
 *   4. selects the k lowest-priority units under a capacity budget
 *   5. moves victim / prefetch units between the HBM pool (tier 0) and
 *      pinned host memory (tier 1)                               (section 3.2)
 * kvm_size implements the architecture-aware sizing of section 3.1 (Eq. 3, 4).
 *
 * Conventions
 *   - Plain C, no exceptions, no allocations handed across the boundary.  The
 *     caller owns every buffer; the library keeps nothing between calls except
 *     an optional pair of internal HIP events used for kernel timing.
 *   - "dev" = pointer to device (HBM) memory, "host" = ordinary host memory,
 *     "pinned" = page-locked host memory that the GPU can reach.
 *   - Every function returns KVM_OK (0) or a negative KVM_E* code; a text for the
 *     last failure on the calling thread is returned by kvm_last_error().
 *     Arguments are validated on the host before anything is launched; a call
 *     that returns an error has launched nothing.
 *   - Device functions are asynchronous on the HIP stream passed as `stream`
 *     (a hipStream_t cast to void*; NULL = the default stream).
 *
 * Data model
 *   row   = (sequence, layer, KV head): one softmax domain of row_ntok tokens,
 *           ceil(row_ntok / 16) blocks.
 *   uid   = row_off[row] + block : index of a unit in all per-unit arrays
 *           (slot_tbl, mass, S, prio, state, pair).  Rows must not overlap in
 *           uid space; gaps are allowed (their state must be 0).
 *   slot  = index of a unit-sized frame in the HBM pool.
 *   slot_tbl[uid] >= 0 : the unit lives in pool frame slot_tbl[uid]
 *   slot_tbl[uid] <  0 : not in HBM; -1 - slot_tbl[uid] is the caller's label of
 *                        its place in the host tier.
 *
 * K unit layout (unit_k_bytes = 16 * dim * 2 bytes, 16-bit elements):
 *   element (token t, channel c) sits at element index (c / 8) * 128 + t * 8 + c % 8,
 *   i.e. [dim/8][16 tokens][8 channels]: the 16 tokens of one 8-channel group are
 *   contiguous 16-byte vectors.  This is the key-cache layout of the original
 *   PagedAttention kernel restricted to one head; a wavefront that reads 1 KiB
 *   of it gets 16 tokens x 4 channel groups with no shuffling.
 *   For MLA the unit holds the latent (d_latent + d_rope channels) in the same
 *   layout and there is no V.  V units are opaque bytes to this library.
 */
#ifndef KVM_H
#define KVM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- return codes ------------------------------------------------------ */
#define KVM_OK       0
#define KVM_EINVAL  (-1)   /* null pointer, negative count, value out of range   */
#define KVM_ESHAPE  (-2)   /* a shape the library has no kernel for            */
#define KVM_ENOSPC  (-3)   /* workspace / staging / output capacity too small    */
#define KVM_EHIP    (-4)   /* a HIP runtime call failed                          */

/* ---- element types of K and q ----------------------------------------- */
#define KVM_BF16 0
#define KVM_FP16 1

/* ---- attention architectures (section 3.1) ----------------------------- */
#define KVM_ARCH_MHA 0
#define KVM_ARCH_GQA 1
#define KVM_ARCH_MQA 2
#define KVM_ARCH_MLA 3

/* ---- per-unit state byte ------------------------------------------------ */
#define KVM_ST_RESIDENT  1u   /* unit is in an HBM pool frame                    */
#define KVM_ST_ON_HOST   2u   /* unit has been packed to the host tier           */
#define KVM_ST_PROTECTED 4u   /* never a victim (e.g. the block being written)   */
#define KVM_ST_SCORED    8u   /* S holds at least one observation                */
#define KVM_ST_SHARED   16u   /* reads a frame that other units read too (section 3.6): never a victim,
                                 refused by pack / swap / exchange until kvm_dedup_unshare           */

/* ---- group aggregation in kvm_score_step -------------------------------- */
#define KVM_AGG_MAX  0        /* max over the query heads sharing the KV head    */
#define KVM_AGG_MEAN 1        /* mean over them (per-head masses then sum to 1)  */

#define KVM_BLOCK_TOKENS 16
#define KVM_N_PAIRS      16   /* 4 block types x 4 transition types              */

/* ======================================================================== *
 * Sizing — section 3.1, Eq. 3 and Eq. 4.  Host only, no device work.
 * ======================================================================== */
typedef struct kvm_model {
    int32_t n_layers;       /* L                                                  */
    int32_t n_q_heads;      /* h_q                                                */
    int32_t n_kv_heads;     /* h_kv; must divide h_q                              */
    int32_t head_dim;       /* d                                                  */
    int32_t d_latent;       /* > 0 selects MLA                                    */
    int32_t d_rope;         /* MLA rope channels stored beside the latent         */
    int32_t bits_per_elem;  /* 16 (bf16/fp16), 8, 4 (p = 0.5 bytes)               */
    int32_t block_tokens;   /* tokens per block, > 0                              */
    int32_t head_divisor;   /* tensor-parallel divisor applied to KV heads, >= 1;
                               ignored for MLA (the latent is not split)          */
} kvm_model_t;

typedef struct kvm_sizing {
    int32_t  arch;                   /* KVM_ARCH_*                                */
    int32_t  group_size;             /* g = h_q / h_kv (MLA: h_q)                 */
    uint64_t bytes_per_token_layer;  /* B(1) of Eq. 3                             */
    uint64_t bytes_per_token;        /* L * B(1)                                  */
    uint64_t bytes_per_seq;          /* L * B(n_max)                              */
    uint64_t max_batch;              /* floor(M_target / (L * B(n_max))), Eq. 4   */
    uint32_t units_per_block;        /* units one token block spans: L * h_kv / head_divisor (MLA: L) */
    uint32_t unit_k_bytes;           /* block_tokens * d * p (MLA: latent + rope) */
    uint32_t unit_v_bytes;           /* same for V; 0 for MLA                     */
    uint32_t head_weight;            /* weight of one KV head's importance in the eviction
                                        priority (section 3.4): uniform (1) for MHA,
                                        the group size for GQA and MQA, 1 for the single
                                        latent head of MLA; the row_weight of kvm_ema_update */
    uint64_t pool_units;             /* floor(M_target / (unit_k + unit_v))       */
} kvm_sizing_t;

/* Architecture inference: d_latent > 0 -> MLA; else h_q == h_kv -> MHA;
 * else h_kv == 1 -> MQA; else GQA.  Byte counts with fractional p are exact
 * when the product is a whole number of bytes, else KVM_EINVAL.
 * n_max = 0 is allowed (bytes_per_seq = 0, max_batch = 0).
 * Errors: KVM_EINVAL for null pointers, non-positive dimensions,
 * h_q % h_kv != 0, h_kv % head_divisor != 0, bits not in {4, 8, 16, 32}.      */
int kvm_size(const kvm_model_t* model, uint64_t n_max, uint64_t mem_target_bytes,
             kvm_sizing_t* out /* host */);

/* ======================================================================== *
 * Pool and row descriptors shared by the device entry points
 * ======================================================================== */
typedef struct kvm_pool {
    void*    k_pool;        /* dev: n_slots frames of unit_k_bytes                */
    void*    v_pool;        /* dev: n_slots frames of unit_v_bytes; NULL iff unit_v_bytes == 0 */
    uint64_t n_slots;
    int32_t  dim;           /* channels per token in a K unit (head_dim, or 576 for MLA); multiple of 32 */
    int32_t  dtype;         /* KVM_BF16 / KVM_FP16                                */
    uint32_t unit_k_bytes;  /* must equal 16 * dim * 2                            */
    uint32_t unit_v_bytes;  /* multiple of 16                                     */
} kvm_pool_t;

typedef struct kvm_rows {
    int32_t        n_rows;
    int32_t        g;          /* queries per row (heads sharing the KV head), 1..128 */
    int64_t        n_uids;     /* length of every per-unit array                  */
    int64_t        q_elems;    /* length of q in elements (bounds check only)     */
    const int32_t* row_ntok;   /* dev [n_rows] valid tokens in the row, >= 0      */
    const int64_t* row_off;    /* dev [n_rows] uid of the row's block 0           */
    const int64_t* row_q_off;  /* dev [n_rows] element offset of the row's g x dim queries in q;
                                  multiple of 8; unused for inactive rows         */
    const uint8_t* row_active; /* dev [n_rows] or NULL (= all active). 0 marks a row that is not
                                  decoding this step: it is not scored and its S is left alone  */
    const int32_t* slot_tbl;   /* dev [n_uids]                                    */
} kvm_rows_t;
/* A fleet that mixes architectures passes one kvm_rows_t per architecture
 * (different g) over the same per-unit arrays. */

/* ======================================================================== *
 * 2. Scoring — Eq. 1 restricted to the HBM-resident tokens of each row.
 *
 * For an active row with n = row_ntok tokens and resident blocks R, for each
 * query j < g:   z_t = softmax_scale * <q_j, k_t>  for tokens t < n in blocks of R,
 * p = softmax(z) over those tokens, m_j[b] = sum of p over block b.
 * mass[uid(b)] = max_j m_j[b] (KVM_AGG_MAX; the GQA grouping rule of section 3.4)
 * or mean_j.  Entries of non-resident blocks, of blocks beyond the row's
 * length and of inactive rows are not written.  Tokens at or beyond n in the
 * last block are ignored whatever bytes the pool holds there.  A row whose
 * blocks would leave [0, n_uids) or whose queries would leave [0, q_elems) is
 * treated as inactive; table entries >= n_slots are treated as not resident.
 * Rows that overlap in uid space (against the data model) get undefined masses
 * but cause no access outside the arrays; if they overlap so much that their
 * tiles exceed what the workspace was sized for, the call scores nothing.
 * fp32 accumulation; masses agree with an exact evaluation to ~1e-5 relative.
 *
 * q: dev, dtype of the pool, g x dim contiguous per row at row_q_off.
 * ws: dev scratch of at least kvm_workspace_bytes(KVM_OP_SCORE, ...) bytes,
 *     256-byte aligned; contents are garbage afterwards.
 * Errors: KVM_EINVAL (null pointers, agg), KVM_ESHAPE (dim % 32, g out of
 * range, dtype, unit_k_bytes mismatch), KVM_ENOSPC (ws_bytes too small),
 * KVM_EHIP.  n_rows == 0 or n_uids == 0 is a successful no-op.              */
int kvm_score_step(const kvm_pool_t* pool, const kvm_rows_t* rows, const void* q,
                   float softmax_scale, int agg, float* mass /* dev [n_uids] */,
                   void* ws, size_t ws_bytes, void* stream);

/* The same launch can carry the bytes of a deferred exchange (kvm_exchange_begin
 * below): n_pairs extra workgroups at the front of the scorer's grid each swap
 * one (pool frame, host tier record) pair in place while the rest of the grid
 * scores, so the host link works during the scoring and not after it.
 * xfer_frame[i] outside [0, n_slots) or xfer_host[i] outside [0, tier_slots)
 * skips pair i (kvm_exchange_begin writes -1 to both for a pair it refused).  The frames named belong to units the scorer
 * cannot see (kvm_exchange_begin took them out of the table), so scoring and
 * transfer never touch the same memory; results equal kvm_score_step followed
 * by the same transfer.  n_pairs == 0 is kvm_score_step.
 * A pair whose xfer_host[i] carries KVM_XFER_OUT_ONLY (what kvm_pack_begin
 * writes) is one-way: the frame's bytes are copied to host slot
 * xfer_host[i] & ~KVM_XFER_OUT_ONLY, nothing is read from the host and the
 * frame keeps its bytes.  Pairs of both kinds may share one list.
 * Errors: as kvm_score_step; KVM_EINVAL for null transfer buffers.           */
#define KVM_XFER_OUT_ONLY (1ll << 62)
int kvm_score_step_xfer(const kvm_pool_t* pool, const kvm_rows_t* rows, const void* q,
                        float softmax_scale, int agg, float* mass /* dev [n_uids] */,
                        void* ws, size_t ws_bytes,
                        const int32_t* xfer_frame /* dev [n_pairs] */, const int64_t* xfer_host /* dev [n_pairs] */,
                        int64_t n_pairs, void* host_tier /* pinned, tier_slots records */, uint64_t tier_slots,
                        void* stream);

/* ======================================================================== *
 * 1. Beta posteriors — section 3.3, Eq. 5.
 *
 * pair = 4 * block_type + transition_type, types numbered in the order the
 * paper lists them (system_prompt, tool_context, user_context,
 * intermediate_reasoning; same_tool_repeat, tool_switch, reasoning_step,
 * agent_handoff).  For each event: outcome 1 (reuse) -> hits[pair] += 1,
 * outcome 0 (miss) -> misses[pair] += 1.  Events with pair >= 16 or
 * outcome > 1 change no counter and are counted in *n_bad (if not NULL).
 * Then p_hat[i] = (alpha0 + hits[i]) / (alpha0 + beta0 + hits[i] + misses[i]).
 * Counters are exact integers (order-independent); p_hat is fp32.
 * n_events == 0 just refreshes p_hat.
 * Errors: KVM_EINVAL (null pointers, n_events < 0, alpha0/beta0 not > 0).   */
int kvm_beta_update(const uint8_t* ev_pair /* dev [n_events] */,
                    const uint8_t* ev_outcome /* dev [n_events] */, int64_t n_events,
                    uint32_t* hits /* dev [16] in/out */, uint32_t* misses /* dev [16] in/out */,
                    float alpha0, float beta0, float* p_hat /* dev [16] out */,
                    uint32_t* n_bad /* dev [1] in/out, or NULL */, void* stream);

/* Blended reuse estimate — section 3.3, the two paragraphs after Eq. 5.
 *
 * Does everything kvm_beta_update does and, with the same events taken in
 * array order, keeps per pair a ring of its last `window` outcomes:
 *   win[pair * window + i] is 0 or 1; any other value marks a place never
 *   written (the caller fills the array with 0xFF before first use);
 *   win_head[pair] < window is the next place to write.
 * Then, per pair, with n = hits + misses:
 *   conf    = n / (n + kappa)                       (0 when n + kappa == 0)
 *   f       = share of 1s among the written places of the ring, or p_hat when none
 *   p_blend = conf * p_hat + (1 - conf) * f
 * so a pair with few observations follows its recent frequency and a well
 * observed pair its posterior mean.  The paper gives neither the saturation
 * function nor the window; kappa and window are the caller's.
 * The ring update runs in one workgroup (the order of events matters):
 * meant for the thousands of lookups of a decode step, ~1 us per 1024 events.
 * Malformed events touch neither counters nor ring.  A win_head entry >=
 * window is taken modulo window.
 * Errors: KVM_EINVAL (as kvm_beta_update; window outside [1, KVM_MAX_WINDOW];
 * kappa < 0; null win / win_head / conf / p_blend).                         */
#define KVM_MAX_WINDOW 65536
int kvm_beta_blend_update(const uint8_t* ev_pair /* dev [n_events] */,
                          const uint8_t* ev_outcome /* dev [n_events] */, int64_t n_events,
                          uint32_t* hits /* dev [16] in/out */, uint32_t* misses /* dev [16] in/out */,
                          float alpha0, float beta0,
                          uint8_t* win /* dev [16 * window] in/out */, uint32_t* win_head /* dev [16] in/out */,
                          int32_t window, float kappa,
                          float* p_hat /* dev [16] out */, float* conf /* dev [16] out */,
                          float* p_blend /* dev [16] out */,
                          uint32_t* n_bad /* dev [1] in/out, or NULL */, void* stream);

/* ======================================================================== *
 * 3. EMA of the masses and eviction priority — section 3.4.
 *
 * For every block b < ceil(row_ntok/16) of every row r, uid = row_off[r] + b:
 *   if the row is active and state[uid] has RESIDENT (the unit was scored this step):
 *       first observation (SCORED clear):  S[uid] = mass[uid], set SCORED
 *       otherwise:                         S[uid] = decay * S[uid] + (1 - decay) * mass[uid]
 *   prio[uid] = row_weight[r] * S[uid] * p_hat[pair[uid]]  if SCORED, else +inf.
 * row_weight carries the architecture-dependent head weight (1 for MHA and MLA,
 * the group size for GQA/MQA) times any per-head multiplier.
 * Errors: KVM_EINVAL (null pointers, decay outside [0, 1]).                 */
int kvm_ema_update(const kvm_rows_t* rows, const float* mass /* dev [n_uids] */, float ema_decay,
                   const float* row_weight /* dev [n_rows] */, const uint8_t* pair /* dev [n_uids], < 16 */,
                   const float* p_hat /* dev [16] */, uint8_t* state /* dev [n_uids] in/out */,
                   float* S /* dev [n_uids] in/out */, float* prio /* dev [n_uids] out */, void* stream);

/* The same with the two refinements section 3.4 names without formulas (the
 * importance also falls off with positional distance; per-head multipliers
 * are applied during a task transition, section 3.7 item 2):
 *   the observation fed to the EMA is pos_decay^d * mass[uid], d = nb - 1 - b
 *   blocks behind the row's last block (where the decode position lies);
 *   prio = row_weight[r] * mult_r * S * p_hat[pair], mult_r =
 *   head_mult[t * n_heads + row_head[r]] with t = seq_transition[row_seq[r]]
 *   when t <= 3 (a transition of type t is in progress), else 1.
 * head_mult NULL = no multipliers (row_seq, row_head, seq_transition unused).
 * A row whose row_seq / row_head lies outside [0, n_seq) / [0, n_heads) keeps
 * multiplier 1.  pos_decay = 1 and head_mult NULL give kvm_ema_update bit for bit.
 * Errors: as kvm_ema_update; KVM_EINVAL for pos_decay outside (0, 1] or
 * head_mult without the three index arrays.                                 */
typedef struct {
    float          pos_decay;       /* (0, 1]; 1 = no positional decay                   */
    int32_t        n_seq;           /* entries of seq_transition                         */
    int32_t        n_heads;         /* entries of one row of head_mult                   */
    const int32_t* row_seq;         /* dev [n_rows] sequence of each row                 */
    const int32_t* row_head;        /* dev [n_rows] head index, e.g. layer * H + head    */
    const uint8_t* seq_transition;  /* dev [n_seq] 0..3 = transition type, > 3 = none    */
    const float*   head_mult;       /* dev [4][n_heads], or NULL                         */
} kvm_ema_ex_t;
int kvm_ema_update_ex(const kvm_rows_t* rows, const float* mass /* dev [n_uids] */, float ema_decay,
                      const kvm_ema_ex_t* ex /* host */,
                      const float* row_weight /* dev [n_rows] */, const uint8_t* pair /* dev [n_uids], < 16 */,
                      const float* p_hat /* dev [16] */, uint8_t* state /* dev [n_uids] in/out */,
                      float* S /* dev [n_uids] in/out */, float* prio /* dev [n_uids] out */, void* stream);

/* ======================================================================== *
 * 4. Victim selection — the unit whose head-weighted importance is smallest goes
 *    first (section 3.4), generalised to the k smallest under a capacity budget.
 *
 * eligible = RESIDENT and SCORED and neither PROTECTED nor SHARED.
 * k = k_or_neg1 if >= 0, else max(0, #RESIDENT - budget_units);
 * k is then clipped to #eligible and to victims_cap.
 * Output: the k eligible uids smallest under the total order (prio, uid)
 * (NaN priorities rank as +inf, -0 as +0), written in ascending uid order to
 * victims[0..k), and k to *n_victims.  Both on the device; nothing is copied
 * to the host.  ws as for kvm_score_step with KVM_OP_SELECT.
 * Errors: KVM_EINVAL (null pointers, negative sizes, k < -1), KVM_ENOSPC.   */
int kvm_select_victims(const float* prio /* dev [n_uids] */, const uint8_t* state /* dev [n_uids] */,
                       int64_t n_uids, int64_t k_or_neg1, int64_t budget_units,
                       int64_t* victims /* dev [victims_cap] */, int64_t victims_cap,
                       int64_t* n_victims /* dev [1] */, void* ws, size_t ws_bytes, void* stream);

/* For callers that cannot allocate or hand over device memory at the time of the
 * call (code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc): kvm_select_victims with the workspace replaced by a scratch array
 * built into the library's device code, KVM_SELECT_STATIC_SCRATCH_BYTES per GPU,
 * held from the time the library is loaded on a GPU until the process ends.
 * Same arguments otherwise, same result bit for bit.  The call allocates nothing
 * (no hipMalloc / hipFree, no event creation: it is never timed by kvm_timing_*)
 * and records only kernel launches on `stream`, no memset.  The device of
 * `stream` and of the buffers must be the current device; the scratch address is
 * looked up once per device, on the first call made with that device current.
 * Every call on a GPU uses that GPU's one array: calls that overlap on one GPU
 * (two streams, two threads) race and give undefined victims; calls in sequence
 * on one stream, or ordered by events, are fine, and nothing has to be cleared
 * in between (the kernels initialise what they read).
 * Errors: as kvm_select_victims; KVM_ENOSPC when n_uids exceeds
 * KVM_SELECT_STATIC_MAX_UIDS (nothing is launched).                          */
#define KVM_SELECT_STATIC_MAX_UIDS      (1 << 26)
#define KVM_SELECT_STATIC_SCRATCH_BYTES (145408 + 256 + 2 * ((KVM_SELECT_STATIC_MAX_UIDS / 4096) * 4 + 256))
int kvm_select_victims_static(const float* prio /* dev [n_uids] */, const uint8_t* state /* dev [n_uids] */,
                              int64_t n_uids, int64_t k_or_neg1, int64_t budget_units,
                              int64_t* victims /* dev [victims_cap] */, int64_t victims_cap,
                              int64_t* n_victims /* dev [1] */, void* stream);

/* ======================================================================== *
 * 5. Pack / unpack — tier 0 (HBM pool) <-> tier 1 (pinned host), section 3.2.
 *
 * kvm_pack, for i < n in list order, uid = uids[i], slot = slot_tbl[uid]:
 *   staging[i] = K frame `slot` (unit_k_bytes) followed by V frame `slot`
 *   (unit_v_bytes); freed_slots[i] = slot; slot_tbl[uid] = -1 - host_slots[i];
 *   state[uid]: clear RESIDENT, set ON_HOST.
 * Entries whose uid is outside [0, n_uids), not resident or SHARED (a frame that
 * other units read is never handed out; kvm_dedup_unshare first), or whose slot is
 * outside the pool, move nothing, get freed_slots[i] = -1, leave their staging
 * record untouched and are counted in *n_bad.  uids must be distinct.
 * n_dev, if not NULL, is a device-side list length (e.g. kvm_select_victims'
 * n_victims): entries i >= *n_dev are ignored entirely (their freed_slots and
 * staging records are not written), so a victim list can be packed without a
 * host round trip to learn its length; n is then the upper bound the host knows.
 * The records are gathered into staging_dev in chunks and copied to
 * staging_host with hipMemcpyAsync on `stream`; when staging_dev is NULL the
 * gather kernel writes the pinned host buffer directly.
 * staging_host must hold n * (unit_k_bytes + unit_v_bytes) bytes;
 * staging_dev_bytes must hold at least one record.
 * When staging_host is NULL the call only gathers: the n records stay in
 * staging_dev (which must hold them all) and the caller moves them, e.g. with
 * hipMemcpyAsync on a side stream so that the copy overlaps the next step's
 * scoring.  kvm_unpack with staging_host NULL likewise only scatters records
 * that the caller has already brought into staging_dev.
 *
 * kvm_unpack is the inverse: record i of staging_host goes to pool frame
 * dst_slots[i]; slot_tbl[uid] = dst_slots[i]; state: set RESIDENT, clear
 * ON_HOST.  Entries with a bad uid, an already-resident uid or a dst slot
 * outside the pool are skipped and counted; n_dev as for kvm_pack.
 * Both are asynchronous: staging_host may be read (pack) or reused (unpack)
 * once `stream` has drained.
 * Errors: KVM_EINVAL (null pointers, n < 0), KVM_ENOSPC (staging too small). */
int kvm_pack(const kvm_pool_t* pool, int32_t* slot_tbl /* dev in/out */, uint8_t* state /* dev in/out */,
             int64_t n_uids, const int64_t* uids /* dev [n] */, int64_t n, const int64_t* n_dev /* dev [1] or NULL */,
             const int32_t* host_slots /* dev [n] */, int32_t* freed_slots /* dev [n] out */,
             void* staging_dev /* dev or NULL */, size_t staging_dev_bytes,
             void* staging_host /* pinned */, size_t staging_host_bytes,
             uint32_t* n_bad /* dev [1] in/out, or NULL */, void* stream);

int kvm_unpack(const kvm_pool_t* pool, int32_t* slot_tbl /* dev in/out */, uint8_t* state /* dev in/out */,
               int64_t n_uids, const int64_t* uids /* dev [n] */, int64_t n, const int64_t* n_dev /* dev [1] or NULL */,
               const int32_t* dst_slots /* dev [n] */,
               void* staging_dev /* dev or NULL */, size_t staging_dev_bytes,
               const void* staging_host /* pinned */, size_t staging_host_bytes,
               uint32_t* n_bad /* dev [1] in/out, or NULL */, void* stream);

/* kvm_swap = kvm_pack(out_uids) followed by kvm_unpack(in_uids) into the frames just
 * freed (entry i of in_uids takes the frame of entry i of out_uids), in one pass
 * with no device staging: the kernel writes record i to host_out and reads record
 * i from host_in directly, so both directions of the host link work at once
 * (sections 3.2: demotion and promotion are asynchronous and independent).
 * freed_slots[i] is the frame entry i of out_uids left (as kvm_pack, -1 if that
 * entry was skipped); an in entry whose out entry was skipped, whose uid is out
 * of range or which is already resident is skipped too, and its frame stays free.
 * Every skipped half-entry counts once in *n_bad.  n_dev as for kvm_pack.
 * Errors: as kvm_pack.                                                         */
int kvm_swap(const kvm_pool_t* pool, int32_t* slot_tbl /* dev in/out */, uint8_t* state /* dev in/out */,
             int64_t n_uids, const int64_t* out_uids /* dev [n] */, const int64_t* in_uids /* dev [n] */, int64_t n,
             const int64_t* n_dev /* dev [1] or NULL */, const int32_t* host_slots /* dev [n] */,
             int32_t* freed_slots /* dev [n] out */, void* host_out /* pinned */, size_t host_out_bytes,
             const void* host_in /* pinned */, size_t host_in_bytes, uint32_t* n_bad /* dev [1] in/out, or NULL */,
             void* stream);

/* kvm_exchange: the same trade against a host tier that is addressed by slot
 * (record of host slot h at host_tier + h * (unit_k_bytes + unit_v_bytes)), as
 * the table describes it: for i < n (and < *n_out_dev, < *n_in_dev when given)
 * the unit out_uids[i], resident in frame f, and the unit in_uids[i], on the
 * host in slot h = -1 - slot_tbl[in_uids[i]], change places in place: frame f
 * receives the record of slot h, slot h the old contents of frame f;
 * slot_tbl[out] = -1 - h, slot_tbl[in] = f, RESIDENT / ON_HOST flip on both.
 * No spare frame or host slot is used, so a prefetch list produced on the
 * device (kvm_prefetch_keys + kvm_select_victims) can be served without the
 * host gathering records first.  A pair is skipped and counted in *n_bad when
 * out is not resident or is SHARED, in is not on the host (or equals out), or a
 * frame / slot id is out of range.  Units must not repeat within or across the lists.
 * Errors: KVM_EINVAL, KVM_ESHAPE as kvm_pack.                               */
int kvm_exchange(const kvm_pool_t* pool, int32_t* slot_tbl /* dev in/out */, uint8_t* state /* dev in/out */,
                 int64_t n_uids, const int64_t* out_uids /* dev [n] */, const int64_t* in_uids /* dev [n] */, int64_t n,
                 const int64_t* n_out_dev /* dev [1] or NULL */, const int64_t* n_in_dev /* dev [1] or NULL */,
                 void* host_tier /* pinned, tier_slots records */, uint64_t tier_slots,
                 uint32_t* n_bad /* dev [1] in/out, or NULL */, void* stream);

/* kvm_exchange in three parts, so that the bytes can move while the next step
 * is being scored (promotion and demotion off the decode path, section 3.2):
 *   kvm_exchange_begin  validates the pairs exactly as kvm_exchange does and, for
 *       each valid pair, takes the out-unit out of HBM in the table (RESIDENT
 *       off, ON_HOST on, slot_tbl = -1 - host slot of its partner) and notes
 *       frame[i] = the frame it held, host[i] = that host slot; frame[i] = -1 for
 *       a skipped pair (counted in *n_bad) and for i beyond the device-side
 *       counts.  The in-unit's entries are left alone: it is still on the host.
 *   kvm_score_step_xfer(frame, host, n)  moves the bytes during the next scoring.
 *   kvm_exchange_end    gives each valid pair's in-unit the frame
 *       (slot_tbl = frame[i], ON_HOST off, RESIDENT on).
 * After the three calls tables, pools and tier equal what kvm_exchange leaves.
 * Between begin and end neither unit of a pair is in HBM for the scorer, the
 * EMA or the selector (a victim list built in between cannot contain them),
 * and both table entries name the same host slot with ON_HOST set: the caller
 * must not build a prefetch list in between, it could name either of them.
 * Errors: as kvm_exchange; null frame / host.                                */
int kvm_exchange_begin(const kvm_pool_t* pool, int32_t* slot_tbl /* dev in/out */, uint8_t* state /* dev in/out */,
                       int64_t n_uids, const int64_t* out_uids /* dev [n] */, const int64_t* in_uids /* dev [n] */,
                       int64_t n, const int64_t* n_out_dev /* dev [1] or NULL */,
                       const int64_t* n_in_dev /* dev [1] or NULL */, uint64_t tier_slots,
                       int32_t* frame /* dev [n] out */, int64_t* host /* dev [n] out */,
                       uint32_t* n_bad /* dev [1] in/out, or NULL */, void* stream);
int kvm_exchange_end(int32_t* slot_tbl /* dev in/out */, uint8_t* state /* dev in/out */, int64_t n_uids,
                     const int64_t* in_uids /* dev [n] */, const int32_t* frame /* dev [n] */, int64_t n,
                     void* stream);

/* kvm_pack in two parts against a slot-addressed tier, for evictions whose bytes
 * may leave while the next step is being scored (demotion off the decode path,
 * section 3.2):
 *   kvm_pack_begin  validates entry i as kvm_pack does (uid in range and resident,
 *       frame inside the pool; here also host_slots[i] in [0, tier_slots)) and
 *       takes the unit out of HBM in the table (RESIDENT off, ON_HOST on,
 *       slot_tbl = -1 - host_slots[i]); frame[i] = the frame it held, host[i] =
 *       host_slots[i] | KVM_XFER_OUT_ONLY; both -1 for a skipped entry (counted in
 *       *n_bad) and for i at or beyond *n_dev.
 *   kvm_score_step_xfer(frame, host, n)  copies the frames to their records
 *       during the next scoring launch.
 * After that launch tables, state and tier equal what kvm_pack leaves with
 * staging_host = the tier and record i at slot host_slots[i], and frame[] is
 * kvm_pack's freed_slots.  Until then the frames still hold the units' bytes and
 * must not be given to other units; the records are not valid yet, so the units
 * must not be prefetched in between (a prefetch list built in between could
 * name them: build it after the launch).
 * Errors: KVM_EINVAL (null buffers, negative counts, slot ids beyond int32).  */
int kvm_pack_begin(const kvm_pool_t* pool, int32_t* slot_tbl /* dev in/out */, uint8_t* state /* dev in/out */,
                   int64_t n_uids, const int64_t* uids /* dev [n] */, int64_t n,
                   const int64_t* n_dev /* dev [1] or NULL */, const int32_t* host_slots /* dev [n] */,
                   uint64_t tier_slots, int32_t* frame /* dev [n] out */, int64_t* host /* dev [n] out */,
                   uint32_t* n_bad /* dev [1] in/out, or NULL */, void* stream);

/* ======================================================================== *
 * 6. Position-aware prefetching — section 3.5.
 *
 * kvm_span_update: the prefetch window follows the attention pattern each
 * layer shows, narrow for layers that attend locally, wide for layers that
 * attend globally (section 3.5, no formula given).  Reading: the span of an active row is
 * the smallest s >= 1 such that its last s blocks hold at least theta_num /
 * theta_den of the row's total mass this step (blocks not in HBM count as
 * distance and contribute nothing; rows with no mass are skipped);
 * span_sum[layer] += s, span_cnt[layer] += 1 (both accumulate over calls; the
 * caller resets or ages them); then for every layer with span_cnt > 0
 *   layer_window[l] = clamp(16 * ceil(span_sum[l] / span_cnt[l]), w_min, w_max)
 * in tokens; other layers keep their window.  Masses enter as fixed point,
 * floor(min(m, 1) * 2^32) (0 for m <= 0 or NaN), sums and comparisons are exact
 * integers: the result does not depend on summation order.
 * ws: dev scratch of at least kvm_workspace_bytes(KVM_OP_SPAN, ...) bytes
 * (one 32-bit span per row, folded per layer by a second kernel), 4-byte
 * aligned, contents irrelevant before and undefined after; not needed when
 * n_rows or n_uids is 0.
 * Errors: KVM_EINVAL (null pointers, n_layers <= 0, theta outside [0, 1] or
 * theta_den > 65536, w_min < 0, w_max < w_min), KVM_ENOSPC (ws_bytes too
 * small).  Rows with row_layer outside [0, n_layers) are skipped.           */
int kvm_span_update(const kvm_rows_t* rows, const int32_t* row_layer /* dev [n_rows] */, int32_t n_layers,
                    const float* mass /* dev [n_uids] */, const uint8_t* state /* dev [n_uids] */,
                    uint32_t theta_num, uint32_t theta_den,
                    uint64_t* span_sum /* dev [n_layers] in/out */, uint32_t* span_cnt /* dev [n_layers] in/out */,
                    int32_t w_min, int32_t w_max, int32_t* layer_window /* dev [n_layers] in/out */,
                    void* ws, size_t ws_bytes, void* stream);

/* kvm_prefetch_keys: which host-resident units to promote ahead of use.  While
 * a request decodes at position n the blocks within a window w of n are the
 * likeliest to be needed next; the text gives the window once as [n - w, n] and
 * once as [n, n + w]; positions after n hold no keys yet, so [n - w, n] is used.
 * For row r, n = row_pos[r] (tokens; negative = the row asks for nothing),
 * w = layer_window[row_layer[r]]: block b is a candidate iff state has ON_HOST
 * and not RESIDENT and its tokens [16 b, 16 b + 15] meet [n - w, n].  Then
 *   key[uid]  = 1 - p_est[pair[uid]] * pos_decay^(floor(n / 16) - b)   (lower = sooner)
 *   cand[uid] = KVM_ST_RESIDENT | KVM_ST_SCORED
 * and key = +inf, cand = 0 for every other block of the row.  cand has the
 * form kvm_select_victims admits, so the prefetch list (uid ascending) is
 *   kvm_select_victims(key, cand, n_uids, k, 0, list, ...)
 * with k = the number of free frames, and kvm_unpack / kvm_swap move it.
 * p_est: posterior means or the blended estimates of kvm_beta_blend_update.
 * Errors: KVM_EINVAL (null pointers, n_layers <= 0, pos_decay outside (0, 1]). */
int kvm_prefetch_keys(const kvm_rows_t* rows, const int32_t* row_layer /* dev [n_rows] */,
                      const int32_t* row_pos /* dev [n_rows] */, const int32_t* layer_window /* dev [n_layers] */,
                      int32_t n_layers, const uint8_t* state /* dev [n_uids] */, const uint8_t* pair /* dev [n_uids] */,
                      const float* p_est /* dev [16] */, float pos_decay,
                      float* key /* dev [n_uids] out */, uint8_t* cand /* dev [n_uids] out */, void* stream);

/* ======================================================================== *
 * 7. Content addressing — section 3.6.
 *
 * kvm_hash_units: digests[i] = SHA-256 (FIPS 180-4) of the record of uids[i],
 * i.e. of its K frame followed by its V frame, 32 bytes in the standard's byte
 * order.  A uid that is out of range or not RESIDENT gets an all-zero digest
 * and is counted in *n_bad.  One lane hashes one unit (the hash is a serial
 * chain over the record), so the call wants thousands of units to fill the
 * chip; it is bound by integer ALU work (about 30 operations per byte).
 * Errors: KVM_EINVAL, KVM_ESHAPE (unit sizes not multiples of 64).           */
int kvm_hash_units(const kvm_pool_t* pool, const int32_t* slot_tbl /* dev */, const uint8_t* state /* dev */,
                   int64_t n_uids, const int64_t* uids /* dev [n] */, int64_t n,
                   uint8_t* digests /* dev [n][32] out, 4-byte aligned */,
                   uint32_t* n_bad /* dev [1] in/out, or NULL */, void* stream);

/* The store: content store with reference counts (section 3.6): a digest already
 * present gains a reference, the block is not stored twice.  An open-addressing
 * table in device memory, all arrays caller-allocated with `cap` entries (cap a
 * power of two, kept at most half full by the caller) and initialised once to
 * tag = 0, canon = -1, refs = 0, pending = 0xFFFFFFFF.  It is keyed by the first
 * 64 bits of the digest; every match is confirmed on all 256 bits.
 *
 * kvm_dedup_insert, items taken as if one after the other in list order:
 *   digest not in the store (or its count is 0): the item becomes the canonical
 *   copy, count = 1;  otherwise count += 1.
 *   canon_out[i] = uid of the canonical copy (== uids[i]: item i is not a duplicate).
 * So within one call the first occurrence of a new digest is the canonical one.
 * All-zero digests are skipped (canon_out = own uid).  *n_full counts items
 * that found no place (table too full: they stay unique and uncounted),
 * *n_collide items whose 64-bit key met a different digest (they stay unique);
 * with either non-zero the outcome depends on arrival order, otherwise it is
 * the sequential definition exactly.  Entries are never removed; a count that
 * kvm_dedup_release brought to 0 is revived by the next insert of its digest.
 * ws: dev scratch, 8 * n bytes, 8-byte aligned.
 * kvm_dedup_release: count -= 1 for each digest; unknown digests and counts
 * already at 0 are counted in *n_bad.
 * Errors: KVM_EINVAL (null pointers, cap not a power of two, n out of range),
 * KVM_ENOSPC (ws).                                                          */
typedef struct {
    uint64_t* tag;       /* dev [cap]      first 8 digest bytes, 0 = empty              */
    uint8_t*  digest;    /* dev [cap][32]  digest of the canonical copy                 */
    int64_t*  canon;     /* dev [cap]      uid of the canonical copy, -1 = none yet     */
    uint32_t* refs;      /* dev [cap]      reference count                              */
    uint32_t* pending;   /* dev [cap]      scratch between the passes of one insert     */
    uint64_t  cap;
} kvm_store_t;
int kvm_dedup_insert(const kvm_store_t* store /* host struct of dev pointers */,
                     const uint8_t* digests /* dev [n][32] */, const int64_t* uids /* dev [n] */, int64_t n,
                     int64_t* canon_out /* dev [n] out */, uint32_t* n_full /* dev [1] in/out, or NULL */,
                     uint32_t* n_collide /* dev [1] in/out, or NULL */, void* ws, size_t ws_bytes, void* stream);
int kvm_dedup_release(const kvm_store_t* store, const uint8_t* digests /* dev [n][32] */, int64_t n,
                      uint32_t* n_bad /* dev [1] in/out, or NULL */, void* stream);

/* Frames shared by units of equal content (section 3.6: a block whose content the
 * pool already holds is referenced instead of being stored again).
 * kvm_dedup_share: canon[i] is what kvm_dedup_insert reported for uids[i].  Item i
 * with canon[i] != uids[i] whose two units are in range, RESIDENT and not
 * PROTECTED (content still being written), whose duplicate is not SHARED already
 * (others may read its frame) and whose frames are inside the pool and differ: the
 * duplicate gives up its frame (freed[i]) and reads the canonical unit's from now
 * on (slot_tbl[uid] = slot_tbl[canon]); both units get KVM_ST_SHARED;
 * frame_refs[frame] = number of units that read it (2 after the first sharing, one
 * more per further duplicate; 0 for frames that are not shared; the caller zeroes
 * the array once).  Every other item: freed[i] = -1; a uid or canonical uid
 * outside [0, n_uids) is counted in *n_bad.  Within one call no uid may repeat in
 * uids and no unit may be both a duplicate and somebody's canonical copy (what
 * kvm_dedup_insert reports never is).  Scoring, EMA and hashing read shared frames
 * like any other; selection, pack, swap and exchange leave SHARED units alone.
 * kvm_dedup_unshare: a unit gets a frame of its own again (before it may be
 * evicted or written to).  Item i with uids[i] in range, RESIDENT and SHARED and
 * new_frames[i] inside the pool: the bytes it reads are copied to frame
 * new_frames[i], slot_tbl[uid] = new_frames[i], SHARED is cleared,
 * frame_refs[old frame] -= 1; a unit left as the only reader of a frame keeps
 * SHARED until it is unshared itself.  freed[i] = the old frame if nobody reads it
 * any more, else -1 (when the last readers of a frame are unshared in one call,
 * which of their items reports the frame is not defined; exactly one does).
 * Every other item: freed[i] = new_frames[i] (the frame comes back unused);
 * out-of-range uids and frames are counted in *n_bad.  No uid may repeat.
 * Errors: KVM_EINVAL (null buffers, negative counts), KVM_ESHAPE (unit sizes).  */
int kvm_dedup_share(int32_t* slot_tbl /* dev in/out */, uint8_t* state /* dev in/out */, int64_t n_uids,
                    uint64_t n_slots, const int64_t* uids /* dev [n] */, const int64_t* canon /* dev [n] */,
                    int64_t n, uint32_t* frame_refs /* dev [n_slots] in/out */, int32_t* freed /* dev [n] out */,
                    uint32_t* n_bad /* dev [1] in/out, or NULL */, void* stream);
int kvm_dedup_unshare(const kvm_pool_t* pool, int32_t* slot_tbl /* dev in/out */, uint8_t* state /* dev in/out */,
                      int64_t n_uids, const int64_t* uids /* dev [n] */, const int32_t* new_frames /* dev [n] */,
                      int64_t n, uint32_t* frame_refs /* dev [n_slots] in/out */, int32_t* freed /* dev [n] out */,
                      uint32_t* n_bad /* dev [1] in/out, or NULL */, void* stream);

/* ======================================================================== *
 * Helpers
 * ======================================================================== */
#define KVM_OP_SCORE  0
#define KVM_OP_SELECT 1
#define KVM_OP_SPAN   2
/* Bytes of device scratch the op needs for these sizes (SELECT looks at n_uids only, SPAN at
 * n_rows only); 0 for an unknown op or a negative size. */
size_t kvm_workspace_bytes(int op, int64_t n_uids, int32_t n_rows, int32_t g, int32_t dim);

/* Text describing the last error returned on this thread ("" if none). */
const char* kvm_last_error(void);

/* Library version, "major.minor". */
const char* kvm_version(void);

/* Measurement aid: reads every byte of a device buffer once (16-byte non-temporal
 * loads, nothing else).  Its rate is the ceiling for any kernel that has to read
 * the same bytes; time it with kvm_timing_* ("probe_read") or with events.
 * *sink is a device word the kernel may increment.  Errors: KVM_EINVAL.         */
int kvm_probe_read(const void* buf /* dev, 16-byte aligned */, size_t bytes /* multiple of 16 */,
                   uint32_t* sink /* dev [1] */, void* stream);

/* Kernel timing.  While enabled, the device entry points bracket each kernel
 * they launch with HIP events on the caller's stream.  kvm_timing_read
 * synchronises on the recorded events, adds up the elapsed time of every
 * launch of the kernel called `name` since the last kvm_timing_reset, and
 * returns the launch count (0 if the name is unknown); *total_ms gets the sum.
 * Names: "score_partial", "score_finalize", "score_plan", "ema_prio",
 * "beta", "select_hist", "select_emit", "pack", "unpack", "swap", "span",
 * "prefetch_keys", "hash", "dedup", "exchange_flip", "probe_read".          */
int  kvm_timing_enable(int on);
/* Restricts timing to the kernels called `name` (NULL: all of them again).  An event pair
 * costs a few microseconds on the stream, which shows in a pass of twenty small launches;
 * a caller that wants the duration of one kernel and an undisturbed total asks for that one. */
int  kvm_timing_only(const char* name);
void kvm_timing_reset(void);
int  kvm_timing_read(const char* name, double* total_ms);

#ifdef __cplusplus
}
#endif
#endif /* KVM_H */
