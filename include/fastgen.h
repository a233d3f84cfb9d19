/*
 * fastgen.h -- C ABI of the FastGen hot path for AMD MI355X (gfx950).
 *
 * FastGen ("Model Tells You What to Discard", arXiv 2310.01801) compresses the KV cache of
 * every attention head with a policy chosen per head from the prompt's attention map.
 * This library is the data-parallel part of it:
 *
 *   stage 1 (Alg. 1 "Prompt Encoding"):  A = softmax(Q K^T) per head, recovery of every
 *       policy of the family of Eq. 2, choice of the cheapest policy reaching the recovery
 *       threshold T (Eq. 1), compaction of K,V to the kept tokens  f(K, V, C);
 *   stage 2 (Alg. 2 "Token Generation"): per generated token, attention of the new query
 *       over the head's compressed cache plus the new token, then f again with the head's
 *       fixed policy (append / evict in place).
 *
 * A "unit" is one (sequence b, layer l, head h); units are flattened as
 * u = (b * layers + l) * heads + h and are independent of each other. Every device array
 * below is dense and row-major with the last index contiguous.
 *
 * Conventions for every entry point
 *   - plain C linkage; no exceptions, no abort(); the return value is an fg_status and
 *     fastgen_last_error() gives a message for the last failure on that context;
 *   - arguments are validated on the host before anything is launched;
 *   - all device work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and the call returns without synchronising;
 *   - "device" pointers are HIP device memory owned by the caller; inputs are only read
 *     and may be released once the stream has passed the call;
 *   - the library never allocates device memory: the caller supplies one workspace of
 *     fastgen_workspace_bytes() bytes which the context carves up (profiling scratch,
 *     the ragged cache pool, decode scratch). It must stay alive until fastgen_destroy().
 *   - calls on one context must be issued in stream order by one thread at a time.
 */
#ifndef FASTGEN_H_
#define FASTGEN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct fastgen_ctx fastgen_ctx; /* opaque, host memory, owned by the library */

typedef enum {
  FG_OK = 0,
  FG_EINVAL = 1, /* bad argument (null pointer, unsupported shape, misaligned pointer)   */
  FG_ENOMEM = 2, /* workspace too small / host allocation of the context failed          */
  FG_EHIP = 3,   /* a HIP call or kernel launch reported an error                        */
  FG_ESTATE = 4, /* call order violated (create -> profile -> compact -> decode_step...) */
  FG_ECAP = 5    /* more decode steps than max_new_tokens, or the cache pool overflowed  */
} fg_status;

typedef enum { FG_F32 = 0, FG_BF16 = 1 } fg_dtype;

/* Policy ids, in the order of the family of Eq. 2 (Sec. 3.4). */
enum {
  FG_POLICY_SPECIAL = 0,              /* C_special                        */
  FG_POLICY_SPECIAL_PUNCT = 1,        /* C_special+punct.                 */
  FG_POLICY_SPECIAL_PUNCT_FREQ = 2,   /* C_special+punct.+frequent        */
  FG_POLICY_SPECIAL_PUNCT_FREQ_LOCAL = 3, /* ...+local                    */
  FG_POLICY_FULL = 4,                 /* C_full                           */
  FG_NUM_POLICIES = 5
};

/* Token-class byte: which tokens C_special / C_punct. keep (Sec. 3.4). */
enum { FG_CLASS_SPECIAL = 1, FG_CLASS_PUNCT = 2 };

/* Components a hybrid policy is the union of (Sec. 3.4). cfg.family[c] is the component
 * mask of policy id c = 0..3; id 4 is always C_full. The default family is Eq. 2's:
 * {SPECIAL, SPECIAL|PUNCT, SPECIAL|PUNCT|FREQUENT, SPECIAL|PUNCT|FREQUENT|LOCAL}. Other
 * tables give the ablations of App. A.1 (a component left out, components added in another
 * order) and, with forced_policy, the fixed single-policy baselines of Sec. 5.1. */
enum { FG_COMP_SPECIAL = 1, FG_COMP_PUNCT = 2, FG_COMP_FREQUENT = 4, FG_COMP_LOCAL = 8 };

typedef struct {
  int32_t num_units;      /* U = sequences * layers * heads, > 0                              */
  int32_t num_seqs;       /* B; must divide U; unit u belongs to sequence u / (U / B)         */
  int32_t head_dim;       /* d: 64 or 128                                                     */
  int32_t dtype;          /* fg_dtype of Q, K, V, q, k, v, out and of the cache               */
  int32_t prompt_len;     /* n >= 1, the same for every sequence                              */
  int32_t max_new_tokens; /* S >= 0: decode steps the cache is sized for; n + S <= 131072     */
  double T;               /* recovery threshold of Eq. 1, 0 < T <= 1                          */
  double r_l;             /* local window  w = max(1, floor(r_l * n))   (ratio of INPUT len)  */
  double r_f;             /* frequent budget k_f(L) = floor(r_f * L)    (ratio of CURRENT len)*/
  float softmax_scale;    /* logits = scale * q.k ; 0 selects 1/sqrt(head_dim)                */
  int32_t forced_policy;  /* -1: adaptive (Eq. 1); 0..4: every unit uses this (usable) policy */
  int64_t cache_tokens;   /* capacity of the cache pool in tokens summed over all units;
                             0 selects the worst case U * (n + S)                             */
  int32_t family[4];      /* FG_COMP_* mask of policy ids 0..3; all zero selects Eq. 2's
                             family; otherwise a zero entry is an unused id. Eq. 1 takes the
                             cheapest usable policy reaching T (equal cost: smaller id)       */
  int32_t group_size;     /* G: query heads that share one K/V head (grouped-query attention;
                             0 or 1 = multi-head attention as in the paper, at most 16). The
                             cache and the policy belong to the K/V head. Arrays of queries
                             and outputs (Q, lse_opt, q, out) then have U * G units, query
                             head g of unit u at index u * G + g; Eq. 1 averages over the rows
                             of all G heads and the cumulative scores add their attention     */
} fg_config;

/* Size in bytes of the device workspace a context with this configuration needs
 * (0 if the configuration is invalid). Host-only computation. */
size_t fastgen_workspace_bytes(const fg_config* cfg);

/* Creates a context over `workspace` (device memory, 256-byte aligned, `bytes` long).
 * FG_EINVAL for a bad configuration, FG_ENOMEM if `bytes` is too small. The workspace is
 * not touched until the first profile call. */
fg_status fastgen_create(const fg_config* cfg, void* workspace, size_t bytes, fastgen_ctx** out);

/* Releases the host-side context. The workspace stays the caller's. NULL is accepted. */
fg_status fastgen_destroy(fastgen_ctx* ctx);

/* Token classes from token ids (Sec. 3.4: C_special keeps the special tokens such as the
 * begin-of-sentence or instruction markers, C_punct. the punctuation tokens): writes, for every
 * token, FG_CLASS_SPECIAL if its id is in special_ids, FG_CLASS_PUNCT if it is in punct_ids
 * (both bits if in both, 0 otherwise). Usable for the prompt ([B, n] ids -> token_class of
 * fastgen_profile) and for each decode step ([B] ids -> class_new).
 *   token_ids    device [count] int32.
 *   special_ids, punct_ids   HOST arrays of num_special / num_punct ids, at most 64 entries
 *                each (they travel as kernel arguments); NULL is accepted with a count of 0.
 *   token_class  device [count] uint8, written.
 * Stateless: needs no context. FG_EINVAL for null device pointers with count > 0, negative
 * counts or lists longer than 64; count == 0 launches nothing. */
fg_status fastgen_classify(const int32_t* token_ids, int64_t count, const int32_t* special_ids,
                           int32_t num_special, const int32_t* punct_ids, int32_t num_punct,
                           uint8_t* token_class, void* stream);

/* Stage 1a -- attention profiling and policy choice (Alg. 1, Sec. 3.3 Eq. 1, Sec. 3.4 Eq. 2).
 *   Q, K         device [U (Q: U * G), n, d] in cfg.dtype, 16-byte aligned: the prompt's
 *                queries/keys.
 *   token_class  device [B, n] uint8, FG_CLASS_* bits of every prompt token.
 *   lse_opt      NULL, or device [U * G, n] float: natural-log row log-sum-exp of the causal,
 *                scaled logits as a prefill attention kernel produces it; when given, the
 *                pass that computes it is skipped.
 *   policy       NULL or device [U] int32: chosen policy id of every unit.
 *   recovery     NULL or device [U, 5] double: R_c, the mean kept attention mass of policy c.
 *   kept_count   NULL or device [U, 5] int32: |K_c|, tokens policy c keeps at the end of
 *                the prompt.
 * The attention map itself is never written to memory. */
fg_status fastgen_profile(fastgen_ctx* ctx, const void* Q, const void* K,
                          const uint8_t* token_class, const float* lse_opt, int32_t* policy,
                          double* recovery, int32_t* kept_count, void* stream);

/* Stage 1a for callers that cannot allocate device memory and hold no workspace (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): fastgen_profile without
 * a context. The scratch its kernels need (row statistics, column and band sums, kept flags,
 * per-unit results) lives in a static device array of 32 MiB inside the library, one copy per
 * GPU, held until the process ends; the call allocates nothing, on the host or the device.
 *   cfg          the configuration fastgen_create would take (max_new_tokens and cache_tokens
 *                only size the slot reservation and do not matter here). The shape is limited
 *                by the array: U * n * (8 * G + 21) + 112 * U bytes, each of the twelve regions
 *                rounded up to 256 bytes, must not exceed 32 MiB (e.g. U * n <= 1.1 M tokens at
 *                G = 1); larger shapes return FG_ENOMEM and launch nothing.
 *   Q, K, token_class, lse_opt, policy, recovery, kept_count, stream: as for fastgen_profile;
 *                the caller owns inputs and outputs. The device that owns `stream` must be the
 *                current device.
 * Results are the same as fastgen_profile's for the same inputs. Every call on one GPU uses
 * that GPU's one array: calls that overlap on a GPU (two streams, two threads) race; calls on
 * one stream are ordered. Nothing of a previous call is read. There is no context to compact
 * from: follow with fastgen_create / fastgen_profile when the cache is wanted. On failure
 * fastgen_last_error(NULL) returns the message (per host thread). */
fg_status fastgen_profile_static(const fg_config* cfg, const void* Q, const void* K,
                                 const uint8_t* token_class, const float* lse_opt,
                                 int32_t* policy, double* recovery, int32_t* kept_count,
                                 void* stream);

/* Stage 1b -- compaction f(K, V, C) (Alg. 1): copies the rows of K, V [U, n, d] that the
 * unit's policy keeps into the context's ragged cache (ascending position), together with
 * each kept token's cumulative attention score, position and class. Needs a preceding
 * fastgen_profile on the same stream. */
fg_status fastgen_compact(fastgen_ctx* ctx, const void* K, const void* V, void* stream);

/* Stage 2 -- one decode step for every unit (Alg. 2 inner loop; policies of Sec. 3.4).
 *   q, k_new, v_new  device [U, d] (q: [U * G, d]) in cfg.dtype: the new token's
 *                    query/key/value per unit.
 *   class_new        device [B] uint8: FG_CLASS_* bits of the new token of each sequence.
 *   out              device [U * G, d] in cfg.dtype: softmax(scale * q K^T) V over the held
 *                    tokens including the new one.
 * After the output is formed the cumulative scores are updated (policies containing
 * `frequent`) and every unit's kept set is re-derived from its policy; evicted tokens are
 * released in place. FG_ECAP after max_new_tokens steps.
 * A cache pool that the caller made smaller than the reservations need (cfg.cache_tokens) is
 * found on the device, during fastgen_compact: the host cannot know it without synchronising,
 * so this call still returns FG_OK, its kernels return without touching memory and `out` is
 * left unwritten. The `status` output of fastgen_export_state reports it (FG_ECAP); a caller
 * that sets cache_tokens must read it once after fastgen_compact before trusting any output. */
fg_status fastgen_decode_step(fastgen_ctx* ctx, const void* q, const void* k_new,
                              const void* v_new, const uint8_t* class_new, void* out,
                              void* stream);

/* Stage 2 with the stability probe of Sec. 4 (accumulated attention score of each structure at
 * later decoding steps): fastgen_decode_step, and in addition
 *   step_recovery  device [U, 5] double: the mass that this step's attention row (over the
 *                  tokens held during the step) puts on the tokens of every member of the
 *                  policy family, evaluated at the current length as in Sec. 3.4 (special /
 *                  punctuation by class, frequent = the k_f(L) largest cumulative scores
 *                  including this step's attention, local = the last w positions); entry 4
 *                  (C_full) is the whole row. For a head on the full cache these are the
 *                  recoveries of Eq. 1 for the new row.
 * A probed step keeps the cumulative scores of every unit, not only of the policies that
 * contain `frequent`; outputs and kept sets are the same as without the probe. */
fg_status fastgen_decode_step_probe(fastgen_ctx* ctx, const void* q, const void* k_new,
                                    const void* v_new, const uint8_t* class_new, void* out,
                                    double* step_recovery, void* stream);

/* Reads back the cache state (test / checkpoint probe; Alg. 1 returns {C, K^, V^}).
 *   lengths    NULL or device [U] int32: tokens held by each unit.
 *   offsets    NULL or device [U + 1] int64: exclusive prefix sum of lengths.
 *   positions  NULL or device [capacity] int32: held token positions of unit u, ascending,
 *              at [offsets[u], offsets[u+1]); capacity must be >= the total held (the pool
 *              capacity cfg.cache_tokens / U*(n+S) always suffices).
 *   scores     NULL or device [capacity] double: cumulative attention score aligned with
 *              `positions` (meaningful for policies containing `frequent`).
 *   keys, values  NULL or device [capacity, d] in cfg.dtype: cached rows in the same order.
 *   status     NULL or device [1] int32: 0, or FG_ECAP if the cache pool overflowed. */
fg_status fastgen_export_state(fastgen_ctx* ctx, int32_t* lengths, int64_t* offsets,
                               int32_t* positions, double* scores, void* keys, void* values,
                               int32_t* status, void* stream);

/* Optional device-time accounting per phase (a tracing aid; off by default). When enabled,
 * every kernel group is bracketed by HIP events on the caller's stream. */
enum {
  FG_PHASE_SWEEP1 = 0,      /* QK^T -> row log-sum-exp                       */
  FG_PHASE_SWEEP2 = 1,      /* QK^T -> softmax -> column / band sums         */
  FG_PHASE_SELECT = 2,      /* top-k, recoveries, policy, kept flags + scan  */
  FG_PHASE_COMPACT = 3,     /* pool offsets + gather of kept rows            */
  FG_PHASE_DECODE_ATTN = 4, /* split-KV attention over the ragged cache      */
  FG_PHASE_DECODE_UPDATE = 5, /* merge, score update, evict in place         */
  FG_NUM_PHASES = 6
};
/* enable: 0 off; 1 every kernel group; N > 1 the prompt-time phases always and every N-th
 * decode step (a sample: an event record costs several microseconds on the stream). */
fg_status fastgen_enable_timing(fastgen_ctx* ctx, int enable);
/* Waits for the recorded events, then adds up and clears them.
 *   ms        host [FG_NUM_PHASES] double: device milliseconds per phase since the last read.
 *   launches  NULL or host [FG_NUM_PHASES] int64: kernel groups timed per phase. */
fg_status fastgen_read_timing(fastgen_ctx* ctx, double* ms, int64_t* launches);

/* Message for the last non-OK status returned on this context ("" if none). The string is
 * owned by the context and valid until the next call on it. With ctx == NULL: the message of
 * the calling thread's last failed fastgen_profile_static. */
const char* fastgen_last_error(const fastgen_ctx* ctx);

/* Library version string (static storage). */
const char* fastgen_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FASTGEN_H_ */
