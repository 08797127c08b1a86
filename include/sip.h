/*
 * sip.h -- C boundary of the MI355X (gfx950) batched token sampler.
 *
 * One call turns a [B, V] logits matrix into B token ids and their log-probabilities:
 * penalties from each row's token history, temperature, softmax, top-k / top-p / min-p
 * filtering and one seeded categorical draw per row.  This is the "Sampling" step at the
 * end of every decode iteration (paper Sec. 2.1 step 3,
 *   p = Filter(softmax(ApplyPenalty(z, y_<s) / tau); k, p),  y_s ~ Categorical(p);
 * restated operation by operation in Sec. 5.1).
 *
 * Conventions
 *  - Every pointer is a DEVICE pointer unless it says "host".  The caller owns every
 *    buffer.  The library allocates nothing, never synchronises and never writes to
 *    `logits`; all work is enqueued on `hip_stream` (a hipStream_t, NULL = default stream).
 *  - Errors are reported by return code only.  Argument errors are detected on the host
 *    before anything is enqueued; nothing has been written in that case.  Bad *data* in
 *    device memory (NaN logits, top_p <= 0, temperature < 0, history offsets that do not
 *    describe a CSR) gives unspecified results for the affected rows but never an
 *    out-of-bounds access: history offsets are clamped to [0, hist_nnz], token ids
 *    outside [0, V) are skipped.
 *  - Concurrent calls are allowed on different streams if they use different workspaces.
 *  - Same inputs, seed, step and row ids in a call of the same shape (B, V, dtype, sharding)
 *    give the same output bits on every call.  In a call of another shape a row's partial sums
 *    are grouped differently: its token id and best-n ids are still the same unless a decision
 *    of the row lies within rounding of a boundary (a uniform within 1e-6 of a CDF edge), and
 *    its log-probabilities agree within 1e-5 + 2^-22 * |logprob|.
 */
#ifndef SIP_H_
#define SIP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { SIP_F32 = 0, SIP_BF16 = 1 } sip_dtype;

typedef enum {
  SIP_OK = 0,
  SIP_ERR_INVALID_ARG = 1, /* NULL required pointer, non-positive size, misaligned rows, ... */
  SIP_ERR_UNSUPPORTED = 2, /* shape outside what the kernels are built for (see SIP_MAX_*) */
  SIP_ERR_WORKSPACE = 3,   /* workspace NULL, misaligned or smaller than sip_workspace_bytes() */
  SIP_ERR_HIP = 4,         /* a HIP runtime call (kernel launch) failed */
  SIP_ERR_TIMEOUT = 5,     /* sip_wait_ids(): the ticket did not appear in time */
  SIP_ERR_SCRATCH = 6      /* sip_sample_noalloc(): the call needs more scratch than the built-in array holds */
} sip_status;

#define SIP_MAX_V (1 << 19)        /* largest vocabulary the kernels support            */
#define SIP_MAX_B (1 << 20)        /* most rows of one call                             */
#define SIP_MAX_K_LOGPROBS 64      /* largest k_logprobs                                */
#define SIP_MAX_SHARDS 8           /* most vocabulary shards sip_sample_sharded() takes */
#define SIP_MAX_SLOTS (1 << 20)    /* most slots a sampler state can have               */
#define SIP_MAX_L (1 << 17)        /* longest history a slot of a sampler state can hold */

/*
 * Per-row sampling parameters (Sec. 2.1 step 3: tau, k, p; Sec. 7.1 "Workload" adds min-p
 * and the repetition / frequency / presence penalties).  A HOST struct of DEVICE arrays of
 * length B.  A NULL array switches the feature off for every row.
 */
typedef struct {
  const float* temperature;        /* NULL => 1.  0 => greedy row (lowest-index arg max).            */
  const int32_t* top_k;            /* NULL, <= 0 or >= V => off.  1 => greedy row.  Ties at the k-th
                                      largest value are all kept.                                   */
  const float* top_p;              /* NULL or >= 1 => off; otherwise in (0, 1).  Measured on the mass
                                      that survives top-k; ties at the cut are kept together.        */
  const float* min_p;              /* NULL or <= 0 => off; keeps p_v >= min_p * p_max, decided as
                                      fp32 (s_v - s_max) >= fp32(ln min_p).  Applied after top-p.     */
  const float* repetition_penalty; /* NULL or 1 => off; seen tokens: z > 0 ? z / r : z * r           */
  const float* frequency_penalty;  /* NULL or 0 => off; seen tokens: z -= f * count                  */
  const float* presence_penalty;   /* NULL or 0 => off; seen tokens: z -= p                          */
  const int64_t* row_id;           /* NULL => batch position b.  Otherwise the id that keys the
                                      row's random stream, so results do not depend on where a
                                      sequence sits in the batch.                                    */
} sip_params;

/*
 * Bytes of device scratch sip_sample() needs for this shape.  Depends only on its
 * arguments; returns 0 for an invalid shape.  The workspace must be 256-byte aligned; its
 * contents need not be preserved between calls and need not be initialised.
 *
 * Diagnostic: after a call has completed, the first 2 * B int32 of the workspace say, per row,
 * which code path finished it (path[B]) and what the finishing kernel made of it (why[B]).
 *   path: 1 = settled from the candidate list the one pass over the logits left behind; any
 *   other value = finished after reading the row again (normally from cache): 15 = from a second,
 *   longer candidate list (one more read of that row); 16 = by the row's workgroup over the whole
 *   row (plain temperature sampling without any filter: two more reads; a nucleus that reaches
 *   below the candidate list: four to six); anything else = the exact multi-pass path, the value
 *   naming the reason (2 top_k too large for any candidate list, 3-13 the candidate list could
 *   not prove the answer, 17-29 nor could the longer one, 14 vocabulary size outside the
 *   single-pass kernels).
 *   why: 1 = the finishing kernel settled the row; else why it passed the row on: 2 no list was
 *   made, 3 a chunk's list overflowed, 4 more distinct history tokens than the table of
 *   multiplicities holds, 5 list too long, 6 maximum not proven, 7 value span not representable,
 *   8 k-th / n-th largest not in the list, 9 too many equal values in one bin, 10 top_p <= 0,
 *   11 nucleus reaches below the list, 12 min-p cut below the list, 13 no filter at all,
 *   14 no mass / exact-only shape.
 * Results mean the same whichever path ran.
 *
 * Kernels of a call (names as a profiler shows them): stream_kernel (the one pass over the
 * logits), then finish_rescue_kernel for batches of no more rows than the device has compute
 * units, else finish_kernel followed by rescue_kernel (which returns at once when no row was
 * passed on); exact_kernel alone for vocabulary sizes outside the single-pass kernels.
 */
size_t sip_workspace_bytes(int32_t B, int32_t V, sip_dtype dtype, int64_t hist_nnz, int32_t k_logprobs);

/*
 * Sample one token per row (Sec. 2.1 step 3 (1)-(3)).
 *
 *  logits        [B, row_stride] row-major, fp32 or bf16 (SIP_BF16: raw 16-bit patterns);
 *                only the first V entries of a row are used (16-byte loads may touch the
 *                rest of the row's last 16-byte group); base pointer and
 *                row_stride * sizeof(element) must be multiples of 16 bytes; never written.
 *  params        host struct, see sip_params; NULL = every feature off.
 *  hist_indptr   [B+1] CSR offsets into hist_tokens: row b's previously generated tokens
 *                y_<s are hist_tokens[indptr[b] .. indptr[b+1]).  NULL (with hist_nnz = 0)
 *                = no history, penalties do nothing.
 *  hist_tokens   [hist_nnz] token ids; duplicates allowed (the count drives the frequency
 *                penalty); ids outside [0, V) are ignored.
 *  seed, step    key and counter of the Philox4x32-10 stream: counter = (row_id lo, row_id
 *                hi, step lo, step hi), key = (seed lo, seed hi); the row's uniform is the
 *                top 24 bits of output word 0 times 2^-24.
 *  out_ids       [B] sampled token per row.
 *  out_lp_ids    [B, 1 + k_logprobs] column 0: the sampled token; columns 1..k: the
 *  out_lp        k_logprobs most probable tokens, descending, ties lowest index first, and
 *                [B, 1 + k_logprobs] their log-probabilities = log-softmax over the full
 *                vocabulary of the penalised, temperature-scaled logits, before any filter
 *                (greedy rows: temperature taken as 1).  Both NULL iff k_logprobs < 0.
 *  workspace     device scratch of at least sip_workspace_bytes(...) bytes.
 *
 * Returns SIP_OK once everything is enqueued.
 */
sip_status sip_sample(const void* logits, int32_t B, int32_t V, int64_t row_stride, sip_dtype dtype,
                      const sip_params* params,
                      const int64_t* hist_indptr, const int32_t* hist_tokens, int64_t hist_nnz,
                      uint64_t seed, uint64_t step,
                      int32_t* out_ids, int32_t* out_lp_ids, float* out_lp, int32_t k_logprobs,
                      void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * ---- Vocabulary-sharded logits ---------------------------------------------------------------
 * With tensor parallelism of degree t the last pipeline stage's workers each hold B x V/t logits
 * (Sec. 5.1 (3), "pipelined integration": the paper's sampler puts the t pieces side by side
 * instead of gathering them on every worker).  sip_sample_sharded() takes the t pieces where they
 * are -- t base pointers, no concatenated copy: row b of the call is piece 0's row b, then piece
 * 1's, ..., so vocabulary id v lives in piece v / V_shard at column v % V_shard, and V = t * V_shard.
 * The result is defined as that of sip_sample() on the concatenated matrix (log-probabilities may
 * differ in the last bits: partial sums are formed per piece).
 *
 *  shard_logits  HOST array of t DEVICE pointers, each [B, shard_stride] row-major, 16-byte
 *                aligned; V_shard * sizeof(element) and shard_stride * sizeof(element) must be
 *                multiples of 16 bytes (else SIP_ERR_INVALID_ARG); never written.  The array is
 *                read before the call returns.
 *  t             1..SIP_MAX_SHARDS.
 *  workspace     at least sip_workspace_bytes_sharded(...) bytes: it includes room for B whole
 *                rows, used only by rows that leave the single-pass path (their workgroup puts
 *                the row together there first) and by shapes the single-pass kernels do not
 *                serve (V below 16384 or above 262144, V_shard below 8192).
 * Everything else as for sip_sample().
 */
size_t sip_workspace_bytes_sharded(int32_t B, int32_t V_shard, int32_t t, sip_dtype dtype, int64_t hist_nnz,
                                   int32_t k_logprobs);
sip_status sip_sample_sharded(const void* const* shard_logits, int32_t t, int32_t B, int32_t V_shard,
                              int64_t shard_stride, sip_dtype dtype, const sip_params* params,
                              const int64_t* hist_indptr, const int32_t* hist_tokens, int64_t hist_nnz,
                              uint64_t seed, uint64_t step, int32_t* out_ids, int32_t* out_lp_ids, float* out_lp,
                              int32_t k_logprobs, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * ---- Device-resident sampler state ---------------------------------------------------------
 * The counterpart, in device memory, of what Sec. 5.1 keeps on the host between iterations
 * ("memory reuse": a preallocated table of generated ids that each iteration appends to, instead
 * of a history rebuilt per call; "incremental penalty construction": per-iteration work that
 * grows with the B new tokens, not with the history).  A state holds `slots` histories of up to
 * `L_max` tokens.  A sequence keeps its slot for its whole life; sip_sample_state() reads each
 * row's history from its slot and appends the id it sampled; a finished sequence's slot is handed
 * to a new one with sip_state_assign().  Batches that are in flight at once (the p copies of the
 * sampler state the paper keeps for a pipeline of depth p) use disjoint slots of one state, or
 * states of their own.  A decode loop on a state is a pure sequence of enqueues: no host copy of
 * the history, no synchronisation, and nothing in it that a stream capture cannot record.
 *
 * Layout of the caller-owned, 256-byte aligned buffer (all little endian, part of this ABI so
 * that callers can read it back):
 *   byte 0    uint64  tick      sampling calls made on the state since sip_state_init()
 *   byte 8    uint32  overflow  ids that found their slot full, plus prompts cut to L_max
 *   byte 256  int32   len[slots]
 *   byte 256 + round_up(4 * slots, 256)       int32 distinct[slots]: distinct tokens in the slot's
 *                                             table below, -1 = the table has been given up
 *   byte 256 + 2 * round_up(4 * slots, 256)   int32 tokens[slots][L_max]
 *   after that, rounded up to 256             per slot a table token -> number of occurrences in
 *                                             the slot's history: uint32 key[4096] (0xFFFFFFFF =
 *                                             free), uint32 count[4096]; open addressing in 1024
 *                                             buckets of 4 slots, home bucket (token * 0x9E3779B1)
 *                                             >> 22.  Updated at the one new token per call
 *                                             (Sec. 5.1 "incremental penalty construction"); a
 *                                             history with more than 3072 distinct tokens gives
 *                                             its table up and is counted per call like a CSR.
 * Calls that touch the same SLOTS of a state must be ordered (same stream, or events between
 * streams); calls on disjoint sets of slots may be in flight at once on different streams with
 * different workspaces (the batches a pipeline keeps in flight): each takes its own value of the
 * call counter, in the order in which their first kernels happen to start.
 */

/* Bytes of a state with this shape; 0 if slots or L_max is not in 1..SIP_MAX_SLOTS / 1..SIP_MAX_L. */
size_t sip_state_bytes(int32_t slots, int32_t L_max);

/* Enqueue: every slot empty, tick = 0, overflow = 0.  `state` is a device buffer of at least
 * sip_state_bytes() bytes (else SIP_ERR_WORKSPACE).  Must precede any other use of the buffer. */
sip_status sip_state_init(void* state, size_t state_bytes, int32_t slots, int32_t L_max, void* hip_stream);

/*
 * Enqueue: hand n slots to new sequences.  Slot slot_ids[i] (device array [n]) forgets what it
 * held and takes tokens[indptr[i] .. indptr[i+1]) -- the sequence's history so far, normally its
 * prompt -- as its history; indptr (device, [n+1]) and tokens (device, [nnz]) may be NULL with
 * nnz = 0 for empty histories.  A prompt longer than L_max keeps its first L_max tokens and adds
 * one to `overflow`.  Entries of slot_ids outside [0, slots) are skipped; the same slot twice
 * in one call leaves either prompt.  n = 0 is allowed and does nothing.
 */
sip_status sip_state_assign(void* state, size_t state_bytes, int32_t slots, int32_t L_max, int32_t n,
                            const int32_t* slot_ids, const int64_t* indptr, const int32_t* tokens, int64_t nnz,
                            void* hip_stream);

/*
 * sip_sample() on a state (Sec. 2.1 step 3 with y_<s taken from, and y_s appended to, the state).
 * Arguments as for sip_sample() except:
 *  slot_of_row   device [B]: row b's history is slot slot_of_row[b] as it stands before this
 *                call.  A value outside [0, slots) = a row without history that leaves no trace.
 *                The slots named by one call must be distinct (otherwise one of the ids is kept).
 *  step          the Philox step of this call is step + tick, so that a recorded call, replayed,
 *                draws fresh numbers each time.
 *  workspace     at least sip_workspace_bytes(B, V, dtype, (int64_t)B * L_max, k_logprobs) bytes.
 * After the rows are sampled, out_ids[b] is appended to slot_of_row[b] (a full slot stays as it
 * is and `overflow` grows by one) and tick grows by one.  Same error behaviour as sip_sample():
 * an argument or workspace error is found before anything is enqueued and leaves the state as it is.
 */
sip_status sip_sample_state(const void* logits, int32_t B, int32_t V, int64_t row_stride, sip_dtype dtype,
                            const sip_params* params, void* state, size_t state_bytes, int32_t slots,
                            int32_t L_max, const int32_t* slot_of_row, uint64_t seed, uint64_t step,
                            int32_t* out_ids, int32_t* out_lp_ids, float* out_lp, int32_t k_logprobs,
                            void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * ---- Hand-off of the ids to the host without a stream synchronisation --------------------------
 * The scheduler of a pipelined server needs the B ids of a batch as soon as they exist, to send
 * them back to the first stage (Sec. 5.1: the sampler returns its output asynchronously; Sec. 6
 * "BIC-O": through a ring of slots that the consumer polls), while the device goes on with the
 * next batch.  sip_publish_ids(), enqueued after a sampling call on the same stream, copies the
 * ids into pinned host memory and then stores `ticket` into a host flag; a host thread waits for
 * the ticket with sip_wait_ids() -- plain loads, no hipStreamSynchronize, no hipMemcpy -- and
 * finds all B ids in place.  Tickets of successive calls on one flag must increase.
 *
 *  ids        device [B]: the out_ids of the sampling call.
 *  host_ids   [B] and host_flag: pinned host memory that the device can address (hipHostMalloc;
 *  host_flag  for such memory the host pointer is the device pointer); 4- and 8-byte aligned.
 *             The caller initialises the flag below its first ticket (say 0) before the first call.
 * A ring of (host_ids, host_flag) pairs lets several batches be in flight.
 */
sip_status sip_publish_ids(const int32_t* ids, int32_t B, int32_t* host_ids, uint64_t* host_flag, uint64_t ticket,
                           void* hip_stream);

/*
 * HOST function: spin until *host_flag >= ticket (acquire), at most timeout_ns nanoseconds
 * (UINT64_MAX: no limit).  SIP_OK: the ids published with that ticket are visible to the calling
 * thread.  SIP_ERR_TIMEOUT otherwise.  Touches no HIP call.
 */
sip_status sip_wait_ids(const uint64_t* host_flag, uint64_t ticket, uint64_t timeout_ns);

/*
 * ---- Everything in one call ---------------------------------------------------------------------
 * The entry points above each take one combination of where the logits are (one matrix / t
 * pieces) and where the histories are (CSR / state).  sip_sample_call() takes a description of
 * the call and allows every combination, with the hand-off to the host behind it if asked for:
 * what a tensor-parallel last stage of a pipeline does every iteration.  A HOST struct; zero it
 * and fill in what applies.  Meaning, alignment and error behaviour of every field as in the
 * entry point it comes from.
 */
typedef struct {
  /* logits: either one matrix ... */
  const void* logits;                /* [B, row_stride]; used when t_shards == 0                       */
  int64_t row_stride;
  int32_t V;                         /* used when t_shards == 0 (otherwise V = t_shards * V_shard)     */
  /* ... or t_shards pieces (sip_sample_sharded) */
  const void* const* shard_logits;   /* host array of t_shards device pointers                         */
  int32_t t_shards, V_shard;
  int64_t shard_stride;
  int32_t B;
  sip_dtype dtype;
  const sip_params* params;          /* NULL = every feature off                                       */
  /* histories: either a CSR ... */
  const int64_t* hist_indptr;
  const int32_t* hist_tokens;
  int64_t hist_nnz;
  /* ... or a device-resident state (sip_sample_state); state != NULL excludes the CSR */
  void* state;
  size_t state_bytes;
  int32_t slots, L_max;
  const int32_t* slot_of_row;
  uint64_t seed, step;
  int32_t* out_ids;
  int32_t* out_lp_ids;
  float* out_lp;
  int32_t k_logprobs;
  /* hand-off (sip_publish_ids); both NULL = none */
  int32_t* host_ids;
  uint64_t* host_flag;
  uint64_t ticket;
  void* workspace;                   /* at least sip_call_workspace_bytes(call) bytes                  */
  size_t workspace_bytes;
  void* hip_stream;
  /* Prompt tokens handed in separately from the generated ones (Sec. 2.1 defines y_<s as the generated
   * tokens, a sequence as prompt plus output): a CSR like the history's, device pointers, NULL / 0 =
   * none.  The repetition penalty then applies to the tokens of prompt and history together, the
   * frequency and presence penalties to those of the history alone.  Not with a state (whose slots
   * hold prompt and output as one history): SIP_ERR_INVALID_ARG. */
  const int64_t* prompt_indptr;      /* [B+1]                                                          */
  const int32_t* prompt_tokens;      /* [prompt_nnz]; ids outside [0, V) are ignored                   */
  int64_t prompt_nnz;
} sip_call;

/* Workspace the call needs (workspace / workspace_bytes / outputs of `call` are not looked at);
 * 0 if the description is invalid. */
size_t sip_call_workspace_bytes(const sip_call* call);
sip_status sip_sample_call(const sip_call* call);

/*
 * One-time set-up for the calling thread's current device: raises the dynamic-LDS limit of the
 * kernels that need more than the default and looks up the address of the built-in scratch
 * array of sip_sample_noalloc().  Every entry point does this by itself on its first call on a
 * device, but that first call then contains HIP calls that a stream capture cannot record:
 * call sip_init() once per device (with that device current) before capturing a graph whose
 * first node would otherwise be the library's first call on the device.  Idempotent and
 * thread-safe.  SIP_ERR_HIP if the runtime refuses.
 */
sip_status sip_init(void);

/*
 * ---- For callers that cannot allocate ---------------------------------------------------------
 * sip_sample() with the workspace taken from an array that is part of the library's device code
 * instead of from the caller: for callers that cannot call hipMalloc where they sample (code
 * under stream capture, tight serving loops, harnesses that forbid allocation).  Arguments,
 * results and error behaviour are those of sip_sample(); the call makes no hipMalloc / hipFree
 * and no allocating library call.
 *
 *  - The array holds sip_noalloc_scratch_bytes() bytes on every device the library runs on, for
 *    the life of the process.  A call whose sip_workspace_bytes() exceeds that is rejected on the
 *    host with SIP_ERR_SCRATCH before anything is enqueued.
 *  - All calls on one device share that device's array: calls that overlap in time on one device
 *    (different streams without an ordering between them) race.  Calls on one stream are safe.
 *  - The per-row path codes (see sip_workspace_bytes) are not available to the caller.
 */
size_t sip_noalloc_scratch_bytes(void);
sip_status sip_sample_noalloc(const void* logits, int32_t B, int32_t V, int64_t row_stride, sip_dtype dtype,
                              const sip_params* params,
                              const int64_t* hist_indptr, const int32_t* hist_tokens, int64_t hist_nnz,
                              uint64_t seed, uint64_t step,
                              int32_t* out_ids, int32_t* out_lp_ids, float* out_lp, int32_t k_logprobs,
                              void* hip_stream);

/* Host string for a status code (static storage, never NULL). */
const char* sip_status_string(sip_status status);

/* Library version: major * 10000 + minor * 100 + patch. */
int sip_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SIP_H_ */
