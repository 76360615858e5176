/*
 * sam.h - C ABI of the batched suffix-automaton draft library for AMD gfx950.
 *
 * The library implements the retrieval path of SAM-Decoding (arxiv 2411.10666):
 * for a batch of independent decoding sequences it keeps, in device memory,
 *   - one static suffix automaton built over a token corpus (Section 3.1), and
 *   - one dynamic suffix automaton per sequence, extended online with that
 *     sequence's own tokens (Section 3.1, Section 3.3),
 * and, per generation round, pushes the newly accepted tokens through both
 * (Transfer, Algorithm 1; Expand, Algorithm 2), picks the source by match
 * length (Section 3.2, "static only if l1 > l2 + l_bias") and reads the next
 * draft_len tokens after the earliest end position of the match (Section 3.2,
 * d = T[p+1 : p+n]).
 *
 * Conventions
 *   - Tokens are int32 in [0, vocab).  Arrays are 0-indexed and row-major.
 *   - "host" / "device" on a pointer says where the memory must live.  Device
 *     pointers are plain HIP device addresses on the current device.
 *   - States are numbered in the creation order of Algorithm 2: root 0; per
 *     token the new state, then the clone if one is made.
 *   - A state's end position is the paper's 1-indexed min_endpos (a prefix
 *     length), so the draft is the 0-indexed slice T[p : p+draft_len).
 *   - Every function returns SAM_OK (0) or a negative error code and never
 *     throws; sam_last_error() gives a thread-local message for the last
 *     failure on the calling thread.
 *   - Calls that take a stream enqueue work on it and return without waiting,
 *     except where a comment says the call synchronises.  `hip_stream` is a
 *     hipStream_t passed as void* (NULL = the default stream).
 *   - The caller owns all input and output buffers.  The library owns the two
 *     opaque handles and everything behind them.  A sam_corpus is immutable
 *     after sam_build and may be shared by any number of batches; it must
 *     outlive them.  Calls on one sam_batch must not overlap in time.
 */
#ifndef SAM_H_
#define SAM_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SAM_OK          0
#define SAM_EINVAL     -1   /* bad argument (null pointer, size out of range)   */
#define SAM_ENOMEM     -2   /* host or device allocation failed                 */
#define SAM_ECAPACITY  -3   /* a sequence would grow past max_seq_len           */
#define SAM_ETOKEN     -4   /* a token outside [0, vocab)                       */
#define SAM_EDEVICE    -5   /* a HIP call failed                                */

/* bits of the device-side status word (sam_batch_status) */
#define SAM_STATUS_CAPACITY  1u   /* some sequence hit max_seq_len; it was not advanced */
#define SAM_STATUS_TOKEN     2u   /* some sequence saw a token outside [0, vocab); that
                                     token and the rest of its row were not fed         */
#define SAM_STATUS_COUNT     4u   /* some count was < 0 or > max_accept; sequence skipped */
#define SAM_STATUS_INTERNAL  8u   /* a table walk hit its safety bound (corrupted tables,
                                     e.g. overlapping calls on one batch); results invalid */

/* values written to `source` */
#define SAM_SOURCE_NONE     0   /* match_len == 0, no draft */
#define SAM_SOURCE_DYNAMIC  1
#define SAM_SOURCE_STATIC   2
#define SAM_SOURCE_AUXILIARY 3  /* only with sam_batch_set_threshold: the match is not longer
                                   than the auxiliary drafter's virtual length           */

typedef struct sam_corpus sam_corpus;
typedef struct sam_batch  sam_batch;

const char *sam_last_error(void);

/* Digest of the source files this binary was compiled from (16 hex digits, set by the
 * build script; "unknown" for a build that did not pass one).  Lets a loader refuse a
 * binary that is older than the sources beside it. */
const char *sam_build_id(void);

/*
 * Build-SAM (Algorithm 2) over `corpus_tokens` on the host, then copy the
 * automaton to device memory as flat arrays: the corpus text, one record per
 * state with its suffix link, the link's length and up to two of its
 * transitions, a direct-indexed table of the root's transitions and a bucketed
 * open-addressed (state, token) -> {target, min_endpos(target)} hash that holds
 * the transitions of the states with more than two.  The device holds the
 * complete transition table while the records are made (sam_corpus_info
 * reports what stays afterwards).
 *   corpus_tokens : host, int32 [n_tokens]; a multi-document corpus is passed
 *                   already joined by a separator token (Section 3.1).
 *   n_tokens      : 1 .. 2^31-2, and at most about 10^9: the host's transition
 *                   table (4.29 slots per token) is indexed with 32 bits, a longer
 *                   corpus is refused with SAM_EINVAL.   vocab : 1 .. 2^31-1.
 *   out           : receives the handle; free it with sam_corpus_free.
 * Synchronises.  Errors: SAM_EINVAL, SAM_ETOKEN (a corpus token outside the
 * vocabulary), SAM_ENOMEM, SAM_EDEVICE.
 */
int sam_build(const int32_t *corpus_tokens, int64_t n_tokens, int32_t vocab,
              sam_corpus **out);

/*
 * Progress reports from sam_build / sam_build_host_only, for corpora that take
 * minutes: `fn` (NULL to switch off) is called on the building thread about every
 * 16 M tokens with phase "build", then during "finalize" and before "upload".
 * Process-wide; set it before the build call.
 */
typedef void (*sam_progress_fn)(const char *phase, int64_t done, int64_t total, void *user);
int sam_set_progress_callback(sam_progress_fn fn, void *user);

/*
 * Same host construction as sam_build but nothing is copied to a device, so it
 * runs on a machine without a GPU.  The handle can be inspected
 * (sam_corpus_info / _export / _find) but not used by sam_batch_init.
 */
int sam_build_host_only(const int32_t *corpus_tokens, int64_t n_tokens, int32_t vocab,
                        sam_corpus **out);

/*
 * Write a built corpus automaton to a file, and read one back instead of
 * building it (a 500 M-token corpus takes minutes to build).  The file holds the
 * host arrays as raw bytes behind a 64-byte header; it is valid for this library
 * layout version on a machine of the same byte order.  The top-k table is not
 * stored (sam_corpus_build_topk recomputes it).  sam_corpus_load copies the
 * automaton to the current device like sam_build; _host_only does not.  Loading
 * verifies the header, the file length and the consistency of every state and
 * transition, so a damaged file is refused.
 * Errors: SAM_EINVAL (cannot open, not such a file, damaged), SAM_ENOMEM,
 * SAM_EDEVICE.
 */
int sam_corpus_save(const sam_corpus *corpus, const char *path);
int sam_corpus_load(const char *path, sam_corpus **out);
int sam_corpus_load_host_only(const char *path, sam_corpus **out);

/* Counts of the built automaton and bytes of device memory it occupies
 * (0 for a host-only handle).  Any output pointer may be NULL. */
int sam_corpus_info(const sam_corpus *corpus, int64_t *n_states, int64_t *n_trans,
                    int64_t *device_bytes);

/*
 * Copy the host-side state table out, for inspection: length, link (-1 for the
 * root) and min_endpos per state, each host int32 [n_states].  Any may be NULL.
 */
int sam_corpus_export(const sam_corpus *corpus, int32_t *length, int32_t *link,
                      int32_t *min_endpos);

/* Host lookup of one transition through the same tables the device uses:
 * *target = next(state)[token], or -1 if there is none. */
int sam_corpus_find(const sam_corpus *corpus, int64_t state, int32_t token,
                    int64_t *target);

/*
 * Algorithm 3 (Appendix A.1): the frequency of every state (1 for states made by
 * expansion, 0 for clones and the root, plus the frequencies of all successors),
 * the k most frequent successors of every state (ties: smaller token id) and
 * their probabilities freq(successor) / freq(state), rounded to float.  Computed
 * on the host; if the corpus is on a device the table {token, target,
 * probability} x k per state is copied there (12*k bytes per state).  k: 1 .. 8.
 * May be called again with another k; synchronises the device.
 * Errors: SAM_EINVAL, SAM_ENOMEM, SAM_EDEVICE.
 */
int sam_corpus_build_topk(sam_corpus *corpus, int32_t k);

/*
 * Copy the host-side result of sam_corpus_build_topk out: freq host uint64
 * [n_states]; token, target host int32 [n_states, k] (-1 = unused entry); prob
 * host float [n_states, k].  Any may be NULL.
 */
int sam_corpus_export_topk(const sam_corpus *corpus, uint64_t *freq, int32_t *token,
                           int32_t *target, float *prob);

void sam_corpus_free(sam_corpus *corpus);

/*
 * Create a batch of `batch` sequences and ingest their prompts: every prompt
 * token goes through the static Transfer and the dynamic Transfer + Expand
 * (Section 3.3 applied to the prompt; Section 3.1 builds the dynamic automaton
 * over prompt and generated tokens alike).
 *   corpus         : from sam_build, or NULL for dynamic-only operation.
 *   prompt_tokens  : device, int32, all prompts concatenated.
 *   prompt_offsets : device, int64 [batch+1], prompt b is
 *                    prompt_tokens[offsets[b] : offsets[b+1]); non-decreasing.
 *   vocab          : token range when corpus is NULL; ignored (the corpus's
 *                    vocabulary is used) otherwise.
 *   max_seq_len    : capacity of every sequence (prompt + generated tokens),
 *                    1 .. 2^28.  Device memory is reserved for the worst case
 *                    (2*max_seq_len states; at most max_seq_len transitions
 *                    live outside the state records), so a sequence never
 *                    runs out of table space before it runs out of length.
 *   max_accept     : row length of `accepted` in sam_batch_step, 1 .. 4096.
 *   draft_len      : draft tokens per sequence, 1 .. 1024.
 *   l_bias         : the static source is chosen only if l1 > l2 + l_bias.
 * Synchronises (it reads the offsets back to validate them).  Errors:
 * SAM_EINVAL, SAM_ECAPACITY (a prompt longer than max_seq_len), SAM_ETOKEN
 * (reported after the ingest kernel ran), SAM_ENOMEM, SAM_EDEVICE.
 */
int sam_batch_init(const sam_corpus *corpus, const int32_t *prompt_tokens,
                   const int64_t *prompt_offsets, int32_t batch, int32_t vocab,
                   int32_t max_seq_len, int32_t max_accept, int32_t draft_len,
                   int32_t l_bias, void *hip_stream, sam_batch **out);

/*
 * sam_batch_init for callers that cannot allocate device memory: code running
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * The batch's tables (per-sequence text, state records, transition slots,
 * cursors, status word), which sam_batch_init allocates, live instead in a fixed
 * buffer of SAM_NOALLOC_MAX_BYTES that is part of the library's device code, one
 * copy per GPU, held until the process ends.  The call and every later call on
 * the returned batch (sam_batch_step, _replay, _debug, _sizes, _tree_draft, _free)
 * allocate and free no device memory.
 *   prompt_offsets_host : host, int64 [batch+1]; the same values as the device
 *                    array.  They are validated from this copy, so the call does
 *                    not read anything back and does not synchronise.
 *   all other arguments as for sam_batch_init.
 * Differences from sam_batch_init: asynchronous; a prompt token outside the
 * vocabulary is reported by sam_batch_status (SAM_STATUS_TOKEN), not by the
 * return code.  Sizes whose tables do not fit the buffer are refused with
 * SAM_EINVAL (the message names both sizes).  One such batch per GPU at a time:
 * a second call before sam_batch_free of the first returns SAM_EINVAL.  The
 * buffer keeps the previous batch's contents and is cleared by the call, on the
 * given stream, with kernels (no memset nodes); work of the previous batch that
 * is still running on another stream would race with it.
 * The handle is owned by the library; release it with sam_batch_free.
 * Errors: SAM_EINVAL, SAM_ECAPACITY (a prompt longer than max_seq_len),
 * SAM_EDEVICE.
 */
#define SAM_NOALLOC_MAX_BYTES (32 * 1024 * 1024)
int sam_batch_init_noalloc(const sam_corpus *corpus, const int32_t *prompt_tokens,
                           const int64_t *prompt_offsets, const int64_t *prompt_offsets_host,
                           int32_t batch, int32_t vocab, int32_t max_seq_len, int32_t max_accept,
                           int32_t draft_len, int32_t l_bias, void *hip_stream, sam_batch **out);

/*
 * One generation round for the whole batch, one kernel launch.  For sequence b
 * the first counts[b] tokens of row b of `accepted` are fed in order: static
 * Transfer per token (Algorithm 1), dynamic match on the automaton as it stands
 * and then Expand (Section 3.3, Algorithm 2).  Then the source is selected and
 * the draft read.
 *   accepted  : device, int32 [batch, max_accept].
 *   counts    : device, int32 [batch], each 0 .. max_accept.  0 leaves the
 *               sequence untouched and re-emits its current draft.
 *   match_len : device, int32 [batch]; length of the chosen match.
 *   draft     : device, int32 [batch, draft_len]; padded with -1.
 *   draft_len : device, int32 [batch]; tokens before the padding.  The draft
 *               is cut at the end of the source text.
 *   source    : device, int32 [batch]; SAM_SOURCE_*.
 * Asynchronous.  Device-side faults (capacity, bad token, bad count) never
 * touch another sequence; they set bits readable with sam_batch_status.
 * Errors: SAM_EINVAL, SAM_EDEVICE (launch failure).
 */
int sam_batch_step(sam_batch *batch, const int32_t *accepted, const int32_t *counts,
                   int32_t *match_len, int32_t *draft, int32_t *draft_len,
                   int32_t *source, void *hip_stream);

/*
 * A recorded schedule of n_steps generation rounds in ONE launch, for offline
 * replay and for measuring the path without launch gaps: every sequence runs
 * through its own rows on its own, so none waits for another's longest row.
 * The results are exactly those of n_steps calls of sam_batch_step.
 *   accepted : device, int32 [n_steps, batch, max_accept].
 *   counts   : device, int32 [n_steps, batch].
 *   match_len, draft_len, source : device, int32 [n_steps, batch].
 *   draft    : device, int32 [n_steps, batch, draft_len].
 * Asynchronous.  Device-side faults as in sam_batch_step (a faulty row is
 * skipped, the sequence goes on with its next row).
 * Errors: SAM_EINVAL, SAM_EDEVICE.
 */
int sam_batch_replay(sam_batch *batch, int32_t n_steps, const int32_t *accepted,
                     const int32_t *counts, int32_t *match_len, int32_t *draft,
                     int32_t *draft_len, int32_t *source, void *hip_stream);

/*
 * Tree draft from the static automaton (Section 3.2, Algorithm 4): for every
 * sequence, best-first expansion over the top-k successors starting at the static
 * cursor's state.  Entry 0 of a draft is the sequence's last token (parent -1,
 * probability 1); every further entry is a token, the index of its parent entry
 * and the product of the transition probabilities on its path (float, one
 * rounding per edge).  The largest probability is expanded first, ties go to the
 * entry created first.  A sequence with no tokens yet gets size 0.
 *   max_size : entries per draft including entry 0, 1 .. 128.
 *   tokens, parents : device, int32 [batch, max_size], padded with -1.
 *   probs    : device, float [batch, max_size], padded with 0.
 *   sizes    : device, int32 [batch].
 * Needs a corpus with a top-k table.  Asynchronous; does not change the batch.
 * Errors: SAM_EINVAL, SAM_EDEVICE.
 */
int sam_batch_tree_draft(sam_batch *batch, int32_t max_size, int32_t *tokens, int32_t *parents,
                         float *probs, int32_t *sizes, void *hip_stream);

/*
 * Recycle sequences of a live batch for new requests (continuous batching): each
 * listed sequence is forgotten (its dynamic automaton emptied, its static cursor
 * back at the root) and the new prompt is ingested exactly as sam_batch_init
 * does.  Other sequences are not touched.
 *   slots          : device, int32 [n_slots], distinct sequence indices in
 *                    [0, batch).
 *   prompt_tokens  : device, int32, the new prompts concatenated.
 *   prompt_offsets : device, int64 [n_slots+1]; prompt i (for sequence slots[i])
 *                    is prompt_tokens[offsets[i] : offsets[i+1]).
 * Reads slots and offsets back to validate them (synchronises the stream), then
 * enqueues the work and returns.  A bad prompt token raises SAM_STATUS_TOKEN.
 * Errors: SAM_EINVAL, SAM_ECAPACITY, SAM_ENOMEM, SAM_EDEVICE.
 */
int sam_batch_reset(sam_batch *batch, const int32_t *slots, int32_t n_slots,
                    const int32_t *prompt_tokens, const int64_t *prompt_offsets,
                    void *hip_stream);

/*
 * Hook for an auxiliary drafter (Section 3.4): the auxiliary method has the fixed
 * virtual match length l_threshold; from the next sam_batch_step on, a sequence
 * whose chosen match length is <= l_threshold gets source = SAM_SOURCE_AUXILIARY
 * (match_len, draft and draft_len are still those of the automaton, so the
 * caller may use either).  l_threshold < 0 (the initial state) switches the hook
 * off.  Host-side only; takes effect for launches enqueued after the call.
 */
int sam_batch_set_threshold(sam_batch *batch, int32_t l_threshold);

/*
 * Both cursors of every sequence, for checking: static (s1, l1) and dynamic
 * (s2, l2), each device int32 [batch]; any may be NULL.  The dynamic cursor is
 * the state holding the longest suffix of the sequence that also ends earlier
 * in it.  Asynchronous.
 */
int sam_batch_debug(const sam_batch *batch, int32_t *s1, int32_t *l1, int32_t *s2,
                    int32_t *l2, void *hip_stream);

/*
 * Per-sequence sizes of the dynamic automata: text length, states and
 * transitions, each device int32 [batch]; any may be NULL.  Asynchronous.
 */
int sam_batch_sizes(const sam_batch *batch, int32_t *text_len, int32_t *n_states,
                    int32_t *n_trans, void *hip_stream);

/* OR of the SAM_STATUS_* bits raised so far.  Synchronises the stream. */
int sam_batch_status(const sam_batch *batch, uint32_t *status, void *hip_stream);

/*
 * Testing aid.  Per-sequence tables come in two layouts: a compact one (16-bit
 * state ids; chosen when max_seq_len <= 16366 and vocab <= 131072) and a wide
 * one (32-bit ids, any size).  Bit 0 of mode makes every later sam_batch_init
 * in this process use the wide layout; bit 1 makes it size the per-sequence
 * slot tables as tightly as correctness allows (max_seq_len + 16 slots instead
 * of twice that), so that nearly full buckets and sweeps into the next bucket,
 * rare otherwise, happen all the time; bit 2 makes its kernels run the C++ form
 * of the two token loops instead of the assembly one; bit 3 makes every later
 * sam_build size the corpus automaton's transition table at 4.5 GiB whatever the
 * corpus (about that much host and device memory), so that table offsets beyond
 * 32 bits are reached with a corpus that builds in a moment; bit 4 makes the
 * step kernel of every later sam_batch_init run with its two prefetching waves,
 * which otherwise join for batches of 128 sequences or more and for corpus
 * automata larger than 256 MB; bit 5 keeps them
 * out whatever the batch size (for measuring what they cost and bring).  mode 0
 * restores the defaults.  Results are identical in every mode.
 */
int sam_set_layout_override(int mode);

/* Bytes of device memory the batch holds. */
int sam_batch_info(const sam_batch *batch, int64_t *device_bytes);

void sam_batch_free(sam_batch *batch);

/*
 * Measurement aid, not part of the method: what the memory system of the
 * current device delivers for the access patterns of the path, so that the
 * path's own throughput can be put beside it.  Allocates its own device
 * memory, runs on the default stream, returns when done.
 *   SAM_MEMBENCH_CHASE  : one wavefront follows `count` dependent loads, each of
 *                         a whole 128-byte line (the shape of a bucket probe),
 *                         through a pseudo-random cycle over `size` bytes
 *                         (a power of two); footprints up to 128 MiB are walked
 *                         once beforehand, larger ones start cold.
 *                         result = nanoseconds per load.
 *   SAM_MEMBENCH_GATHER : `workgroups` x 256 lanes, each `count` independent
 *                         random 16-byte reads from a table of `size` bytes.
 *                         result = reads per second.
 *   SAM_MEMBENCH_COPY   : device copy of `size` bytes.
 *                         result = bytes per second, read + written.
 *   SAM_MEMBENCH_LAUNCH : `count` back-to-back launches of an empty kernel of
 *                         `workgroups` x 128 lanes.  result = microseconds each.
 * Errors: SAM_EINVAL (sizes out of range), SAM_EDEVICE.
 */
#define SAM_MEMBENCH_CHASE  0
#define SAM_MEMBENCH_GATHER 1
#define SAM_MEMBENCH_COPY   2
#define SAM_MEMBENCH_LAUNCH 3
int sam_membench(int32_t kind, int64_t size, int64_t count, int32_t workgroups, double *result);

#ifdef __cplusplus
}
#endif
#endif /* SAM_H_ */
