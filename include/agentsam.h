/*
 * agentsam.h - C ABI of the MI355X (gfx950) hot path of AgentSAM speculative
 * decoding: one speculative step over a batch of agent sessions.
 *
 *   sam_build / sam_append / sam_flatten   host-side online suffix automaton over a
 *                                          session (or multi-session) token memory
 *   sam_draft                              device: longest matched suffix of each session's
 *                                          recent tokens and up to k continuation tokens
 *   spec_verify_attn                       device: causal GQA attention of the 1+k
 *                                          verification rows over a paged KV cache
 *   spec_accept                            device: greedy argmax per row and the accepted
 *                                          draft prefix
 *
 * Conventions
 *   - Every function returns 0 (AGENTSAM_OK) or a negative AGENTSAM_ERR_* code; nothing is
 *     thrown across the boundary.  agentsam_strerror() gives the text.
 *   - "host" pointers are ordinary process memory; "device" pointers are HIP device memory
 *     of the current device.  The library never allocates or frees device memory: every
 *     device buffer (flattened automaton, workspace, outputs) belongs to the caller.
 *   - Device entry points only enqueue work on `stream` (a hipStream_t passed as void*,
 *     NULL = the default stream) and return; argument errors are reported synchronously,
 *     device-side results are valid after the caller synchronises the stream.
 *   - All integer arrays are int32 unless stated; all arrays are dense, row-major.
 */
#ifndef AGENTSAM_H
#define AGENTSAM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define AGENTSAM_OK                0
#define AGENTSAM_ERR_NULL         -1   /* a required pointer is NULL                           */
#define AGENTSAM_ERR_ARG          -2   /* a size or parameter is out of range                  */
#define AGENTSAM_ERR_UNSUPPORTED  -3   /* a valid but unsupported shape / dtype                */
#define AGENTSAM_ERR_WORKSPACE    -4   /* workspace smaller than spec_verify_attn_workspace()  */
#define AGENTSAM_ERR_NOMEM        -5   /* host allocation failed                               */
#define AGENTSAM_ERR_HIP          -6   /* a HIP launch failed (see hipGetLastError)            */
#define AGENTSAM_ERR_TOKEN        -7   /* a token id is negative                               */

#define AGENTSAM_F32   0
#define AGENTSAM_BF16  1

const char *agentsam_strerror(int code);

/* Per-call tuning word of spec_verify_attn and spec_verify_attn_workspace (the two must be given the
 * same word: the workspace layout depends on it).  0 lets the library choose everything; the fields
 * exist for experiments and for the tests of split invariance.  Results never depend on the word
 * beyond rounding (the split decides what each softmax weight is rounded against).
 *   schedule   how a bf16 batch is spread over the GPU: CHUNKS = every (session, kv head) stream cut into
 *              chunks, one workgroup per chunk; BALANCED = all streams laid end to end and cut into one
 *              equal share per resident workgroup; default: BALANCED when there are at least two streams
 *              per resident workgroup and the block table covers more than 8192 positions, else CHUNKS.
 *   cascade    shared-prefix run (bf16): ON = look for pages that all sessions list at the same place of
 *              their block tables and process them once per group of sessions instead of once per
 *              session; OFF = never; default: look when the K/V stream is large enough (>= 11 GB) for the
 *              detection to cost nothing.
 *   kv chunk   KV positions handled by one workgroup under the CHUNKS schedule (a multiple of 128,
 *              128 .. 2^30); default: chosen from the batch. */
#define AGENTSAM_ATTN_SCHEDULE_CHUNKS    ((uint64_t)1)
#define AGENTSAM_ATTN_SCHEDULE_BALANCED  ((uint64_t)2)
#define AGENTSAM_ATTN_CASCADE_OFF        ((uint64_t)1 << 2)
#define AGENTSAM_ATTN_CASCADE_ON         ((uint64_t)2 << 2)
#define AGENTSAM_ATTN_KV_CHUNK(positions) ((uint64_t)((positions) / 128) << 8)

/* ------------------------------------------------------------------------------------------
 * Suffix automaton over a token memory (paper Sec. 5.4.2: a request's context is indexed in a
 * suffix automaton that grows one token at a time, the verified tokens of every step included;
 * Alg. 4, BuildSAM and step 2).
 *
 * A memory is a sequence of non-negative token ids.  Several sessions may be concatenated in
 * one memory, each terminated by `sep_token`, an id no query ever contains (Sec. 5.4.2,
 * cross-session memory): matches then never span two sessions and drafts stop at a separator.
 * sam_t is opaque, host-resident and owned by the library until sam_free().
 * ---------------------------------------------------------------------------------------- */
typedef struct sam sam_t;

/* Build the automaton of tokens[0..n) (host pointer; n may be 0).  *out receives the handle. */
int sam_build(const int32_t *tokens, int64_t n, int32_t sep_token, sam_t **out);

/* Extend the automaton with n more tokens (host pointer): amortised O(1) hash operations per token
 * (the changes a maintained device copy needs are logged in O(1) per token as well; the walk that
 * finds which end positions moved is done once per sam_delta_export, see there). */
int sam_append(sam_t *s, const int32_t *tokens, int64_t n);

/* Sizes of the flattened form: states (root included), transitions, memory tokens. */
int sam_flat_sizes(const sam_t *s, int64_t *n_states, int64_t *n_edges, int64_t *n_tokens);

/* Write the flattened automaton into caller-provided HOST arrays (the caller uploads them):
 *   len[ns]       longest string of each state
 *   link[ns]      suffix link (state id, -1 for the root, which is local state 0)
 *   row_ptr[ns+1] CSR offsets of each state's transitions
 *   edge_tok[ne], edge_dst[ne]   transitions, sorted by token within a state
 *   lastpos[ns]   the largest end position of the state's strings that still has a
 *                 continuation (next token exists and is not sep_token), or -1
 *   corpus[nt]    the token memory itself
 *   state_rec[4*ns] one 16-byte record per state for the draft walk, so that following a
 *                 transition costs one dependent load in the common case:
 *                   [0] token of the state's first (smallest-token) transition, -1 if none
 *                   [1] its destination d if it is the only transition, -2-d if there are more
 *                       (the rest are found in the CSR row), -1 if none
 *                   [2] suffix link (as in link[])    [3] len of the suffix link's state (0 for the root),
 *                       stored as -1-len for a state with more than 64 transitions (see sam_wide_table)
 * Several automata can be packed back to back in one set of arrays: state ids (link,
 * edge_dst) are offset by state_base, row_ptr values by edge_base, lastpos by corpus_base,
 * and the pointers passed here address this automaton's slice (row_ptr[ns] of one slice is
 * row_ptr[0] of the next). */
int sam_flatten(const sam_t *s, int32_t state_base, int32_t edge_base, int32_t corpus_base,
                int32_t *len, int32_t *link, int32_t *row_ptr, int32_t *edge_tok,
                int32_t *edge_dst, int32_t *lastpos, int32_t *corpus, int32_t *state_rec);

/* Very wide states (the root, a few very frequent tokens) would take several dependent probes of
 * their sorted row per lookup.  Their transitions are therefore also offered in an open-addressing
 * table with one probe per lookup: 16-byte slots {key low, key high, destination, 0}, key =
 * state << 32 | token, linear probing with the hash of csrc/sam_hash.h, free slots hold key ~0.
 *   sam_wide_slots   the number of slots this automaton needs (a power of two, at most half full).
 *   sam_wide_table   inserts the automaton's wide transitions into table[4*slots] (HOST), which the
 *                    caller has filled with -1; automata packed in one set of arrays may share one
 *                    table (slots = a power of two >= the sum of their needs).
 * The table is optional for sam_draft (NULL: the sorted rows are searched). */
int sam_wide_slots(const sam_t *s, int64_t *slots);
int sam_wide_table(const sam_t *s, int32_t state_base, int32_t *table, int64_t slots);

void sam_free(sam_t *s);

/* ------------------------------------------------------------------------------------------
 * Keeping a device copy current without flattening again (Sec. 5.4.2: what a step verifies goes
 * into the automaton as the context grows; Alg. 4 step 2).
 *
 * After sam_flatten() the automaton records what a device copy of those arrays is missing once
 * sam_append() has run: states whose walk record or last eligible end position changed (new
 * states included), transitions added or redirected to a clone, and the new tokens.
 *
 *   sam_delta_sizes   counts of each; n_overlay = transitions logged since the last sam_flatten (an upper
 *                     bound of the distinct keys the overlay table must hold: keep its capacity >= twice
 *                     that), n_overlay_new = those logged since the last sam_delta_export; flat_states =
 *                     states covered by the last sam_flatten (only those have a transition row).
 *                     AGENTSAM_ERR_ARG before any flatten.
 *   sam_delta_export  writes, into caller-provided HOST arrays,
 *       rec_idx[n_rec], rec_val[4*n_rec]          state ids and their new 16-byte walk records; a
 *                                                 record of a maintained state names ANY one of its
 *                                                 transitions, flagged -2-d when there are others
 *       lastpos_idx[n_lastpos], lastpos_val[..]   state ids and their new lastpos
 *       ov_key[<= n_overlay_new], ov_dst[..]      the transitions added or redirected since the last
 *                                                 export (overlay_all = 0) or since the last sam_flatten
 *                                                 (overlay_all != 0, n_overlay entries at most: for a
 *                                                 table that had to be re-created larger), key =
 *                                                 state << 32 | token, every key once with its latest
 *                                                 destination; *n_ov_written = how many
 *       new_tokens[n_new_tokens]                  to be written at corpus[corpus_base + old length ..)
 *     and forgets these changes (the log of transitions is kept until the next sam_flatten).  Cost:
 *     proportional to what is exported; the last eligible end positions are brought up to date here
 *     (and in sam_delta_sizes), one walk towards the root per chain of suffix links that changed, not
 *     one per appended token.  Ids are offset by state_base / corpus_base as in sam_flatten.  The
 *     device arrays state_rec and lastpos must have room for the grown automaton (at most 2 states per
 *     token).
 *   sam_apply_delta   device: scatters the exported records and lastpos values into state_rec and lastpos
 *                     and inserts the exported transitions into the overlay table overlay_key[cap] /
 *                     overlay_dst[cap] (device; open addressing with linear probing and the hash of
 *                     csrc/sam_hash.h; free slots hold key ~0, which is how the caller creates it; cap a
 *                     power of two that keeps the table at most half full, see n_overlay).  All inputs
 *                     are device copies of the exported arrays.  One launch, O(delta).  A lookup on the
 *                     same arrays must not run at the same time (order them on the stream or with events).
 *   sam_reflatten_due *due = 1 when the log of transitions since the last sam_flatten has grown beyond
 *                     max_overlay_fraction of the transitions that flatten wrote (or there was none): time
 *                     to flatten again (on the builder's child thread: sam_builder_flatten) and to switch
 *                     the lookups to the new arrays and an empty overlay once they are uploaded.
 *   sam_draft_delta   device: sam_draft on a maintained copy.  A transition is looked up in the
 *                     state's record, then in the overlay, then - for states below rows_end[b], the
 *                     end of the state-id range that has flattened rows in session b's automaton -
 *                     in the flattened row.  Same outputs and limits as sam_draft.  wide_table /
 *                     wide_slots (optional, NULL / 0: none): what sam_wide_table wrote at or after
 *                     the last sam_flatten; the flattened rows with more than 64 transitions (as
 *                     row_ptr tells) are then looked up there instead of being searched.  It need
 *                     not follow later appends: the overlay is asked first.
 * ---------------------------------------------------------------------------------------- */
int sam_delta_sizes(const sam_t *s, int64_t *n_rec, int64_t *n_lastpos, int64_t *n_overlay, int64_t *n_overlay_new,
                    int64_t *n_new_tokens, int64_t *flat_states);

int sam_delta_export(sam_t *s, int32_t state_base, int32_t corpus_base,
                     int32_t *rec_idx, int32_t *rec_val, int32_t *lastpos_idx, int32_t *lastpos_val,
                     int32_t overlay_all, uint64_t *ov_key, int32_t *ov_dst, int64_t *n_ov_written, int32_t *new_tokens);

int sam_apply_delta(const int32_t *rec_idx, const int32_t *rec_val, int64_t n_rec,
                    const int32_t *lastpos_idx, const int32_t *lastpos_val, int64_t n_lastpos,
                    const uint64_t *ov_key, const int32_t *ov_dst, int64_t n_ov,
                    int32_t *state_rec, int32_t *lastpos,
                    uint64_t *overlay_key, int32_t *overlay_dst, int64_t overlay_cap, void *stream);

int sam_reflatten_due(const sam_t *s, double max_overlay_fraction, int32_t *due);

int sam_draft_delta(const int32_t *row_ptr, const int32_t *edge_tok, const int32_t *edge_dst,
                    const int32_t *lastpos, const int32_t *corpus, const int32_t *state_rec,
                    const uint64_t *overlay_key, const int32_t *overlay_dst, int64_t overlay_cap,
                    const int32_t *rows_end, const int32_t *root, const int32_t *corpus_end,
                    const int32_t *recent, const int32_t *recent_len,
                    int32_t B, int32_t m, int32_t k, int32_t min_match, int32_t sep_token,
                    int32_t *draft, int32_t *n_draft, int32_t *match_len, int32_t *match_end,
                    const int32_t *wide_table, int64_t wide_slots, void *stream);

/* ------------------------------------------------------------------------------------------
 * sam_draft_step: sam_draft with the matched state carried from call to call (Alg. 4, decoding
 * loop; Sec. 5.4.2: the lookup continues from the state the verified text has reached).  A call
 * consumes only the tokens committed since the previous call, so its cost does not depend on how
 * long the match is, and the match is not cut to a window.
 *
 *   cur_state[B], cur_len[B]   device, in and out: the state and length of the carried match.  A
 *                              session starts with cur_len = 0 (cur_state then ignored; any negative
 *                              cur_state also means a fresh session).  Otherwise the pair must be
 *                              what this entry point wrote for the same automaton, which may have
 *                              grown since (sam_append + sam_apply_delta): a state that was split
 *                              meanwhile is followed to the clone that now holds the string.  State
 *                              ids are creation order + state_base, so the pair stays valid across a
 *                              new sam_flatten as long as the automaton keeps its state_base.
 *   new_tok[B,max_new], n_new[B]   device: the tokens to consume, oldest first (n_new clipped to
 *                              [0,max_new]; no limit on max_new).
 * Definition of the carried length after token t_n, with the memory as it is at the call:
 *   L_n = max { l+1 : 0 <= l <= L_(n-1), the last l+1 tokens (t_(n-l) .. t_n) occur in the memory },
 *   0 if t_n does not occur.  On a memory that does not change this is the longest suffix of
 *   everything consumed so far; after the memory has grown it can be shorter than that (a longer
 *   match that only the new text makes possible is not looked for).
 * The proposal is the one sam_draft makes for a window of exactly those L_n tokens; outputs as
 * sam_draft.  Automaton arrays as sam_draft (overlay_key NULL: a flattened automaton, wide_table
 * optional) or as sam_draft_delta (overlay_key, overlay_dst, overlay_cap, rows_end given: a
 * maintained copy; wide_table optional, as there).
 * ---------------------------------------------------------------------------------------- */
int sam_draft_step(const int32_t *row_ptr, const int32_t *edge_tok, const int32_t *edge_dst,
                   const int32_t *lastpos, const int32_t *corpus, const int32_t *state_rec,
                   const uint64_t *overlay_key, const int32_t *overlay_dst, int64_t overlay_cap,
                   const int32_t *rows_end, const int32_t *wide_table, int64_t wide_slots,
                   const int32_t *root, const int32_t *corpus_end,
                   const int32_t *new_tok, const int32_t *n_new, int32_t B, int32_t max_new,
                   int32_t k, int32_t min_match, int32_t sep_token,
                   int32_t *cur_state, int32_t *cur_len,
                   int32_t *draft, int32_t *n_draft, int32_t *match_len, int32_t *match_end,
                   void *stream);

/* ------------------------------------------------------------------------------------------
 * Asynchronous construction (Sec. 5.4.2, asynchronous SAM construction; Alg. 4 step 2: the
 * automaton is extended off the decoding thread).  A builder owns one child thread, a
 * waiting queue and the automata of the requests submitted to it.
 *
 *   sam_builder_submit   copies the tokens (a prompt, or tokens generated since) into the queue and
 *                        returns at once; the request's automaton is created by its first entry.
 *   sam_builder_poll     *out = the request's automaton if none of its entries is waiting or being
 *                        processed, else NULL: the automaton is "not yet available" and the caller
 *                        decodes that request without drafts.  *pending_tokens = tokens not yet in it.
 *                        A returned automaton stays valid and unchanged until the caller's next submit
 *                        or release for that request (use it with sam_flatten, sam_delta_export, ...;
 *                        never sam_free it).  Returns the error of a failed background append, if any.
 *   sam_builder_flatten  queues a sam_flatten of the request's automaton (same arguments; the arrays are
 *                        HOST memory of the caller with room for cap_states / cap_edges / cap_tokens
 *                        entries, and must stay untouched until the request has nothing pending).  It
 *                        runs on the child thread after the entries submitted before it, so a grown
 *                        automaton is flattened again off the decoding thread.
 *                        sam_builder_flatten_result: AGENTSAM_OK once the last one has written the arrays,
 *                        AGENTSAM_ERR_WORKSPACE if they were too small (the automaton stays usable),
 *                        AGENTSAM_ERR_ARG if the request never had one.
 *   sam_builder_wait     blocks until the request has nothing pending.
 *   sam_builder_release  forgets the request; its automaton is freed (at once, or when the child
 *                        thread reaches its last entry).  The id may not be reused until then.
 *   sam_builder_destroy  stops the child thread (entries still waiting are abandoned) and frees
 *                        every automaton.
 * Calls on one builder may come from any thread; AGENTSAM_ERR_ARG for an unknown request id.
 * ---------------------------------------------------------------------------------------- */
typedef struct sam_builder sam_builder_t;

int sam_builder_create(sam_builder_t **out);
int sam_builder_submit(sam_builder_t *b, int64_t request_id, const int32_t *tokens, int64_t n, int32_t sep_token);
int sam_builder_poll(sam_builder_t *b, int64_t request_id, sam_t **out, int64_t *pending_tokens);
int sam_builder_flatten(sam_builder_t *b, int64_t request_id, int32_t state_base, int32_t edge_base, int32_t corpus_base,
                        int32_t *len, int32_t *link, int32_t *row_ptr, int32_t *edge_tok, int32_t *edge_dst,
                        int32_t *lastpos, int32_t *corpus, int32_t *state_rec, int64_t cap_states, int64_t cap_edges,
                        int64_t cap_tokens);
int sam_builder_flatten_result(sam_builder_t *b, int64_t request_id);
int sam_builder_wait(sam_builder_t *b, int64_t request_id);
int sam_builder_release(sam_builder_t *b, int64_t request_id);
void sam_builder_destroy(sam_builder_t *b);

/* ------------------------------------------------------------------------------------------
 * sam_draft (paper Sec. 5.4.2 and Alg. 4, FollowTransitions: the drafts are a continuation, of a
 * given length, of an earlier occurrence of the text verified so far).
 *
 * For each session b: feed its window recent[b, m-recent_len[b] .. m) (right-aligned) through
 * the automaton whose root is root[b]; this yields the longest suffix of the window that occurs
 * in the memory.  Among the occurrences that still have a continuation, the most recent one is
 * taken (falling back to shorter suffixes along the suffix links when none has), and the k tokens
 * after it are emitted, stopping before corpus_end[b] and before sep_token.
 *
 * Device inputs : the flattened arrays (len and link are not read: state_rec carries what the
 *                 walk needs of them); root[B], corpus_end[B] (exclusive end of the
 *                 session's memory in `corpus`), recent[B,m], recent_len[B] (0..m).
 * Device outputs: draft[B,k] (-1 padded), n_draft[B], match_len[B], match_end[B] (index into
 *                 `corpus`, -1 when nothing matched).  match_len < min_match gives no draft.
 * wide_table    : device copy of the sam_wide_table() table with wide_slots slots, or NULL.
 * Limits: 0 <= k <= 64, 1 <= m <= 64 (one wavefront holds a window), B >= 0. */
int sam_draft(const int32_t *len, const int32_t *link, const int32_t *row_ptr,
              const int32_t *edge_tok, const int32_t *edge_dst, const int32_t *lastpos,
              const int32_t *corpus, const int32_t *state_rec, const int32_t *root, const int32_t *corpus_end,
              const int32_t *recent, const int32_t *recent_len,
              int32_t B, int32_t m, int32_t k, int32_t min_match, int32_t sep_token,
              int32_t *draft, int32_t *n_draft, int32_t *match_len, int32_t *match_end,
              const int32_t *wide_table, int64_t wide_slots, void *stream);

/* ------------------------------------------------------------------------------------------
 * sam_draft_merged (Alg. 4, MergeSAM of the session's automaton with those of retrieved contexts;
 * Sec. 5.4.2: each automaton enters the merge with a weight taken from its similarity score).
 *
 * Every session queries M automata with the same window: root[B,M], corpus_end[B,M], weight[B,M]
 * (all automata live in the one set of flattened arrays).  The automata are not physically merged;
 * the paper gives no merge rule, so this library's reading is: each automaton proposes as in
 * sam_draft, and the proposal with the largest weight * match_len is taken (among automata with
 * weight > 0 that propose at least one token; on equal scores the longer match, then the lower
 * index).  source[b] = index of the automaton taken, -1 when none proposes (then n_draft = 0).
 * workspace: device scratch of B*M*(k+3) int32.  Other arguments, outputs and limits as sam_draft. */
int sam_draft_merged(const int32_t *row_ptr, const int32_t *edge_tok, const int32_t *edge_dst,
                     const int32_t *lastpos, const int32_t *corpus, const int32_t *state_rec,
                     const int32_t *root, const int32_t *corpus_end, const float *weight, int32_t M,
                     const int32_t *recent, const int32_t *recent_len,
                     int32_t B, int32_t m, int32_t k, int32_t min_match, int32_t sep_token,
                     int32_t *draft, int32_t *n_draft, int32_t *match_len, int32_t *match_end,
                     int32_t *source, void *workspace, size_t workspace_bytes,
                     const int32_t *wide_table, int64_t wide_slots, void *stream);

/* ------------------------------------------------------------------------------------------
 * spec_verify_attn (Alg. 4, validation by the main model: the attention of the pass in which the
 * target model scores the base token and the k drafts of every session at once).
 *
 *   R = 1+k query rows per session; row i sits at KV position seq_lens[b]-R+i and attends
 *   positions 0 .. seq_lens[b]-R+i (the K/V of the R new positions are already in the cache).
 *   out[b,i,h,:] = softmax_j(scale * q[b,i,h,:] . K_b[j, h/(Hq/Hkv), :]) . V_b[j, h/(Hq/Hkv), :]
 *
 * Device inputs : q[B,R,Hq,D]; k_cache, v_cache [num_pages,Hkv,page_size,D]; block_table
 *                 [B,max_pages] (page id of KV positions p*page_size..); seq_lens[B].
 *                 dtype selects f32 or bf16 storage of q/k/v; accumulation is fp32.
 *                 seq_lens[b] is taken as min(max(seq_lens[b], 0), max_pages*page_size).  A row whose
 *                 position seq_lens[b]-R+i is negative (seq_lens[b] < R) sees nothing: its output is
 *                 zeros (every row of an empty session); the other rows are computed as always.
 * Device output : out[B,R,Hq,D] in out_dtype.
 * workspace     : device scratch of at least spec_verify_attn_workspace() bytes (partial
 *                 results of the KV splits); contents need no initialisation.
 * Sessions may list the same pages (a shared prefix): results are those of the definition above
 * whatever is shared; see the cascade field of the tuning word for how sharing is used.
 * A page id outside [0,num_pages) is treated as a page of zeros (never dereferenced).
 * Supported: D in {64,128}; Hq % Hkv == 0; bf16 needs page_size % 32 == 0; scale > 0;
 * (Hq/Hkv)*R <= 192 for bf16, R <= 32 for f32. */
int spec_verify_attn_workspace(int32_t B, int32_t R, int32_t Hq, int32_t Hkv, int32_t D,
                               int32_t page_size, int32_t max_pages, int32_t dtype, uint64_t tuning,
                               size_t *bytes);

int spec_verify_attn(const void *q, const void *k_cache, const void *v_cache,
                     const int32_t *block_table, int32_t max_pages, const int32_t *seq_lens,
                     int32_t B, int32_t R, int32_t Hq, int32_t Hkv, int32_t D, int32_t page_size,
                     int64_t num_pages, float scale, int32_t dtype, int32_t out_dtype,
                     void *out, void *workspace, size_t workspace_bytes, uint64_t tuning, void *stream);

/* spec_verify_attn_static: spec_verify_attn for callers that cannot allocate device memory (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  Same arguments,
 * results and errors, but no workspace argument: the partial results go to a static device array
 * inside the library, AGENTSAM_STATIC_WORKSPACE_BYTES (32 MiB) per GPU, held until the process ends.
 * The call allocates nothing (no hipMalloc / hipFree, no allocating library routine).
 * AGENTSAM_ERR_WORKSPACE when spec_verify_attn_workspace() for the same arguments exceeds that size
 * (the headline batch, 64 sessions x 8 kv heads of 36 packed rows, needs 9.6 MB).  All calls on one
 * GPU share the one array: calls that overlap on a GPU (two streams, two threads) race and give
 * undefined results; calls ordered on one stream are safe.  The first call on a GPU looks the
 * array's address up (no device work): make it outside a graph capture. */
#define AGENTSAM_STATIC_WORKSPACE_BYTES (32u << 20)
int spec_verify_attn_static(const void *q, const void *k_cache, const void *v_cache,
                            const int32_t *block_table, int32_t max_pages, const int32_t *seq_lens,
                            int32_t B, int32_t R, int32_t Hq, int32_t Hkv, int32_t D, int32_t page_size,
                            int64_t num_pages, float scale, int32_t dtype, int32_t out_dtype,
                            void *out, uint64_t tuning, void *stream);

/* ------------------------------------------------------------------------------------------
 * spec_accept (Alg. 4: the matched draft prefix is committed and decoding goes on from the first
 * mismatch; Sec. 5.4.1: lossless, i.e. the output equals greedy decoding).
 *
 *   tgt[b,i]        = lowest index of the maximum of logits[b,i,:]   (NaN never wins)
 *   accept_len[b]   = number of leading drafts j < n_draft[b] with draft[b,j] == tgt[b,j]
 *   out_tokens[b,:] = tgt[b,0..accept_len[b]] (accepted drafts + bonus token), then -1
 *
 * Device inputs : logits[B,1+k,V] (f32 or bf16), draft[B,k], n_draft[B].
 * Device outputs: accept_len[B], out_tokens[B,1+k], tgt[B,1+k].
 * Limits: 0 <= k <= 64 (as sam_draft), V >= 1. */
int spec_accept(const void *logits, int32_t logits_dtype, const int32_t *draft,
                const int32_t *n_draft, int32_t B, int32_t k, int64_t V,
                int32_t *accept_len, int32_t *out_tokens, int32_t *tgt, void *stream);

/* ------------------------------------------------------------------------------------------
 * Host-side controllers of the serving loop (all pointers are host memory).
 *
 * Speculation depth (Sec. 5.4.2, adaptive switch for speculative decoding; Alg. 4 step 4: beyond
 * some context length or batch size validating the drafts costs more than they save).
 *
 *   spec_choose_k         from a measured table: k_values[n] (strictly increasing, k_values[0] = 0) and
 *                         t_step[n], the time of this path's step with that many drafts.  With every
 *                         draft accepted independently with probability p_accept, a step with k drafts
 *                         commits 1 + p + ... + p^k tokens and costs
 *                             t_step(k) + max(other_floor, other_per_row * batch * (1 + k)),
 *                         the second term being the layers outside this path (weights streamed once,
 *                         then work per verified row; pass 0, 0 for this path alone).
 *                         *k_star = the depth with the most committed tokens per unit of cost (the
 *                         smaller on equal rates), *gain = that rate over the rate of k = 0 (>= 1; may
 *                         be NULL).  Speculating pays iff p + ... + p^k > cost(k) / cost(0) - 1.
 *   spec_switch_frontier  the same choice over a grid: batches[nb] and contexts[nc] strictly increasing,
 *                         t_step[nb][nc][n_k].  k_star[nb][nc] as above; context_threshold[i] = the
 *                         largest grid context up to which k_star > 0 without interruption at
 *                         batches[i] (-1: none), batch_threshold[j] likewise along the batches at
 *                         contexts[j].  These are the two thresholds of spec_adaptive_k.
 *   spec_adaptive_k       the switch itself: *k_out = 0 if context_len > context_threshold or
 *                         batch > batch_threshold, else k.
 *
 * agentsched_pick (Alg. 3): which queued request to admit next.  Per request i: hit[i] = KV blocks it
 * would reuse, need[i] = new KV blocks it needs, prompt_tok[i] = prompt length, wait[i] = time waited.
 * With H = sum hit, U = max(0, free_blocks - H), D = sum need:
 *     lambda  = lambda_max * logistic(k * (D / (U + eps) - 1))                 price of a block
 *     w       = clamp(1 - lambda / lambda_max, 0, 1)
 *     cost_i  = w * prompt_tok[i] / tokens_per_block + (1 - w) * need[i]
 *     score_i = a * hit[i] - (b + lambda) * cost_i + c * wait[i]
 * *picked = the highest-scoring request with need[i] <= free_blocks (the earlier one on equal scores),
 * -1 if none fits.  score may be NULL.  a, b, c, k, lambda_max, eps are the deployment's constants (the
 * paper prints none).
 * ---------------------------------------------------------------------------------------- */
int spec_choose_k(const int32_t *k_values, const double *t_step, int32_t n, double p_accept, int32_t batch,
                  double other_floor, double other_per_row, int32_t *k_star, double *gain);

int spec_switch_frontier(const int32_t *batches, int32_t n_batches, const int64_t *contexts, int32_t n_contexts,
                         const int32_t *k_values, int32_t n_k, const double *t_step, double p_accept,
                         double other_floor, double other_per_row, int32_t *k_star, int64_t *context_threshold,
                         int32_t *batch_threshold);

int spec_adaptive_k(int32_t batch, int64_t context_len, int32_t k, int32_t batch_threshold,
                    int64_t context_threshold, int32_t *k_out);

int agentsched_pick(int64_t free_blocks, const int64_t *hit, const int64_t *need, const int64_t *prompt_tok,
                    const double *wait, int64_t n, double lambda_max, double k, double eps, double a, double b,
                    double c, int32_t tokens_per_block, double *lambda_out, double *score, int64_t *picked);

#ifdef __cplusplus
}
#endif
#endif /* AGENTSAM_H */
