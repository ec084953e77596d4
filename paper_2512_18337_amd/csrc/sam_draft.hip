// sam_draft: batched suffix-automaton draft lookup, one wavefront per session.
//
// Paper Sec. 5.4.2 / Alg. 4 (FollowTransitions): the drafts are a continuation, of a given
// length, of an earlier occurrence of the text verified so far, found by walking the automaton.
//
// The walk itself is a chain of dependent loads (state -> transition row -> next state), so a
// session cannot be made faster by adding lanes; the 64 lanes are used where there is width:
// the window is fetched with one coalesced load and broadcast lane by lane, a state's sorted
// transition row is searched 64 entries at a time (64-ary narrowing for the few very wide
// states such as the root), and the continuation is read and cut with one load and a ballot.
// Throughput comes from the sessions running side by side on different compute units.
#include <algorithm>

#include "common.h"
#include "sam_hash.h"

namespace {

// The overlay of an incrementally maintained automaton: transitions added or redirected since the
// last full flatten, in an open-addressing table keyed by (state, token).  Wave-uniform probe.
struct Overlay {
    const unsigned long long *key;
    const int32_t *dst;
    unsigned mask;                   // capacity - 1 (capacity a power of two, at most half full)
};

// The table of the transitions of very wide states (16-byte slots {key low, key high, destination, 0}).
struct WideTable {
    const int4 *slot;
    unsigned mask;                   // slots - 1; slot == nullptr: no table, search the sorted rows
};

__device__ __forceinline__ int wide_find(const WideTable &wt, int s, int c) {
    const unsigned long long k = ((unsigned long long)(unsigned)s << 32) | (unsigned)c;
    unsigned j = (unsigned)agentsam_hash64(k) & wt.mask;
    for (unsigned probes = 0; probes <= wt.mask; ++probes) {
        const int4 e = wt.slot[j];                           // one 16-byte (scalar) load per probe
        const unsigned long long kk = ((unsigned long long)(unsigned)e.y << 32) | (unsigned)e.x;
        if (kk == k) return e.z;
        if (kk == AGENTSAM_HASH_EMPTY) return -1;
        j = (j + 1) & wt.mask;
    }
    return -1;
}

__device__ __forceinline__ int link_len(int w) { return w < 0 ? -1 - w : w; }   // record field 3 without the wide flag

__device__ __forceinline__ int overlay_find(const Overlay &ov, int s, int c) {
    const unsigned long long k = ((unsigned long long)(unsigned)s << 32) | (unsigned)c;
    unsigned j = (unsigned)agentsam_hash64(k) & ov.mask;
    for (unsigned probes = 0; probes <= ov.mask; ++probes) {          // bounded even for a full table
        const unsigned long long kk = ov.key[j];
        if (kk == k) return ov.dst[j];
        if (kk == AGENTSAM_HASH_EMPTY) return -1;
        j = (j + 1) & ov.mask;
    }
    return -1;
}

__device__ __forceinline__ int wave_bcast(int v, int src_lane) { return __shfl(v, src_lane, 64); }

// Destination of the transition (row [r0,r1) sorted by token) labelled c, or -1.  Wave-uniform.
__device__ __forceinline__ int find_edge(const int32_t *__restrict__ edge_tok,
                                         const int32_t *__restrict__ edge_dst,
                                         int r0, int r1, int c, int lane) {
    int lo = r0, hi = r1;
    while (hi - lo > 64) {
        const int step = (hi - lo + 63) >> 6;
        const int idx = lo + lane * step;
        const bool le = (idx < hi) && (edge_tok[idx] <= c);
        const int j = __popcll(__ballot(le));              // sorted row: the lanes with tok <= c form a prefix
        if (j == 0) return -1;
        lo = lo + (j - 1) * step;
        hi = min(hi, lo + step);
    }
    const int idx = lo + lane;
    const bool in = idx < hi;
    const int tk = in ? edge_tok[idx] : -1;
    const int ds = in ? edge_dst[idx] : -1;
    const unsigned long long eq = __ballot(in && tk == c);
    if (eq == 0ull) return -1;
    return wave_bcast(ds, __ffsll((long long)eq) - 1);
}

// The flat automaton as the kernels see it.
struct FlatSam {
    const int32_t *row_ptr, *edge_tok, *edge_dst, *lastpos, *corpus;
    const int4 *state_rec;
    const int32_t *rows_end;         // maintained automaton only: states below rows_end[b] have a flattened row
};

// One step of the walk: consume token c from (state s, matched length l).  Afterwards s is the state
// of the longest suffix of (old match + c) that occurs in the memory and l its length.
// One 16-byte record per state {first token, its destination (or -2-d when the state has more
// transitions), suffix link, len of the link's state} makes the common step - a state with a single
// transition that matches - cost one dependent load.  s, l and every branch are wave-uniform and kept
// in scalar registers, so the record is fetched with a scalar load and the loop carries no exec-mask
// bookkeeping.  root_pref: the root's transition on c if the caller fetched it ahead, -2 if not.
template <bool OVERLAY>
__device__ __forceinline__ void consume_token(const FlatSam &A, const Overlay &ov, const WideTable &wt, int b, int root,
                                              int root_pref, int c, int lane, int &s, int &l) {
    for (;;) {
        if (root_pref != -2 && s == root) {
            if (root_pref >= 0) { s = root_pref; ++l; } else { l = 0; }
            return;
        }
        const int4 rec = A.state_rec[s];
        const int r0 = __builtin_amdgcn_readfirstlane(rec.x), r1 = __builtin_amdgcn_readfirstlane(rec.y);
        int dst = -1;
        if (r0 == c) {
            dst = r1 >= 0 ? r1 : -2 - r1;
        } else if (!OVERLAY) {
            if (r1 < -1 && c > r0) {                   // rows are sorted: c can only be further right
                if (wt.slot != nullptr && __builtin_amdgcn_readfirstlane(rec.w) < 0)
                    dst = __builtin_amdgcn_readfirstlane(wide_find(wt, s, c));
                else
                    dst = __builtin_amdgcn_readfirstlane(
                        find_edge(A.edge_tok, A.edge_dst, A.row_ptr[s] + 1, A.row_ptr[s + 1], c, lane));
            }
        } else if (r1 < -1) {
            // Maintained automaton: the record holds any one transition; the overlay overrides the
            // flattened row (a transition may have been redirected to a clone), and only states
            // that existed at the last flatten have a row at all.
            dst = __builtin_amdgcn_readfirstlane(overlay_find(ov, s, c));
            if (dst < 0 && s < __builtin_amdgcn_readfirstlane(A.rows_end[b])) {
                // The wide table mirrors the flattened rows of states that had more than
                // AGENTSAM_WIDE_DEGREE transitions at the last flatten; a maintained record no longer
                // carries that flag, the row's length still tells.
                const int e0 = __builtin_amdgcn_readfirstlane(A.row_ptr[s]);
                const int e1 = __builtin_amdgcn_readfirstlane(A.row_ptr[s + 1]);
                if (wt.slot != nullptr && e1 - e0 > AGENTSAM_WIDE_DEGREE)
                    dst = __builtin_amdgcn_readfirstlane(wide_find(wt, s, c));
                else
                    dst = __builtin_amdgcn_readfirstlane(find_edge(A.edge_tok, A.edge_dst, e0, e1, c, lane));
            }
        }
        if (dst >= 0) { s = dst; ++l; return; }
        if (s == root) { l = 0; return; }
        s = __builtin_amdgcn_readfirstlane(rec.z);
        l = link_len(__builtin_amdgcn_readfirstlane(rec.w));
    }
}

// Is the root a state whose transitions are in the wide table?  (Then they are fetched ahead, one
// window token per lane.)  Flattened automaton: the flag in its record; maintained copy: the
// length of its flattened row.
template <bool OVERLAY>
__device__ __forceinline__ bool root_in_wide_table(const FlatSam &A, const WideTable &wt, int b, int root) {
    if (wt.slot == nullptr) return false;
    if (!OVERLAY) return __builtin_amdgcn_readfirstlane(A.state_rec[root].w) < 0;
    if (root >= __builtin_amdgcn_readfirstlane(A.rows_end[b])) return false;
    return __builtin_amdgcn_readfirstlane(A.row_ptr[root + 1]) - __builtin_amdgcn_readfirstlane(A.row_ptr[root]) >
           AGENTSAM_WIDE_DEGREE;
}

// The root's transition on token c (per lane), for a root that root_in_wide_table() accepted.
template <bool OVERLAY>
__device__ __forceinline__ int root_transition(const Overlay &ov, const WideTable &wt, int root, int c) {
    if (OVERLAY) {
        const int d = overlay_find(ov, root, c);             // added or redirected since the last flatten
        if (d >= 0) return d;
    }
    return wide_find(wt, root, c);
}

// The proposal of (state s, matched length l): the tokens that followed the most recent occurrence
// that still has a continuation; all strings of one state share their end positions, so if this state
// has none, the next candidate is the suffix link's longest string.
__device__ __forceinline__ void emit_draft(const FlatSam &A, int b, int root, int s, int l, int k, int min_match, int sep,
                                           int corpus_end_b, int lane, int32_t *__restrict__ draft,
                                           int32_t *__restrict__ n_draft, int32_t *__restrict__ match_len,
                                           int32_t *__restrict__ match_end) {
    int L = l, e = -1;
    while (s != root) {
        const int lp = A.lastpos[s];
        if (lp >= 0) { e = lp; break; }
        const int4 rec = A.state_rec[s];
        s = rec.z;
        L = link_len(rec.w);
    }
    if (e < 0 || L < min_match) { e = -1; L = 0; }

    int n = 0;
    int tk = -1;
    if (e >= 0 && k > 0) {
        const int idx = e + 1 + lane;
        const bool in = (lane < k) && (idx < corpus_end_b);
        tk = in ? A.corpus[idx] : sep;
        const unsigned long long stop = __ballot(!(in && tk != sep));
        n = stop ? (__ffsll((long long)stop) - 1) : 64;
    }
    if (lane < k) draft[(int64_t)b * k + lane] = (lane < n) ? tk : -1;
    if (lane == 0) {
        n_draft[b] = n;
        match_len[b] = L;
        match_end[b] = e;
    }
}

template <bool OVERLAY>
__global__ __launch_bounds__(64) void sam_draft_kernel(
    const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ edge_tok,
    const int32_t *__restrict__ edge_dst, const int32_t *__restrict__ lastpos,
    const int32_t *__restrict__ corpus, const int4 *__restrict__ state_rec,
    const int32_t *__restrict__ root_arr, const int32_t *__restrict__ corpus_end,
    const int32_t *__restrict__ recent, const int32_t *__restrict__ recent_len,
    int m, int k, int min_match, int sep,
    int32_t *__restrict__ draft, int32_t *__restrict__ n_draft, int32_t *__restrict__ match_len,
    int32_t *__restrict__ match_end, Overlay ov, const int32_t *__restrict__ rows_end, WideTable wt,
    int lookups_per_session) {
    // one wavefront per lookup; a session may query several automata with the same window
    const int b = blockIdx.x;
    const int wb = b / lookups_per_session;
    const int lane = threadIdx.x;
    const FlatSam A{row_ptr, edge_tok, edge_dst, lastpos, corpus, state_rec, rows_end};
    const int root = __builtin_amdgcn_readfirstlane(root_arr[b]);
    const int ql = __builtin_amdgcn_readfirstlane(max(0, min(m, recent_len[wb])));
    // lane i holds the i-th token of the (right-aligned) window
    const int wtok = (lane < ql) ? recent[(int64_t)wb * m + (m - ql) + lane] : -1;

    // longest suffix of the window that occurs in the memory: state s, matched length l.
    // Every mismatch sends the walk back towards the root, so the root's transition is the lookup
    // made most often.  When the root is a wide state, all 64 of them (one per window token) are
    // fetched up front, side by side, one per lane, and the walk takes them from a register.
    int root_next = -2;                                        // -2: not fetched
    const bool root_ahead = root_in_wide_table<OVERLAY>(A, wt, b, root);
    if (root_ahead) root_next = (lane < ql) ? root_transition<OVERLAY>(ov, wt, root, wtok) : -1;

    int s = __builtin_amdgcn_readfirstlane(root), l = 0;
    for (int t = 0; t < ql; ++t) {
        const int c = __builtin_amdgcn_readlane(wtok, t);
        const int pref = root_ahead ? __builtin_amdgcn_readlane(root_next, t) : -2;
        consume_token<OVERLAY>(A, ov, wt, b, root, pref, c, lane, s, l);
    }
    emit_draft(A, b, root, s, l, k, min_match, sep, corpus_end[b], lane, draft, n_draft, match_len, match_end);
}

// Stateful form: the matched state of every session is carried from call to call, so a call consumes
// only the tokens committed since the previous one (Alg. 4: x_t is the current verified suffix; the
// decoder follows transitions from where it stands).  cur_state/cur_len: in and out.
template <bool OVERLAY>
__global__ __launch_bounds__(64) void sam_draft_step_kernel(
    FlatSam A, const int32_t *__restrict__ root_arr, const int32_t *__restrict__ corpus_end,
    const int32_t *__restrict__ new_tok, const int32_t *__restrict__ n_new, int max_new,
    int k, int min_match, int sep, int32_t *__restrict__ cur_state, int32_t *__restrict__ cur_len,
    int32_t *__restrict__ draft, int32_t *__restrict__ n_draft, int32_t *__restrict__ match_len,
    int32_t *__restrict__ match_end, Overlay ov, WideTable wt) {
    const int b = blockIdx.x;
    const int lane = threadIdx.x;
    const int root = __builtin_amdgcn_readfirstlane(root_arr[b]);
    int s = __builtin_amdgcn_readfirstlane(cur_state[b]);
    int l = __builtin_amdgcn_readfirstlane(cur_len[b]);
    if (s < 0 || l <= 0) { s = root; l = 0; }                // a fresh session
    // The memory may have grown since the state was stored: a state can have been split, its shorter
    // strings now living in a clone that became its suffix link.  The string of length l belongs to
    // the state r on the link path with len(link(r)) < l <= len(r).
    while (s != root) {
        const int4 rec = A.state_rec[s];
        if (link_len(__builtin_amdgcn_readfirstlane(rec.w)) < l) break;
        s = __builtin_amdgcn_readfirstlane(rec.z);
    }
    const int nn = __builtin_amdgcn_readfirstlane(max(0, min(max_new, n_new[b])));
    const bool root_wide = root_in_wide_table<OVERLAY>(A, wt, b, root);
    for (int t0 = 0; t0 < nn; t0 += 64) {                    // 64 tokens at a time, one per lane
        const int cnt = min(64, nn - t0);
        const int wtok = (lane < cnt) ? new_tok[(int64_t)b * max_new + t0 + lane] : -1;
        int root_next = -2;
        if (root_wide) root_next = (lane < cnt) ? root_transition<OVERLAY>(ov, wt, root, wtok) : -1;
        for (int t = 0; t < cnt; ++t) {
            const int c = __builtin_amdgcn_readlane(wtok, t);
            const int pref = root_wide ? __builtin_amdgcn_readlane(root_next, t) : -2;
            consume_token<OVERLAY>(A, ov, wt, b, root, pref, c, lane, s, l);
        }
    }
    if (lane == 0) { cur_state[b] = s; cur_len[b] = l; }
    emit_draft(A, b, root, s, l, k, min_match, sep, corpus_end[b], lane, draft, n_draft, match_len, match_end);
}

}  // namespace

extern "C" int sam_draft(const int32_t *len, const int32_t *link, const int32_t *row_ptr,
                         const int32_t *edge_tok, const int32_t *edge_dst, const int32_t *lastpos,
                         const int32_t *corpus, const int32_t *state_rec, const int32_t *root,
                         const int32_t *corpus_end,
                         const int32_t *recent, const int32_t *recent_len,
                         int32_t B, int32_t m, int32_t k, int32_t min_match, int32_t sep_token,
                         int32_t *draft, int32_t *n_draft, int32_t *match_len, int32_t *match_end,
                         const int32_t *wide_table, int64_t wide_slots, void *stream) {
    if (B < 0 || m < 1 || m > 64 || k < 0 || k > 64 || min_match < 0) return AGENTSAM_ERR_ARG;
    if (wide_table && (wide_slots < 2 || (wide_slots & (wide_slots - 1)) != 0 || wide_slots > (1ll << 31)))
        return AGENTSAM_ERR_ARG;
    if (B == 0) return AGENTSAM_OK;
    (void)len; (void)link;                                   // carried by state_rec
    if (!row_ptr || !lastpos || !state_rec || !root || !corpus_end || !recent || !recent_len ||
        !n_draft || !match_len || !match_end || (k > 0 && !draft))
        return AGENTSAM_ERR_NULL;
    // edge_tok / edge_dst / corpus may be NULL only for an automaton with no transitions (empty
    // memory): then every row is empty and nothing matches, so they are never dereferenced.
    AGENTSAM_LAUNCH(sam_draft_kernel<false>, dim3((unsigned)B), dim3(64), (hipStream_t)stream,
                    row_ptr, edge_tok, edge_dst, lastpos, corpus, (const int4 *)state_rec, root, corpus_end, recent, recent_len, (int)m, (int)k, (int)min_match, (int)sep_token, draft, n_draft, match_len, match_end, Overlay{nullptr, nullptr, 0u}, nullptr, WideTable{(const int4 *)wide_table, wide_table ? (unsigned)(wide_slots - 1) : 0u}, 1);
    return AGENTSAM_OK;
}

extern "C" int sam_draft_delta(const int32_t *row_ptr, const int32_t *edge_tok, const int32_t *edge_dst,
                               const int32_t *lastpos, const int32_t *corpus, const int32_t *state_rec,
                               const uint64_t *overlay_key, const int32_t *overlay_dst, int64_t overlay_cap,
                               const int32_t *rows_end, const int32_t *root, const int32_t *corpus_end,
                               const int32_t *recent, const int32_t *recent_len,
                               int32_t B, int32_t m, int32_t k, int32_t min_match, int32_t sep_token,
                               int32_t *draft, int32_t *n_draft, int32_t *match_len, int32_t *match_end,
                               const int32_t *wide_table, int64_t wide_slots, void *stream) {
    if (B < 0 || m < 1 || m > 64 || k < 0 || k > 64 || min_match < 0) return AGENTSAM_ERR_ARG;
    if (overlay_cap < 2 || (overlay_cap & (overlay_cap - 1)) != 0 || overlay_cap > (1ll << 31)) return AGENTSAM_ERR_ARG;
    if (wide_table && (wide_slots < 2 || (wide_slots & (wide_slots - 1)) != 0 || wide_slots > (1ll << 31)))
        return AGENTSAM_ERR_ARG;
    if (B == 0) return AGENTSAM_OK;
    if (!row_ptr || !lastpos || !state_rec || !overlay_key || !overlay_dst || !rows_end || !root || !corpus_end ||
        !recent || !recent_len || !n_draft || !match_len || !match_end || (k > 0 && !draft))
        return AGENTSAM_ERR_NULL;
    const Overlay ov{(const unsigned long long *)overlay_key, overlay_dst, (unsigned)(overlay_cap - 1)};
    AGENTSAM_LAUNCH(sam_draft_kernel<true>, dim3((unsigned)B), dim3(64), (hipStream_t)stream,
                    row_ptr, edge_tok, edge_dst, lastpos, corpus, (const int4 *)state_rec, root, corpus_end, recent, recent_len, (int)m, (int)k, (int)min_match, (int)sep_token, draft, n_draft, match_len, match_end, ov, rows_end, WideTable{(const int4 *)wide_table, wide_table ? (unsigned)(wide_slots - 1) : 0u}, 1);
    return AGENTSAM_OK;
}

extern "C" int sam_draft_step(const int32_t *row_ptr, const int32_t *edge_tok, const int32_t *edge_dst,
                              const int32_t *lastpos, const int32_t *corpus, const int32_t *state_rec,
                              const uint64_t *overlay_key, const int32_t *overlay_dst, int64_t overlay_cap,
                              const int32_t *rows_end, const int32_t *wide_table, int64_t wide_slots,
                              const int32_t *root, const int32_t *corpus_end,
                              const int32_t *new_tok, const int32_t *n_new, int32_t B, int32_t max_new,
                              int32_t k, int32_t min_match, int32_t sep_token,
                              int32_t *cur_state, int32_t *cur_len,
                              int32_t *draft, int32_t *n_draft, int32_t *match_len, int32_t *match_end,
                              void *stream) {
    if (B < 0 || max_new < 0 || k < 0 || k > 64 || min_match < 0) return AGENTSAM_ERR_ARG;
    const bool maintained = overlay_key != nullptr;
    if (maintained && (overlay_cap < 2 || (overlay_cap & (overlay_cap - 1)) != 0 || overlay_cap > (1ll << 31)))
        return AGENTSAM_ERR_ARG;
    if (wide_table && (wide_slots < 2 || (wide_slots & (wide_slots - 1)) != 0 || wide_slots > (1ll << 31)))
        return AGENTSAM_ERR_ARG;
    if (B == 0) return AGENTSAM_OK;
    if (!row_ptr || !lastpos || !state_rec || !root || !corpus_end || !n_new || (max_new > 0 && !new_tok) ||
        !cur_state || !cur_len || !n_draft || !match_len || !match_end || (k > 0 && !draft))
        return AGENTSAM_ERR_NULL;
    if (maintained && (!overlay_dst || !rows_end)) return AGENTSAM_ERR_NULL;
    const FlatSam A{row_ptr, edge_tok, edge_dst, lastpos, corpus, (const int4 *)state_rec, rows_end};
    const WideTable wt{(const int4 *)wide_table, wide_table ? (unsigned)(wide_slots - 1) : 0u};
    if (maintained) {
        const Overlay ov{(const unsigned long long *)overlay_key, overlay_dst, (unsigned)(overlay_cap - 1)};
        AGENTSAM_LAUNCH(sam_draft_step_kernel<true>, dim3((unsigned)B), dim3(64), (hipStream_t)stream,
                    A, root, corpus_end, new_tok, n_new, (int)max_new, (int)k, (int)min_match, (int)sep_token, cur_state, cur_len, draft, n_draft, match_len, match_end, ov, wt);
    } else {
        AGENTSAM_LAUNCH(sam_draft_step_kernel<false>, dim3((unsigned)B), dim3(64), (hipStream_t)stream,
                    A, root, corpus_end, new_tok, n_new, (int)max_new, (int)k, (int)min_match, (int)sep_token, cur_state, cur_len, draft, n_draft, match_len, match_end, Overlay{nullptr, nullptr, 0u}, wt);
    }
    return AGENTSAM_OK;
}

namespace {
// One thread per exported item: walk records and end positions are scattered; a new or redirected transition
// is put into the overlay table (linear probing; the slot of its key is claimed with a compare-and-swap,
// or found if an earlier delta put the key there, and the destination is overwritten).  The export hands
// out every key once, so two threads never write one slot.  The probe count is bounded by the table size.
__global__ __launch_bounds__(256) void sam_apply_delta_kernel(const int32_t *__restrict__ rec_idx, const int4 *__restrict__ rec_val,
                                                              int64_t n_rec, const int32_t *__restrict__ lp_idx,
                                                              const int32_t *__restrict__ lp_val, int64_t n_lp,
                                                              const unsigned long long *__restrict__ ov_key,
                                                              const int32_t *__restrict__ ov_dst, int64_t n_ov,
                                                              int4 *__restrict__ state_rec, int32_t *__restrict__ lastpos,
                                                              unsigned long long *__restrict__ table_key,
                                                              int32_t *__restrict__ table_dst, unsigned table_mask) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n_rec) state_rec[rec_idx[i]] = rec_val[i];
    if (i < n_lp) lastpos[lp_idx[i]] = lp_val[i];
    if (i < n_ov) {
        const unsigned long long k = ov_key[i];
        unsigned j = (unsigned)agentsam_hash64(k) & table_mask;
        for (unsigned probes = 0; probes <= table_mask; ++probes) {
            const unsigned long long was = atomicCAS(table_key + j, (unsigned long long)AGENTSAM_HASH_EMPTY, k);
            if (was == AGENTSAM_HASH_EMPTY || was == k) {
                table_dst[j] = ov_dst[i];
                break;
            }
            j = (j + 1) & table_mask;
        }
    }
}
}  // namespace

extern "C" int sam_apply_delta(const int32_t *rec_idx, const int32_t *rec_val, int64_t n_rec,
                               const int32_t *lastpos_idx, const int32_t *lastpos_val, int64_t n_lastpos,
                               const uint64_t *ov_key, const int32_t *ov_dst, int64_t n_ov,
                               int32_t *state_rec, int32_t *lastpos,
                               uint64_t *overlay_key, int32_t *overlay_dst, int64_t overlay_cap, void *stream) {
    if (n_rec < 0 || n_lastpos < 0 || n_ov < 0) return AGENTSAM_ERR_ARG;
    if ((n_rec > 0 && (!rec_idx || !rec_val || !state_rec)) || (n_lastpos > 0 && (!lastpos_idx || !lastpos_val || !lastpos)) ||
        (n_ov > 0 && (!ov_key || !ov_dst || !overlay_key || !overlay_dst)))
        return AGENTSAM_ERR_NULL;
    if (n_ov > 0 && (overlay_cap < 2 || (overlay_cap & (overlay_cap - 1)) != 0 || overlay_cap > (1ll << 31) || 2 * n_ov > overlay_cap))
        return AGENTSAM_ERR_ARG;
    const int64_t n = std::max(n_rec, std::max(n_lastpos, n_ov));
    if (n == 0) return AGENTSAM_OK;
    if ((n + 255) / 256 > 0x7fffffffll) return AGENTSAM_ERR_ARG;
    AGENTSAM_LAUNCH(sam_apply_delta_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), (hipStream_t)stream,
                    rec_idx, (const int4 *)rec_val, n_rec, lastpos_idx, lastpos_val, n_lastpos,
                    (const unsigned long long *)ov_key, ov_dst, n_ov, (int4 *)state_rec, lastpos,
                    (unsigned long long *)overlay_key, overlay_dst, (unsigned)(n_ov > 0 ? overlay_cap - 1 : 0));
    return AGENTSAM_OK;
}


// ------------------------------------------------------------------------------------------
// Several automata per session (Alg. 4: S_merged = MergeSAM(S_session, S_cross, weights); Sec. 5.4.2:
// the session's own context and the top-K retrieved contexts, weighted by their similarity scores).
// The automata are not physically merged: every (session, automaton) pair is one lookup of the kernel
// above, and the proposal of the automaton with the largest weight x matched length is taken.
// ------------------------------------------------------------------------------------------
namespace {
__global__ __launch_bounds__(64) void sam_select_kernel(const float *__restrict__ weight, const int32_t *__restrict__ c_draft,
                                                        const int32_t *__restrict__ c_n, const int32_t *__restrict__ c_len,
                                                        const int32_t *__restrict__ c_end, int /*B*/, int M, int k,
                                                        int32_t *__restrict__ draft, int32_t *__restrict__ n_draft,
                                                        int32_t *__restrict__ match_len, int32_t *__restrict__ match_end,
                                                        int32_t *__restrict__ source) {
    const int b = blockIdx.x, lane = threadIdx.x;
    int best = -1;
    float best_score = 0.f;
    int best_len = 0;
    for (int j = 0; j < M; ++j) {                            // uniform over the wavefront
        const int x = b * M + j;
        const int len = c_len[x];
        const float w = weight[x];
        if (c_n[x] <= 0 || !(w > 0.f)) continue;             // no proposal from this automaton (or it is switched off)
        const float score = w * (float)len;
        if (best < 0 || score > best_score || (score == best_score && len > best_len)) {
            best = j; best_score = score; best_len = len;
        }
    }
    const int x = b * M + (best < 0 ? 0 : best);
    if (lane < k) draft[(int64_t)b * k + lane] = best < 0 ? -1 : c_draft[(int64_t)x * k + lane];
    if (lane == 0) {
        n_draft[b] = best < 0 ? 0 : c_n[x];
        match_len[b] = best < 0 ? 0 : c_len[x];
        match_end[b] = best < 0 ? -1 : c_end[x];
        source[b] = best;
    }
}
}  // namespace

extern "C" int sam_draft_merged(const int32_t *row_ptr, const int32_t *edge_tok, const int32_t *edge_dst,
                                const int32_t *lastpos, const int32_t *corpus, const int32_t *state_rec,
                                const int32_t *root, const int32_t *corpus_end, const float *weight, int32_t M,
                                const int32_t *recent, const int32_t *recent_len,
                                int32_t B, int32_t m, int32_t k, int32_t min_match, int32_t sep_token,
                                int32_t *draft, int32_t *n_draft, int32_t *match_len, int32_t *match_end,
                                int32_t *source, void *workspace, size_t workspace_bytes,
                                const int32_t *wide_table, int64_t wide_slots, void *stream) {
    if (B < 0 || M < 1 || m < 1 || m > 64 || k < 0 || k > 64 || min_match < 0) return AGENTSAM_ERR_ARG;
    if ((int64_t)B * M > 0x7fffffffll) return AGENTSAM_ERR_ARG;
    if (wide_table && (wide_slots < 2 || (wide_slots & (wide_slots - 1)) != 0 || wide_slots > (1ll << 31)))
        return AGENTSAM_ERR_ARG;
    if (B == 0) return AGENTSAM_OK;
    if (!row_ptr || !lastpos || !state_rec || !root || !corpus_end || !weight || !recent || !recent_len ||
        !n_draft || !match_len || !match_end || !source || (k > 0 && !draft) || !workspace)
        return AGENTSAM_ERR_NULL;
    const size_t n = (size_t)B * M;
    if (workspace_bytes < n * (size_t)(k + 3) * sizeof(int32_t)) return AGENTSAM_ERR_WORKSPACE;
    int32_t *c_draft = (int32_t *)workspace, *c_n = c_draft + n * k, *c_len = c_n + n, *c_end = c_len + n;
    AGENTSAM_LAUNCH(sam_draft_kernel<false>, dim3((unsigned)n), dim3(64), (hipStream_t)stream,
                    row_ptr, edge_tok, edge_dst, lastpos, corpus, (const int4 *)state_rec, root, corpus_end, recent, recent_len, (int)m, (int)k, (int)min_match, (int)sep_token, c_draft, c_n, c_len, c_end, Overlay{nullptr, nullptr, 0u}, nullptr, WideTable{(const int4 *)wide_table, wide_table ? (unsigned)(wide_slots - 1) : 0u}, (int)M);
    AGENTSAM_LAUNCH(sam_select_kernel, dim3((unsigned)B), dim3(64), (hipStream_t)stream,
                    weight, c_draft, c_n, c_len, c_end, (int)B, (int)M, (int)k, draft, n_draft, match_len, match_end, source);
    return AGENTSAM_OK;
}
