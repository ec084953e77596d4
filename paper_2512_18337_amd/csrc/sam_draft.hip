// sam_draft: batched suffix-automaton draft lookup, one wavefront per session.
//
// Paper Sec. 5.4.2 / Alg. 4 (FollowTransitions): given the current verified suffix, follow
// the automaton's transitions to retrieve a matching continuation of a specified length.
//
// The walk itself is a chain of dependent loads (state -> transition row -> next state), so a
// session cannot be made faster by adding lanes; the 64 lanes are used where there is width:
// the window is fetched with one coalesced load and broadcast lane by lane, a state's sorted
// transition row is searched 64 entries at a time (64-ary narrowing for the few very wide
// states such as the root), and the continuation is read and cut with one load and a ballot.
// Throughput comes from the sessions running side by side on different compute units.
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
    const int root = __builtin_amdgcn_readfirstlane(root_arr[b]);
    const int ql = __builtin_amdgcn_readfirstlane(max(0, min(m, recent_len[wb])));
    // lane i holds the i-th token of the (right-aligned) window
    const int wtok = (lane < ql) ? recent[(int64_t)wb * m + (m - ql) + lane] : -1;

    // longest suffix of the window that occurs in the memory: state s, matched length l.
    // One 16-byte record per state {first token, its destination (or -2-d when the state has
    // more transitions), suffix link, len of the link's state} makes the common step - a state
    // with a single transition that matches - cost one dependent load.
    // s, l and every branch below are wave-uniform and kept in scalar registers, so the record is
    // fetched with a scalar load and the loop carries no exec-mask bookkeeping.
    // Every mismatch sends the walk back towards the root, so the root's transition is the lookup
    // made most often.  When the root is a wide state, all 64 of them (one per window token) are
    // fetched up front, side by side, one per lane, and the walk takes them from a register.
    int root_next = -2;                                        // -2: not fetched
    const bool root_ahead = !OVERLAY && wt.slot != nullptr && __builtin_amdgcn_readfirstlane(state_rec[root].w) < 0;
    if (root_ahead) root_next = (lane < ql) ? wide_find(wt, root, wtok) : -1;

    int s = __builtin_amdgcn_readfirstlane(root), l = 0;
    for (int t = 0; t < ql; ++t) {
        const int c = __builtin_amdgcn_readlane(wtok, t);
        for (;;) {
            if (root_ahead && s == root) {
                const int dst = __builtin_amdgcn_readlane(root_next, t);
                if (dst >= 0) { s = dst; ++l; } else { l = 0; }
                break;
            }
            const int4 rec = state_rec[s];
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
                            find_edge(edge_tok, edge_dst, row_ptr[s] + 1, row_ptr[s + 1], c, lane));
                }
            } else if (r1 < -1) {
                // Maintained automaton: the record holds any one transition; the overlay overrides the
                // flattened row (a transition may have been redirected to a clone), and only states
                // that existed at the last flatten have a row at all.
                dst = __builtin_amdgcn_readfirstlane(overlay_find(ov, s, c));
                if (dst < 0 && s < __builtin_amdgcn_readfirstlane(rows_end[b]))
                    dst = __builtin_amdgcn_readfirstlane(
                        find_edge(edge_tok, edge_dst, row_ptr[s], row_ptr[s + 1], c, lane));
            }
            if (dst >= 0) { s = dst; ++l; break; }
            if (s == root) { l = 0; break; }
            s = __builtin_amdgcn_readfirstlane(rec.z);
            l = link_len(__builtin_amdgcn_readfirstlane(rec.w));
        }
    }

    // most recent occurrence that still has a continuation; all strings of one state share their
    // end positions, so if this state has none, the next candidate is the suffix link's longest string
    int L = l, e = -1;
    while (s != root) {
        const int lp = lastpos[s];
        if (lp >= 0) { e = lp; break; }
        const int4 rec = state_rec[s];
        s = rec.z;
        L = link_len(rec.w);
    }
    if (e < 0 || L < min_match) { e = -1; L = 0; }

    int n = 0;
    int tk = -1;
    if (e >= 0 && k > 0) {
        const int idx = e + 1 + lane;
        const bool in = (lane < k) && (idx < corpus_end[b]);
        tk = in ? corpus[idx] : sep;
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
    hipLaunchKernelGGL(sam_draft_kernel<false>, dim3((unsigned)B), dim3(64), 0, (hipStream_t)stream,
                       row_ptr, edge_tok, edge_dst, lastpos, corpus, (const int4 *)state_rec, root, corpus_end,
                       recent, recent_len, (int)m, (int)k, (int)min_match, (int)sep_token,
                       draft, n_draft, match_len, match_end, Overlay{nullptr, nullptr, 0u}, nullptr,
                       WideTable{(const int4 *)wide_table, wide_table ? (unsigned)(wide_slots - 1) : 0u}, 1);
    AGENTSAM_LAUNCH_CHECK();
    return AGENTSAM_OK;
}

extern "C" int sam_draft_delta(const int32_t *row_ptr, const int32_t *edge_tok, const int32_t *edge_dst,
                               const int32_t *lastpos, const int32_t *corpus, const int32_t *state_rec,
                               const uint64_t *overlay_key, const int32_t *overlay_dst, int64_t overlay_cap,
                               const int32_t *rows_end, const int32_t *root, const int32_t *corpus_end,
                               const int32_t *recent, const int32_t *recent_len,
                               int32_t B, int32_t m, int32_t k, int32_t min_match, int32_t sep_token,
                               int32_t *draft, int32_t *n_draft, int32_t *match_len, int32_t *match_end,
                               void *stream) {
    if (B < 0 || m < 1 || m > 64 || k < 0 || k > 64 || min_match < 0) return AGENTSAM_ERR_ARG;
    if (overlay_cap < 2 || (overlay_cap & (overlay_cap - 1)) != 0 || overlay_cap > (1ll << 31)) return AGENTSAM_ERR_ARG;
    if (B == 0) return AGENTSAM_OK;
    if (!row_ptr || !lastpos || !state_rec || !overlay_key || !overlay_dst || !rows_end || !root || !corpus_end ||
        !recent || !recent_len || !n_draft || !match_len || !match_end || (k > 0 && !draft))
        return AGENTSAM_ERR_NULL;
    const Overlay ov{(const unsigned long long *)overlay_key, overlay_dst, (unsigned)(overlay_cap - 1)};
    hipLaunchKernelGGL(sam_draft_kernel<true>, dim3((unsigned)B), dim3(64), 0, (hipStream_t)stream,
                       row_ptr, edge_tok, edge_dst, lastpos, corpus, (const int4 *)state_rec, root, corpus_end,
                       recent, recent_len, (int)m, (int)k, (int)min_match, (int)sep_token,
                       draft, n_draft, match_len, match_end, ov, rows_end, WideTable{nullptr, 0u}, 1);
    AGENTSAM_LAUNCH_CHECK();
    return AGENTSAM_OK;
}

namespace {
__global__ __launch_bounds__(256) void sam_apply_delta_kernel(const int32_t *__restrict__ rec_idx, const int4 *__restrict__ rec_val,
                                                              int64_t n_rec, const int32_t *__restrict__ lp_idx,
                                                              const int32_t *__restrict__ lp_val, int64_t n_lp,
                                                              int4 *__restrict__ state_rec, int32_t *__restrict__ lastpos) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n_rec) state_rec[rec_idx[i]] = rec_val[i];
    if (i < n_lp) lastpos[lp_idx[i]] = lp_val[i];
}
}  // namespace

extern "C" int sam_apply_delta(const int32_t *rec_idx, const int32_t *rec_val, int64_t n_rec,
                               const int32_t *lastpos_idx, const int32_t *lastpos_val, int64_t n_lastpos,
                               int32_t *state_rec, int32_t *lastpos, void *stream) {
    if (n_rec < 0 || n_lastpos < 0) return AGENTSAM_ERR_ARG;
    if ((n_rec > 0 && (!rec_idx || !rec_val || !state_rec)) || (n_lastpos > 0 && (!lastpos_idx || !lastpos_val || !lastpos)))
        return AGENTSAM_ERR_NULL;
    const int64_t n = n_rec > n_lastpos ? n_rec : n_lastpos;
    if (n == 0) return AGENTSAM_OK;
    if ((n + 255) / 256 > 0x7fffffffll) return AGENTSAM_ERR_ARG;
    hipLaunchKernelGGL(sam_apply_delta_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                       rec_idx, (const int4 *)rec_val, n_rec, lastpos_idx, lastpos_val, n_lastpos,
                       (int4 *)state_rec, lastpos);
    AGENTSAM_LAUNCH_CHECK();
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
                                                        const int32_t *__restrict__ c_end, int B, int M, int k,
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
    hipLaunchKernelGGL(sam_draft_kernel<false>, dim3((unsigned)n), dim3(64), 0, (hipStream_t)stream,
                       row_ptr, edge_tok, edge_dst, lastpos, corpus, (const int4 *)state_rec, root, corpus_end,
                       recent, recent_len, (int)m, (int)k, (int)min_match, (int)sep_token,
                       c_draft, c_n, c_len, c_end, Overlay{nullptr, nullptr, 0u}, nullptr,
                       WideTable{(const int4 *)wide_table, wide_table ? (unsigned)(wide_slots - 1) : 0u}, (int)M);
    AGENTSAM_LAUNCH_CHECK();
    hipLaunchKernelGGL(sam_select_kernel, dim3((unsigned)B), dim3(64), 0, (hipStream_t)stream,
                       weight, c_draft, c_n, c_len, c_end, (int)B, (int)M, (int)k, draft, n_draft, match_len, match_end,
                       source);
    AGENTSAM_LAUNCH_CHECK();
    return AGENTSAM_OK;
}
