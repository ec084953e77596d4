// Host-side online suffix automaton over a token memory, and its flattening to the
// arrays sam_draft reads on the device.
//
// Paper Sec. 5.4.2: a request's context is indexed in a suffix automaton that grows one token at
// a time (linear in the context length), the verified tokens of every step included; Alg. 4,
// BuildSAM and step 2.  The construction is the textbook online algorithm (new state, walk suffix
// links adding transitions, clone on a length mismatch).
//
// Storage is sized for memories of millions of tokens over vocabularies of ~150k ids:
// transitions live in one arena (per-state singly linked lists, needed to copy a state's
// transitions when it is cloned) and are found through one open-addressing hash keyed by
// (state, token), so a lookup is O(1) whatever the state's degree.
#include <algorithm>
#include <cstdint>
#include <cstring>
#include <new>
#include <vector>

#include "agentsam.h"
#include "sam_hash.h"

struct sam {
    int32_t sep = -1;
    int32_t last = 0;
    std::vector<int32_t> len, link, created_at, head;   // per state; created_at = -1 for clones/root
    std::vector<int32_t> e_tok, e_dst, e_next;          // transition arena
    std::vector<uint64_t> h_key;                        // hash: key -> arena index
    std::vector<int32_t> h_val;
    uint64_t h_mask = 0;
    uint64_t h_used = 0;
    std::vector<int32_t> corpus;

    // Incremental maintenance (Sec. 5.4.2: what a step verifies goes into the automaton as the context
    // grows; Alg. 4 step 2).  After a full sam_flatten the automaton keeps track of what the device copy
    // is missing: states whose walk record or last eligible end position changed, transitions added or
    // redirected (they go into an overlay hash table that the draft lookup consults before the flattened
    // transition rows), and the new tokens.
    mutable bool track = false;
    mutable int32_t flat_states = 0;                 // states of the last full flatten: rows exist below this id
    mutable int64_t flat_edges = 0;                  // transitions of the last full flatten
    mutable int64_t exported_tokens = 0;             // memory tokens the device copy already has
    mutable std::vector<int32_t> lp;                 // last eligible end position per state, as of the last propagation
    mutable std::vector<uint8_t> rec_dirty, lp_dirty;
    mutable std::vector<int32_t> rec_list, lp_list;
    mutable std::vector<int32_t> ov_state, ov_tok, ov_dst;   // every transition added or redirected since the flatten, in order
    mutable size_t ov_exported = 0;                  // log entries the last export has handed out
    // End positions that became eligible since the last propagation: (state of the prefix that ends there,
    // position), positions increasing.  Appending only logs the pair; propagate_lastpos() pushes them up
    // the suffix links, once per export instead of once per token.
    mutable std::vector<int32_t> pend_state, pend_pos;

    void mark_rec(int32_t v) {
        if (!track || rec_dirty[(size_t)v]) return;
        rec_dirty[(size_t)v] = 1;
        rec_list.push_back(v);
    }
    void mark_lp(int32_t v) const {
        if (!track || lp_dirty[(size_t)v]) return;
        lp_dirty[(size_t)v] = 1;
        lp_list.push_back(v);
    }
    // Position e is an end position of exactly the states on the suffix-link path from the state of the
    // prefix T[0..e] to the root (in the automaton as it is NOW: states split since e arrived have their
    // clones on that path), so its lastpos candidates are that path.  Newest position first: a walk stops
    // at the first state that already holds a later position, because end-position sets grow towards the
    // root and every state above holds at least as late a one.  A call therefore touches each state at
    // most once per distinct chain, however many tokens were appended since the last call.
    void propagate_lastpos() const {
        for (size_t i = pend_pos.size(); i-- > 0;) {
            const int32_t e = pend_pos[i];
            for (int32_t v = pend_state[i]; v != -1 && lp[(size_t)v] < e; v = link[(size_t)v]) {
                lp[(size_t)v] = e;
                mark_lp(v);
            }
        }
        pend_state.clear();
        pend_pos.clear();
    }

    static constexpr uint64_t kEmpty = ~0ull;

    static uint64_t mix(uint64_t k) { return agentsam_hash64(k); }
    static uint64_t key_of(int32_t st, int32_t tok) { return ((uint64_t)(uint32_t)st << 32) | (uint32_t)tok; }

    void rehash(uint64_t cap) {
        std::vector<uint64_t> nk(cap, kEmpty);
        std::vector<int32_t> nv(cap, -1);
        uint64_t mask = cap - 1;
        for (uint64_t i = 0; i < h_key.size(); ++i) {
            if (h_key[i] == kEmpty) continue;
            uint64_t j = mix(h_key[i]) & mask;
            while (nk[j] != kEmpty) j = (j + 1) & mask;
            nk[j] = h_key[i]; nv[j] = h_val[i];
        }
        h_key.swap(nk); h_val.swap(nv); h_mask = mask;
    }
    int32_t find(int32_t st, int32_t tok) const {       // arena index or -1
        uint64_t k = key_of(st, tok), j = mix(k) & h_mask;
        while (h_key[j] != kEmpty) {
            if (h_key[j] == k) return h_val[j];
            j = (j + 1) & h_mask;
        }
        return -1;
    }
    void add_edge(int32_t st, int32_t tok, int32_t dst) {
        if ((h_used + 1) * 10 > (h_mask + 1) * 6) rehash((h_mask + 1) * 2);
        int32_t e = (int32_t)e_tok.size();
        e_tok.push_back(tok); e_dst.push_back(dst); e_next.push_back(head[st]);
        head[st] = e;
        uint64_t k = key_of(st, tok), j = mix(k) & h_mask;
        while (h_key[j] != kEmpty) j = (j + 1) & h_mask;
        h_key[j] = k; h_val[j] = e; ++h_used;
        if (track) {
            ov_state.push_back(st); ov_tok.push_back(tok); ov_dst.push_back(dst);
            mark_rec(st);
        }
    }
    int32_t new_state(int32_t l, int32_t lk, int32_t created) {
        len.push_back(l); link.push_back(lk); created_at.push_back(created); head.push_back(-1);
        const int32_t v = (int32_t)len.size() - 1;
        if (track) {
            lp.push_back(-1); rec_dirty.push_back(0); lp_dirty.push_back(0);
            mark_rec(v); mark_lp(v);                         // a new state needs both of its device entries
        }
        return v;
    }
    void init(int32_t sep_token) {
        sep = sep_token;
        h_key.assign(1024, kEmpty); h_val.assign(1024, -1); h_mask = 1023; h_used = 0;
        new_state(0, -1, -1);
        last = 0;
    }
    void extend(int32_t c) {
        const int32_t pos = (int32_t)corpus.size();
        const int32_t prev_last = last;
        corpus.push_back(c);
        const int32_t cur = new_state(len[last] + 1, 0, pos);
        int32_t p = last;
        int32_t e = -1;
        while (p != -1 && (e = find(p, c)) < 0) {
            add_edge(p, c, cur);
            p = link[p];
        }
        if (p != -1) {
            const int32_t q = e_dst[e];
            if (len[p] + 1 == len[q]) {
                link[cur] = q;
            } else {
                const int32_t cl = new_state(len[p] + 1, link[q], -1);
                for (int32_t x = head[q]; x != -1; x = e_next[x]) add_edge(cl, e_tok[x], e_dst[x]);
                // the clone ends wherever q ended so far (positions still waiting in the log reach it through
                // the suffix links when they are propagated: q's link is the clone from now on)
                if (track) lp[(size_t)cl] = lp[(size_t)q];
                while (p != -1) {
                    const int32_t ee = find(p, c);
                    if (ee < 0 || e_dst[ee] != q) break;
                    e_dst[ee] = cl;
                    if (track) {
                        ov_state.push_back(p); ov_tok.push_back(c); ov_dst.push_back(cl);
                        mark_rec(p);
                    }
                    p = link[p];
                }
                link[q] = cl;
                link[cur] = cl;
                mark_rec(q);
            }
        }
        last = cur;
        // The previous position now has a continuation (unless the new token is the separator): it is
        // the most recent eligible end position of every string that ends there.  Logged here in O(1),
        // pushed up the suffix links by propagate_lastpos().
        if (track && pos >= 1 && c != sep) {
            pend_state.push_back(prev_last);
            pend_pos.push_back(pos - 1);
        }
    }
};

extern "C" {

const char *agentsam_strerror(int code) {
    switch (code) {
        case AGENTSAM_OK: return "ok";
        case AGENTSAM_ERR_NULL: return "a required pointer is NULL";
        case AGENTSAM_ERR_ARG: return "argument out of range";
        case AGENTSAM_ERR_UNSUPPORTED: return "unsupported shape or dtype";
        case AGENTSAM_ERR_WORKSPACE: return "workspace too small";
        case AGENTSAM_ERR_NOMEM: return "host allocation failed";
        case AGENTSAM_ERR_HIP: return "HIP launch failed";
        case AGENTSAM_ERR_TOKEN: return "negative token id";
        default: return "unknown error";
    }
}

static int check_tokens(const int32_t *t, int64_t n) {
    for (int64_t i = 0; i < n; ++i)
        if (t[i] < 0) return AGENTSAM_ERR_TOKEN;
    return AGENTSAM_OK;
}

int sam_append(sam_t *s, const int32_t *tokens, int64_t n) {
    if (!s || (n > 0 && !tokens)) return AGENTSAM_ERR_NULL;
    if (n < 0) return AGENTSAM_ERR_ARG;
    if ((int64_t)s->corpus.size() + n > (int64_t)0x3fffffff) return AGENTSAM_ERR_ARG;  // 2N states fit int32
    int rc = check_tokens(tokens, n);
    if (rc) return rc;
    try {
        s->corpus.reserve(s->corpus.size() + (size_t)n);
        for (int64_t i = 0; i < n; ++i) s->extend(tokens[i]);
    } catch (const std::bad_alloc &) {
        return AGENTSAM_ERR_NOMEM;
    }
    return AGENTSAM_OK;
}

int sam_build(const int32_t *tokens, int64_t n, int32_t sep_token, sam_t **out) {
    if (!out || (n > 0 && !tokens)) return AGENTSAM_ERR_NULL;
    if (n < 0) return AGENTSAM_ERR_ARG;
    *out = nullptr;
    sam *s = new (std::nothrow) sam();
    if (!s) return AGENTSAM_ERR_NOMEM;
    try {
        s->init(sep_token);
    } catch (const std::bad_alloc &) {
        delete s;
        return AGENTSAM_ERR_NOMEM;
    }
    int rc = sam_append(s, tokens, n);
    if (rc) { delete s; return rc; }
    *out = s;
    return AGENTSAM_OK;
}

int sam_flat_sizes(const sam_t *s, int64_t *n_states, int64_t *n_edges, int64_t *n_tokens) {
    if (!s) return AGENTSAM_ERR_NULL;
    if (n_states) *n_states = (int64_t)s->len.size();
    if (n_edges) *n_edges = (int64_t)s->e_tok.size();
    if (n_tokens) *n_tokens = (int64_t)s->corpus.size();
    return AGENTSAM_OK;
}

int sam_flatten(const sam_t *s, int32_t state_base, int32_t edge_base, int32_t corpus_base,
                int32_t *len, int32_t *link, int32_t *row_ptr, int32_t *edge_tok,
                int32_t *edge_dst, int32_t *lastpos, int32_t *corpus, int32_t *state_rec) {
    if (!s || !len || !link || !row_ptr || !lastpos || !state_rec) return AGENTSAM_ERR_NULL;
    const int64_t ns = (int64_t)s->len.size(), ne = (int64_t)s->e_tok.size(), nt = (int64_t)s->corpus.size();
    if ((ne > 0 && (!edge_tok || !edge_dst)) || (nt > 0 && !corpus)) return AGENTSAM_ERR_NULL;
    if (state_base < 0 || edge_base < 0 || corpus_base < 0) return AGENTSAM_ERR_ARG;
    if ((int64_t)state_base + ns > INT32_MAX || (int64_t)edge_base + ne > INT32_MAX ||
        (int64_t)corpus_base + nt > INT32_MAX) return AGENTSAM_ERR_ARG;
    try {
        // states by decreasing len (counting sort), to push end positions up the suffix links
        std::vector<int32_t> cnt((size_t)nt + 2, 0), order((size_t)ns);
        for (int64_t v = 0; v < ns; ++v) ++cnt[(size_t)s->len[v] + 1];
        for (size_t i = 1; i < cnt.size(); ++i) cnt[i] += cnt[i - 1];
        for (int64_t v = 0; v < ns; ++v) order[(size_t)cnt[(size_t)s->len[v]]++] = (int32_t)v;
        std::vector<int32_t> lp((size_t)ns, -1);
        for (int64_t v = 0; v < ns; ++v) {
            const int32_t p = s->created_at[v];
            if (p >= 0 && (int64_t)p + 1 < nt && s->corpus[(size_t)p + 1] != s->sep) lp[(size_t)v] = p;
        }
        for (int64_t i = ns - 1; i > 0; --i) {               // order[0] is the root
            const int32_t v = order[(size_t)i], u = s->link[v];
            if (u >= 0 && lp[(size_t)v] > lp[(size_t)u]) lp[(size_t)u] = lp[(size_t)v];
        }
        std::vector<std::pair<int32_t, int32_t>> tmp;
        int64_t at = 0;
        for (int64_t v = 0; v < ns; ++v) {
            len[v] = s->len[v];
            link[v] = s->link[v] < 0 ? -1 : s->link[v] + state_base;
            lastpos[v] = lp[(size_t)v] < 0 ? -1 : lp[(size_t)v] + corpus_base;
            row_ptr[v] = (int32_t)(at + edge_base);
            tmp.clear();
            for (int32_t x = s->head[v]; x != -1; x = s->e_next[x]) tmp.emplace_back(s->e_tok[x], s->e_dst[x]);
            if (tmp.size() > 1) std::sort(tmp.begin(), tmp.end());
            for (const auto &pr : tmp) {
                edge_tok[at] = pr.first;
                edge_dst[at] = pr.second + state_base;
                ++at;
            }
            int32_t *rec = state_rec + 4 * v;
            rec[0] = tmp.empty() ? -1 : tmp[0].first;
            rec[1] = tmp.empty() ? -1 : (tmp.size() == 1 ? tmp[0].second + state_base : -2 - (tmp[0].second + state_base));
            rec[2] = link[v];
            rec[3] = s->link[v] < 0 ? 0 : s->len[s->link[v]];
            if ((int64_t)tmp.size() > AGENTSAM_WIDE_DEGREE) rec[3] = -1 - rec[3];   // its row is also in the wide table
        }
        row_ptr[ns] = (int32_t)(at + edge_base);
        if (nt > 0) std::memcpy(corpus, s->corpus.data(), (size_t)nt * sizeof(int32_t));
        // from here on the automaton records what a device copy of these arrays will be missing
        s->track = true;
        s->flat_states = (int32_t)ns;
        s->flat_edges = ne;
        s->exported_tokens = nt;
        s->lp.swap(lp);
        s->rec_dirty.assign((size_t)ns, 0); s->lp_dirty.assign((size_t)ns, 0);
        s->rec_list.clear(); s->lp_list.clear();
        s->ov_state.clear(); s->ov_tok.clear(); s->ov_dst.clear();
        s->ov_exported = 0;
        s->pend_state.clear(); s->pend_pos.clear();
    } catch (const std::bad_alloc &) {
        return AGENTSAM_ERR_NOMEM;
    }
    return AGENTSAM_OK;
}

// States with more than AGENTSAM_WIDE_DEGREE transitions (the root, a few very frequent tokens): their
// sorted rows would take several dependent probes to search, so their transitions are also offered in an
// open-addressing table of 16-byte slots {key low, key high, destination, 0}, one probe per lookup.
static int64_t wide_transitions(const sam *s, std::vector<int32_t> *states) {
    int64_t total = 0;
    const size_t ns = s->len.size();
    for (size_t v = 0; v < ns; ++v) {
        int64_t deg = 0;
        for (int32_t x = s->head[v]; x != -1 && deg <= AGENTSAM_WIDE_DEGREE; x = s->e_next[(size_t)x]) ++deg;
        if (deg > AGENTSAM_WIDE_DEGREE) {
            for (int32_t x = s->head[v]; x != -1; x = s->e_next[(size_t)x]) ++total;
            if (states) states->push_back((int32_t)v);
        }
    }
    return total;
}

int sam_wide_slots(const sam_t *s, int64_t *slots) {
    if (!s || !slots) return AGENTSAM_ERR_NULL;
    const int64_t n = wide_transitions(s, nullptr);
    int64_t cap = 2;
    while (cap < 2 * n) cap *= 2;
    *slots = cap;
    return AGENTSAM_OK;
}

int sam_wide_table(const sam_t *s, int32_t state_base, int32_t *table, int64_t slots) {
    if (!s || !table) return AGENTSAM_ERR_NULL;
    if (state_base < 0 || slots < 2 || (slots & (slots - 1)) != 0) return AGENTSAM_ERR_ARG;
    try {
        std::vector<int32_t> states;
        const int64_t n = wide_transitions(s, &states);
        if (2 * n > slots) return AGENTSAM_ERR_ARG;          // at most half full (together with what is in it)
        const uint64_t mask = (uint64_t)slots - 1;
        for (int32_t v : states) {
            for (int32_t x = s->head[(size_t)v]; x != -1; x = s->e_next[(size_t)x]) {
                const uint64_t key = ((uint64_t)(uint32_t)(v + state_base) << 32) | (uint32_t)s->e_tok[(size_t)x];
                uint64_t j = agentsam_hash64(key) & mask;
                int64_t probes = 0;
                while (!(table[4 * j] == -1 && table[4 * j + 1] == -1)) {           // key ~0 marks a free slot
                    j = (j + 1) & mask;
                    if (++probes > slots) return AGENTSAM_ERR_ARG;                  // table full
                }
                table[4 * j] = (int32_t)(uint32_t)key;
                table[4 * j + 1] = (int32_t)(uint32_t)(key >> 32);
                table[4 * j + 2] = s->e_dst[(size_t)x] + state_base;
                table[4 * j + 3] = 0;
            }
        }
    } catch (const std::bad_alloc &) {
        return AGENTSAM_ERR_NOMEM;
    }
    return AGENTSAM_OK;
}

int sam_delta_sizes(const sam_t *s, int64_t *n_rec, int64_t *n_lastpos, int64_t *n_overlay, int64_t *n_overlay_new,
                    int64_t *n_new_tokens, int64_t *flat_states) {
    if (!s) return AGENTSAM_ERR_NULL;
    if (!s->track) return AGENTSAM_ERR_ARG;                  // nothing to be relative to: flatten first
    try {
        s->propagate_lastpos();                              // the count of changed end positions is known after this
    } catch (const std::bad_alloc &) {
        return AGENTSAM_ERR_NOMEM;
    }
    if (n_rec) *n_rec = (int64_t)s->rec_list.size();
    if (n_lastpos) *n_lastpos = (int64_t)s->lp_list.size();
    if (n_overlay) *n_overlay = (int64_t)s->ov_state.size();
    if (n_overlay_new) *n_overlay_new = (int64_t)(s->ov_state.size() - s->ov_exported);
    if (n_new_tokens) *n_new_tokens = (int64_t)s->corpus.size() - s->exported_tokens;
    if (flat_states) *flat_states = s->flat_states;
    return AGENTSAM_OK;
}

int sam_reflatten_due(const sam_t *s, double max_overlay_fraction, int32_t *due) {
    if (!s || !due) return AGENTSAM_ERR_NULL;
    if (!(max_overlay_fraction >= 0.0)) return AGENTSAM_ERR_ARG;
    *due = (!s->track || (double)s->ov_state.size() > max_overlay_fraction * (double)std::max<int64_t>(1, s->flat_edges)) ? 1 : 0;
    return AGENTSAM_OK;
}

int sam_delta_export(sam_t *s, int32_t state_base, int32_t corpus_base,
                     int32_t *rec_idx, int32_t *rec_val, int32_t *lastpos_idx, int32_t *lastpos_val,
                     int32_t overlay_all, uint64_t *ov_key, int32_t *ov_dst, int64_t *n_ov_written, int32_t *new_tokens) {
    if (!s || !n_ov_written) return AGENTSAM_ERR_NULL;
    if (!s->track) return AGENTSAM_ERR_ARG;
    try {
        s->propagate_lastpos();
    } catch (const std::bad_alloc &) {
        return AGENTSAM_ERR_NOMEM;
    }
    const size_t nr = s->rec_list.size(), nl = s->lp_list.size();
    const size_t ov0 = overlay_all ? 0 : s->ov_exported, ov1 = s->ov_state.size();
    const int64_t ntok = (int64_t)s->corpus.size() - s->exported_tokens;
    if ((nr > 0 && (!rec_idx || !rec_val)) || (nl > 0 && (!lastpos_idx || !lastpos_val)) ||
        (ov1 > ov0 && (!ov_key || !ov_dst)) || (ntok > 0 && !new_tokens))
        return AGENTSAM_ERR_NULL;
    if (state_base < 0 || corpus_base < 0) return AGENTSAM_ERR_ARG;
    if ((int64_t)state_base + (int64_t)s->len.size() > INT32_MAX ||
        (int64_t)corpus_base + (int64_t)s->corpus.size() > INT32_MAX) return AGENTSAM_ERR_ARG;
    // transitions: a later entry of the log overrides an earlier one with the same (state, token), so only
    // the last entry per key is handed out (newest first through a scratch table; the order of the list
    // then no longer matters to whoever inserts it)
    int64_t nw = 0;
    if (ov1 > ov0) {
        try {
            uint64_t cap = 2;
            while (cap < 2 * (uint64_t)(ov1 - ov0)) cap *= 2;
            std::vector<uint64_t> seen((size_t)cap, AGENTSAM_HASH_EMPTY);
            for (size_t i = ov1; i-- > ov0;) {
                const uint64_t key = ((uint64_t)(uint32_t)(s->ov_state[i] + state_base) << 32) | (uint32_t)s->ov_tok[i];
                uint64_t j = agentsam_hash64(key) & (cap - 1);
                while (seen[(size_t)j] != AGENTSAM_HASH_EMPTY && seen[(size_t)j] != key) j = (j + 1) & (cap - 1);
                if (seen[(size_t)j] == key) continue;
                seen[(size_t)j] = key;
                ov_key[nw] = key;
                ov_dst[nw] = s->ov_dst[i] + state_base;
                ++nw;
            }
        } catch (const std::bad_alloc &) {
            return AGENTSAM_ERR_NOMEM;                       // nothing has been forgotten yet
        }
    }
    *n_ov_written = nw;
    for (size_t i = 0; i < nr; ++i) {
        const int32_t v = s->rec_list[i];
        const int32_t h = s->head[(size_t)v];
        rec_idx[i] = v + state_base;
        int32_t *rec = rec_val + 4 * i;
        if (h < 0) {
            rec[0] = -1; rec[1] = -1;
        } else {                                             // any one transition; the others are in the overlay or the rows
            const int32_t d = s->e_dst[(size_t)h] + state_base;
            rec[0] = s->e_tok[(size_t)h];
            rec[1] = s->e_next[(size_t)h] == -1 ? d : -2 - d;
        }
        const int32_t lk = s->link[(size_t)v];
        rec[2] = lk < 0 ? -1 : lk + state_base;
        rec[3] = lk < 0 ? 0 : s->len[(size_t)lk];
        s->rec_dirty[(size_t)v] = 0;
    }
    for (size_t i = 0; i < nl; ++i) {
        const int32_t v = s->lp_list[i];
        lastpos_idx[i] = v + state_base;
        lastpos_val[i] = s->lp[(size_t)v] < 0 ? -1 : s->lp[(size_t)v] + corpus_base;
        s->lp_dirty[(size_t)v] = 0;
    }
    if (ntok > 0)
        std::memcpy(new_tokens, s->corpus.data() + s->exported_tokens, (size_t)ntok * sizeof(int32_t));
    s->rec_list.clear(); s->lp_list.clear();
    s->ov_exported = ov1;
    s->exported_tokens = (int64_t)s->corpus.size();
    return AGENTSAM_OK;
}

void sam_free(sam_t *s) { delete s; }

}  // extern "C"
