// Driver for the host side of the library (automaton builder, delta export, asynchronous builder,
// controllers), meant to be compiled together with those sources under AddressSanitizer +
// UndefinedBehaviorSanitizer, or ThreadSanitizer, and run on the CPU: every output array has exactly the
// size the API asks for, so any write past it is reported.  Prints "ok" and exits 0 when nothing is found.
#include <atomic>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <thread>
#include <vector>

#include "agentsam.h"

#define REQUIRE(x) do { if (!(x)) { std::printf("FAILED line %d: %s\n", __LINE__, #x); std::exit(1); } } while (0)

static uint64_t rng_state = 88172645463325252ull;
static uint32_t rnd() { rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17; return (uint32_t)(rng_state >> 11); }

// text with repeats (copies of earlier spans), a separator now and then
static std::vector<int32_t> make_text(size_t n, int vocab, int sep) {
    std::vector<int32_t> t;
    while (t.size() < n) {
        if (t.size() > 50 && rnd() % 3 == 0) {
            size_t p = rnd() % (t.size() - 20), len = 2 + rnd() % 40;
            for (size_t i = 0; i < len && t.size() < n; ++i) t.push_back(t[p + i] == sep ? 0 : t[p + i]);
        } else if (rnd() % 200 == 0) t.push_back(sep);
        else t.push_back((int32_t)(rnd() % vocab));
    }
    return t;
}

struct Flat {
    std::vector<int32_t> len, link, row_ptr, edge_tok, edge_dst, lastpos, corpus, rec;
};

static Flat flatten(sam_t *s) {
    int64_t ns, ne, nt;
    REQUIRE(sam_flat_sizes(s, &ns, &ne, &nt) == 0);
    Flat f;
    f.len.resize(ns); f.link.resize(ns); f.row_ptr.resize(ns + 1); f.edge_tok.resize(ne); f.edge_dst.resize(ne);
    f.lastpos.resize(ns); f.corpus.resize(nt); f.rec.resize(4 * ns);
    REQUIRE(sam_flatten(s, 7, 11, 13, f.len.data(), f.link.data(), f.row_ptr.data(), f.edge_tok.data(), f.edge_dst.data(),
                        f.lastpos.data(), f.corpus.data(), f.rec.data()) == 0);
    REQUIRE(f.row_ptr[0] == 11 && f.row_ptr[ns] == 11 + ne);
    int64_t slots = 0;
    REQUIRE(sam_wide_slots(s, &slots) == 0);
    if (slots >= 2) {
        std::vector<int32_t> table(4 * slots, -1);
        REQUIRE(sam_wide_table(s, 7, table.data(), slots) == 0);
    }
    return f;
}

static void automaton_and_delta(int vocab) {
    const int sep = vocab;
    std::vector<int32_t> text = make_text(6000, vocab, sep);
    sam_t *s = nullptr;
    REQUIRE(sam_build(text.data(), 1500, sep, &s) == 0);
    REQUIRE(sam_append(s, text.data() + 1500, 700) == 0);
    REQUIRE(sam_append(s, text.data() + 2200, 0) == 0);
    flatten(s);
    size_t at = 2200;
    for (int round = 0; round < 12; ++round) {
        const size_t n = 1 + rnd() % 300;
        REQUIRE(sam_append(s, text.data() + at, (int64_t)n) == 0);
        at += n;
        int64_t n_rec, n_lp, n_ov, n_ov_new, n_new, flat_states, n_written = -1;
        REQUIRE(sam_delta_sizes(s, &n_rec, &n_lp, &n_ov, &n_ov_new, &n_new, &flat_states) == 0);
        REQUIRE(n_new == (int64_t)n);
        const bool all = round % 3 == 2;                      // now and then everything since the flatten
        const int64_t n_list = all ? n_ov : n_ov_new;         // exactly-sized arrays: an overrun is caught
        std::vector<int32_t> rec_idx(n_rec), rec_val(4 * n_rec), lp_idx(n_lp), lp_val(n_lp), ov_dst(n_list), new_tok(n_new);
        std::vector<uint64_t> ov_key(n_list);
        REQUIRE(sam_delta_export(s, 7, 13, rec_idx.data(), rec_val.data(), lp_idx.data(), lp_val.data(), all ? 1 : 0,
                                 ov_key.data(), ov_dst.data(), &n_written, new_tok.data()) == 0);
        REQUIRE(n_written >= 0 && n_written <= n_list);
        int32_t due = -1;
        REQUIRE(sam_reflatten_due(s, 0.05, &due) == 0 && (due == 0 || due == 1));
        for (int64_t i = 0; i < n_new; ++i) REQUIRE(new_tok[i] == text[at - n + i]);
        if (round == 6) flatten(s);                           // a re-flatten in between starts a new log
    }
    sam_free(s);
    sam_t *e = nullptr;
    REQUIRE(sam_build(nullptr, 0, sep, &e) == 0);             // the empty memory
    flatten(e);
    sam_free(e);
}

static void builder_from_several_threads() {
    sam_builder_t *b = nullptr;
    REQUIRE(sam_builder_create(&b) == 0);
    std::atomic<int> bad{0};
    std::vector<std::vector<int32_t>> texts;                 // drawn here: the generator is not for several threads
    for (int i = 0; i < 4; ++i) texts.push_back(make_text(20000, 97, 97));
    auto client = [&](int64_t id) {
        const std::vector<int32_t> &text = texts[(size_t)id - 1];
        size_t at = 0;
        for (int piece = 0; piece < 8; ++piece) {
            const size_t n = piece == 0 ? 9000 : 1 + (size_t)(id * 131 + piece * 17) % 900;
            if (sam_builder_submit(b, id, text.data() + at, (int64_t)n, 97) != 0) ++bad;
            at += n;
            sam_t *s = nullptr; int64_t pending = -1;
            if (sam_builder_poll(b, id, &s, &pending) != 0) ++bad;          // may or may not be ready yet
            if (piece % 3 == 2) {
                if (sam_builder_wait(b, id) != 0) ++bad;
                if (sam_builder_poll(b, id, &s, &pending) != 0 || s == nullptr || pending != 0) ++bad;
                int64_t ns, ne, nt;
                if (s && (sam_flat_sizes(s, &ns, &ne, &nt) != 0 || nt != (int64_t)at)) ++bad;
            }
        }
        if (id % 2 == 0 && sam_builder_release(b, id) != 0) ++bad;          // the others are left to destroy
    };
    std::vector<std::thread> th;
    for (int64_t id = 1; id <= 4; ++id) th.emplace_back(client, id);
    for (auto &t : th) t.join();
    sam_t *s = nullptr; int64_t pending = 0;
    REQUIRE(sam_builder_poll(b, 12345, &s, &pending) != 0);   // unknown request
    sam_builder_destroy(b);
    REQUIRE(bad.load() == 0);
}

static void controllers() {
    int32_t k = -1;
    REQUIRE(spec_adaptive_k(8, 1000, 6, 64, 32768, &k) == 0 && k == 6);
    REQUIRE(spec_adaptive_k(128, 1000, 6, 64, 32768, &k) == 0 && k == 0);
    const int64_t hit[3] = {4, 0, 9}, need[3] = {10, 3, 2}, ptok[3] = {160, 48, 32};
    const double wait[3] = {0.5, 2.0, 0.1};
    double lam = 0, score[3] = {0, 0, 0};
    int64_t picked = -2;
    REQUIRE(agentsched_pick(8, hit, need, ptok, wait, 3, 4.0, 6.0, 1e-6, 1.0, 0.5, 0.2, 16, &lam, score, &picked) == 0);
    REQUIRE(picked >= -1 && picked < 3);
    REQUIRE(agentsched_pick(8, nullptr, nullptr, nullptr, nullptr, 0, 4.0, 6.0, 1e-6, 1.0, 0.5, 0.2, 16, &lam, nullptr, &picked) == 0);
}

int main() {
    automaton_and_delta(3);          // tiny vocabulary: long link chains, many clones
    automaton_and_delta(500);
    automaton_and_delta(100000);     // nearly no repeats beyond the copied spans; a very wide root
    builder_from_several_threads();
    controllers();
    std::printf("ok\n");
    return 0;
}
