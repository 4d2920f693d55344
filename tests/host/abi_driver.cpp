// Host-only exercise of the C ABI for the sanitizer build (AddressSanitizer + UndefinedBehaviorSanitizer
// on the host side of the library): argument validation, size queries, handle creation and destruction
// with NG_INIT_HOST_ONLY (no device is touched, nothing launches), counters, layout, error strings.
// Exits 0 when every check holds; a sanitizer report aborts the process with a non-zero status.
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "ng.h"
#include "ng_internal.h"   // ng::xcd_order, ng::TileRef (internal, host side)

static int g_failed = 0;
#define CHECK(cond)                                                         \
    do {                                                                    \
        if (!(cond)) {                                                      \
            fprintf(stderr, "CHECK failed at line %d: %s\n", __LINE__, #cond); \
            ++g_failed;                                                     \
        }                                                                   \
    } while (0)

struct Set {
    std::vector<ng_matrix_desc> descs;
    std::vector<ng_matrix_buffers> bufs;
    std::vector<void*> owned;
    void* ws = nullptr;
    size_t ws_bytes = 0;
    ng_state* st = nullptr;
    ~Set() {
        ng_destroy(st);
        for (void* p : owned) free(p);
    }
};

static void* aligned(Set& s, size_t bytes) {
    void* p = nullptr;
    if (posix_memalign(&p, 256, bytes < 256 ? 256 : bytes) != 0) abort();
    memset(p, 0, bytes < 256 ? 256 : bytes);
    s.owned.push_back(p);
    return p;
}

static int make(Set& s, const ng_hparams& hp, uint32_t flags) {
    const int n = (int)s.descs.size();
    std::vector<size_t> bytes((size_t)n * NG_NBUF);
    int rc = ng_query_sizes(s.descs.data(), n, &hp, bytes.data(), &s.ws_bytes);
    if (rc != NG_OK) return rc;
    s.bufs.resize(n);
    for (int i = 0; i < n; ++i)
        for (int b = 0; b < NG_NBUF; ++b) s.bufs[i].buf[b] = aligned(s, bytes[(size_t)i * NG_NBUF + b]);
    s.ws = aligned(s, s.ws_bytes);
    return ng_init_state(s.descs.data(), s.bufs.data(), n, &hp, s.ws, s.ws_bytes, flags, nullptr, &s.st);
}

// The tile-table order: every tile exactly once, eight runs (entry k of run x at 8 k + x) of about equal
// cost, longest tiles first inside a run and otherwise in the logical order, padding entries with mat < 0.
static void check_tile_order() {
    std::vector<ng::TileRef> out;
    ng::xcd_order({}, {}, &out);
    CHECK(out.empty());
    ng::xcd_order({ng::TileRef{7, 1, 2, 0}}, {5}, &out);
    CHECK(out.size() == 8);
    int seen = 0;
    for (const ng::TileRef& t : out) seen += t.mat == 7 && t.ti == 1 && t.tj == 2 ? 1 : (t.mat < 0 ? 0 : 100);
    CHECK(seen == 1);
    // 24 blocks of a 1.1B-shaped layer set: 4 x 16 + 2 x 44 tiles of length 2048, then 16 of length 5461
    std::vector<ng::TileRef> logical;
    std::vector<int> cost;
    for (int b = 0; b < 24; ++b)
        for (int k = 0; k < 7; ++k) {
            const int tiles = k < 4 ? 16 : k < 6 ? 44 : 16;
            for (int t = 0; t < tiles; ++t) {
                logical.push_back(ng::TileRef{b * 7 + k, t & 1, t >> 1, 0});
                cost.push_back(k == 6 ? 5461 : 2048);
            }
        }
    ng::xcd_order(logical, cost, &out);
    CHECK(out.size() % 8 == 0 && out.size() >= logical.size());
    std::vector<int> hits(logical.size(), 0);
    long long run_cost[8] = {0}, total = 0;
    for (int c : cost) total += c;
    for (size_t x = 0; x < 8; ++x) {
        int prev_cost = 1 << 30, prev_idx = -1;
        bool padding_seen = false;
        for (size_t k = 0; 8 * k + x < out.size(); ++k) {
            const ng::TileRef& t = out[8 * k + x];
            if (t.mat < 0) { padding_seen = true; continue; }
            CHECK(!padding_seen);   // padding only at the end of a run
            // find the tile in the logical order (mat, ti, tj are unique there)
            int idx = -1;
            for (size_t i = 0; i < logical.size(); ++i)
                if (logical[i].mat == t.mat && logical[i].ti == t.ti && logical[i].tj == t.tj) { idx = (int)i; break; }
            CHECK(idx >= 0);
            if (idx < 0) continue;
            ++hits[idx];
            run_cost[x] += cost[idx];
            CHECK(cost[idx] <= prev_cost);                                  // longest first
            if (cost[idx] == prev_cost) CHECK(idx > prev_idx);              // stable inside a cost class
            prev_cost = cost[idx];
            prev_idx = idx;
        }
    }
    for (int h : hits) CHECK(h == 1);
    for (size_t x = 0; x < 8; ++x) CHECK(run_cost[x] * 8 >= total - 8LL * 5461 && run_cost[x] * 8 <= total + 8LL * 5461);
}

int main() {
    check_tile_order();
    ng_hparams hp;
    CHECK(ng_default_hparams(&hp) == NG_OK);
    CHECK(ng_default_hparams(nullptr) == NG_ERR_INVALID_ARG);
    for (int which = 0; which < 6; ++which) (void)ng_struct_size(which);
    for (int code = 1; code >= -12; --code) CHECK(ng_strerror(code) != nullptr && strlen(ng_strerror(code)) > 0);

    // every layer-set kind the planner distinguishes: bf16 MFMA path with ragged shapes and both sides,
    // fp32 MFMA path, fp32 small-rank path, s = 0, the largest history, bf16 history slots, carry-over
    struct Case { int dtype, hist, s, carry; std::vector<ng_matrix_desc> d; };
    std::vector<Case> cases;
    cases.push_back({NG_BF16, NG_F32, 16, 0, {{2048, 5461, 512, NG_SIDE_LEFT, 5461, 5461}, {5461, 2048, 512, NG_SIDE_RIGHT, 2048, 2050},
                                              {33, 7, 5, NG_SIDE_LEFT, 9, 7}, {1, 12, 1, NG_SIDE_LEFT, 12, 12}}});
    cases.push_back({NG_BF16, NG_BF16, 0, 0, {{200, 333, 24, NG_SIDE_LEFT, 333, 340}}});
    cases.push_back({NG_F32, NG_F32, 64, 1, {{64, 96, 8, NG_SIDE_LEFT, 96, 96}, {96, 64, 3, NG_SIDE_LEFT, 70, 64}}});
    cases.push_back({NG_F32, NG_F32, 4, 1, {{700, 900, 600, NG_SIDE_LEFT, 900, 900}, {130, 64, 20, NG_SIDE_RIGHT, 64, 64}}});
    std::vector<ng_matrix_desc> many;
    for (int i = 0; i < 300; ++i) many.push_back({64 + i % 5, 96 + i % 7, 16, i % 3 == 0 ? NG_SIDE_RIGHT : NG_SIDE_LEFT, 128, 128});
    cases.push_back({NG_BF16, NG_F32, 2, 0, many});
    for (const Case& c : cases) {
        Set s;
        s.descs = c.d;
        ng_hparams h = hp;
        h.grad_dtype = c.dtype;
        h.hist_dtype = c.hist;
        h.s = c.s;
        h.carry_history = c.carry;
        const int rc = make(s, h, NG_INIT_HOST_ONLY);
        CHECK(rc == NG_OK);
        if (rc != NG_OK) continue;
        const int n = (int)s.descs.size();
        for (int i = 0; i < n; ++i) {
            ng_matrix_layout lay;
            CHECK(ng_get_layout(s.st, i, &lay) == NG_OK);
            // one panel: the plain row-major slot; else 2048-column panels with the last one padded
            const int64_t stored_cols = (lay.ldn + lay.panel_cols - 1) / lay.panel_cols * (int64_t)lay.panel_cols;
            CHECK(lay.ldn % 32 == 0 && (lay.panel_cols == lay.ldn || lay.panel_cols == 2048));
            CHECK(lay.slot_elems == (int64_t)s.descs[i].r * stored_cols);
            int64_t t = -1, nref = -1;
            int32_t head = -1, count = -1;
            CHECK(ng_get_counters(s.st, i, &t, &head, &count, &nref) == NG_OK && t == 0 && head == 0 && count == 0 && nref == 0);
            CHECK(ng_set_counters(s.st, i, 7, c.s > 0 ? c.s - 1 : 0, c.s, 3) == NG_OK);
            CHECK(ng_set_counters(s.st, i, 7, c.s > 0 ? c.s : 1, 0, 0) == NG_ERR_INVALID_ARG);
            CHECK(ng_set_counters(s.st, i, 7, 0, c.s + 1, 0) == NG_ERR_INVALID_ARG);
        }
        CHECK(ng_get_layout(s.st, n, nullptr) == NG_ERR_INVALID_ARG);
        CHECK(ng_get_counters(s.st, -1, nullptr, nullptr, nullptr, nullptr) == NG_ERR_INVALID_ARG);
        // nothing may launch on a host-only handle
        std::vector<const void*> g(n, s.ws);
        std::vector<void*> w(n, s.ws);
        CHECK(ng_step(s.st, g.data(), w.data(), 1e-3f, nullptr) == NG_ERR_NO_PROJECTOR);
        CHECK(ng_refresh_projector(s.st, g.data(), nullptr) == NG_ERR_HIP);
        CHECK(ng_commit_projector(s.st, 1, nullptr) == NG_ERR_HIP);
        const int rc_commit = ng_commit_projector(s.st, 0, nullptr);
        CHECK(rc_commit == (c.dtype == NG_BF16 ? NG_ERR_HIP : NG_OK));
        if (rc_commit == NG_OK) {
            CHECK(ng_step(s.st, g.data(), w.data(), 1e-3f, nullptr) == NG_ERR_HIP);
            CHECK(ng_step_static(s.st, g.data(), w.data(), 1e-3f, nullptr) == NG_ERR_HIP ||
                  ng_step_static(s.st, g.data(), w.data(), 1e-3f, nullptr) == NG_ERR_WORKSPACE);
        }
        g[n - 1] = nullptr;
        CHECK(ng_step(s.st, g.data(), w.data(), 1e-3f, nullptr) == NG_ERR_INVALID_ARG);
        CHECK(ng_get_status(s.st, nullptr) == NG_ERR_HIP);
        double ms[NG_NPHASE];
        int64_t steps = -1;
        CHECK(ng_get_phase_ms(s.st, ms, &steps, 1) == NG_OK && steps == 0);
        int64_t t = 0;
        CHECK(ng_get_counters(s.st, 0, &t, nullptr, nullptr, nullptr) == NG_OK && t == 7);   // failed calls left it alone
    }

    // validation failures and bad workspaces must neither leak nor touch freed memory
    {
        Set s;
        s.descs = {{256, 512, 300, NG_SIDE_LEFT, 512, 512}};
        CHECK(make(s, hp, NG_INIT_HOST_ONLY) == NG_ERR_SHAPE);
        s.descs = {{256, 512, 32, NG_SIDE_LEFT, 512, 512}};
        ng_hparams h = hp;
        h.lambda = 0.f;
        CHECK(make(s, h, NG_INIT_HOST_ONLY) == NG_ERR_HPARAM);
        h = hp;
        h.proj_dtype = NG_BF16;   // the bf16-only projector needs bf16 gradients
        CHECK(make(s, h, NG_INIT_HOST_ONLY) == NG_ERR_HPARAM);
        CHECK(make(s, hp, NG_INIT_HOST_ONLY) == NG_OK);
        ng_state* st2 = nullptr;
        CHECK(ng_init_state(s.descs.data(), s.bufs.data(), 1, &hp, s.ws, s.ws_bytes - 1, NG_INIT_HOST_ONLY, nullptr, &st2) == NG_ERR_WORKSPACE);
        CHECK(ng_init_state(s.descs.data(), s.bufs.data(), 1, &hp, (char*)s.ws + 8, s.ws_bytes, NG_INIT_HOST_ONLY, nullptr, &st2) == NG_ERR_WORKSPACE);
        ng_matrix_buffers bad = s.bufs[0];
        bad.buf[NG_BUF_V] = nullptr;
        CHECK(ng_init_state(s.descs.data(), &bad, 1, &hp, s.ws, s.ws_bytes, NG_INIT_HOST_ONLY, nullptr, &st2) == NG_ERR_INVALID_ARG);
        CHECK(st2 == nullptr);
    }
    ng_destroy(nullptr);
    if (g_failed) {
        fprintf(stderr, "%d checks failed\n", g_failed);
        return 1;
    }
    printf("abi_driver: all checks passed\n");
    return 0;
}
