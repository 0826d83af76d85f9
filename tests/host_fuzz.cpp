// Host-only fuzz of the library's CPU-side logic, meant to be built with
//   g++ -std=c++17 -O1 -g -fsanitize=address,undefined -fno-sanitize-recover=all
// (tests/test_host_sanitizers.py does that and runs it).  Two parts:
//   tables : random creates, imports, appends, segment replacements, frees and replayed device-side
//            commits on ms::HostTables, next to a naive model (an owner array searched linearly for the
//            lowest free page) and a stand-in for the device mirror that receives the queued updates
//            in both orders;
//   plan   : random batches through ms::build_plan; every 32-token tile of every sequence must lie in
//            exactly one segment, partial slots must be consistent and the plan must fit its buffers.
// Usage: host_fuzz <seed> <table_ops> <plans>.  Exit status 0 = everything held.
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include <algorithm>
#include <map>
#include <string>
#include <vector>

#include "host_tables.h"
#include "plan.h"

namespace {

struct Rng {   // splitmix64
    uint64_t s;
    explicit Rng(uint64_t seed) : s(seed) {}
    uint64_t next() {
        uint64_t z = (s += 0x9e3779b97f4a7c15ull);
        z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
        z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
        return z ^ (z >> 31);
    }
    int below(int n) { return n <= 0 ? 0 : (int)(next() % (uint64_t)n); }
    int range(int lo, int hi) { return lo + below(hi - lo + 1); }   // inclusive
};

[[noreturn]] void fail(const char* what, const std::string& detail) {
    fprintf(stderr, "host_fuzz: %s: %s\n", what, detail.c_str());
    exit(1);
}
#define REQUIRE(cond, what)                                                          \
    do {                                                                             \
        if (!(cond)) fail(what, std::string(#cond) + " (line " + std::to_string(__LINE__) + ")"); \
    } while (0)

int pages_for(long n) { return (int)((n + MS_PAGE_SIZE - 1) / MS_PAGE_SIZE); }

// ---------------------------------------------------------------------------------------------
// tables
// ---------------------------------------------------------------------------------------------
struct Model {
    std::vector<int> owner;                 // page -> sequence, -1 free
    std::vector<std::vector<int>> pt;
    std::vector<int> len;
    std::vector<char> live;
    int lowest_free() const {
        for (size_t p = 0; p < owner.size(); ++p)
            if (owner[p] < 0) return (int)p;
        return -1;
    }
    int n_free() const { return (int)std::count(owner.begin(), owner.end(), -1); }
    void add_rows(int s, int n) {
        for (int j = 0; j < n; ++j) {
            if (len[s] % MS_PAGE_SIZE == 0) {
                const int p = lowest_free();
                owner[p] = s;
                pt[s].push_back(p);
            }
            len[s]++;
        }
    }
    void cut(int s, int rows) {
        const int keep = pages_for(rows);
        while ((int)pt[s].size() > keep) {
            owner[pt[s].back()] = -1;
            pt[s].pop_back();
        }
        len[s] = rows;
    }
};

struct Mirror {   // what the device holds: page tables and lengths
    int max_pages;
    std::vector<int> pt, len;
    void apply(const std::vector<int>& triples, bool reversed) {
        const size_t n = triples.size() / 3;
        for (size_t k = 0; k < n; ++k) {
            const size_t i = 3 * (reversed ? n - 1 - k : k);
            const int s = triples[i], idx = triples[i + 1], v = triples[i + 2];
            if (idx < 0) len[s] = v; else pt[(size_t)s * max_pages + idx] = v;
        }
    }
};

void compare(const ms::HostTables& t, const Model& m, const char* after) {
    const std::string fault = t.check_tables();
    if (!fault.empty()) fail(after, fault);
    REQUIRE((int)t.free_pages.size() == m.n_free(), after);
    for (int s = 0; s < t.max_seqs; ++s) {
        REQUIRE((bool)t.live[s] == (bool)m.live[s], after);
        REQUIRE(t.len[s] == m.len[s], after);
        REQUIRE(t.pt[s] == m.pt[s], after);
    }
    for (int p : t.free_pages) REQUIRE(m.owner[p] < 0, after);
}

void flush(ms::HostTables& t, Mirror& mir, const char* after) {
    // the device applies a batch of queued entries in no particular order: both extremes must agree
    Mirror fwd = mir, rev = mir;
    fwd.apply(t.pending_pt, false);
    rev.apply(t.pending_pt, true);
    REQUIRE(fwd.pt == rev.pt && fwd.len == rev.len, after);
    mir = fwd;
    t.pending_pt.clear();
    for (int s = 0; s < t.max_seqs; ++s) {
        if (!t.live[s]) continue;
        REQUIRE(mir.len[s] == t.len[s], after);
        for (size_t i = 0; i < t.pt[s].size(); ++i) REQUIRE(mir.pt[(size_t)s * mir.max_pages + i] == t.pt[s][i], after);
    }
}

void fuzz_tables(Rng& rng, int ops) {
    const int n_pages = rng.range(8, 160), max_seqs = rng.range(1, 12), max_pp = rng.range(2, 40);
    ms::HostTables t;
    t.init_tables(n_pages, max_seqs, max_pp);
    Model m;
    m.owner.assign(n_pages, -1);
    m.pt.assign(max_seqs, {});
    m.len.assign(max_seqs, 0);
    m.live.assign(max_seqs, 0);
    Mirror mir;
    mir.max_pages = max_pp;
    mir.pt.assign((size_t)max_seqs * max_pp, -1);
    mir.len.assign(max_seqs, -1);
    int peak = 0;
    auto live_ids = [&] {
        std::vector<int> v;
        for (int s = 0; s < max_seqs; ++s)
            if (m.live[s]) v.push_back(s);
        return v;
    };
    for (int op = 0; op < ops; ++op) {
        const int kind = rng.below(100);
        const std::vector<int> ids = live_ids();
        const unsigned version_before = t.version;
        bool changed = false, queued_pages = false;   // calls that queue page entries send them before they return
        if (kind < 12) {   // create
            int want = -1;
            for (int s = 0; s < max_seqs && want < 0; ++s)
                if (!m.live[s]) want = s;
            const int got = t.create_seq();
            REQUIRE(got == want, "create");
            if (got >= 0) {
                m.live[got] = 1;
                m.len[got] = 0;
                changed = true;
            }
        } else if (kind < 20 && !ids.empty()) {   // free
            const int s = ids[rng.below((int)ids.size())];
            t.free_seq(s);
            m.cut(s, 0);
            m.live[s] = 0;
            changed = true;
        } else if (kind < 30) {   // import
            std::vector<int> free_now(t.free_pages.begin(), t.free_pages.end());
            for (size_t i = free_now.size(); i > 1; --i) std::swap(free_now[i - 1], free_now[rng.below((int)i)]);
            const int n = rng.below(std::min<int>((int)free_now.size(), max_pp) + 1);
            free_now.resize(n);
            const int length = n == 0 ? 0 : (n - 1) * MS_PAGE_SIZE + rng.range(1, MS_PAGE_SIZE);
            REQUIRE(t.pages_importable(free_now.data(), n), "import");
            if (n >= 1) {   // the refusals: a page listed twice, a page in use, a page out of range
                std::vector<int> bad = free_now;
                bad.push_back(free_now[0]);
                REQUIRE(!t.pages_importable(bad.data(), (int)bad.size()), "import refuses duplicates");
                bad.back() = n_pages + rng.below(3);
                REQUIRE(!t.pages_importable(bad.data(), (int)bad.size()), "import refuses out-of-range pages");
                bad.back() = -1;
                REQUIRE(!t.pages_importable(bad.data(), (int)bad.size()), "import refuses negative pages");
                for (int p = 0; p < n_pages; ++p)
                    if (m.owner[p] >= 0) {
                        bad.back() = p;
                        REQUIRE(!t.pages_importable(bad.data(), (int)bad.size()), "import refuses pages in use");
                        break;
                    }
            }
            const int s = t.create_seq();
            if (s >= 0) {
                t.import_seq(s, free_now.data(), n, length);
                m.live[s] = 1;
                m.len[s] = length;
                m.pt[s] = free_now;
                for (int p : free_now) m.owner[p] = s;
                changed = queued_pages = true;
            }
        } else if (kind < 60 && !ids.empty()) {   // append to a few sequences (a sequence may be listed twice)
            const int B = rng.range(1, 4);
            std::vector<int> who(B), cnt(B), extra(max_seqs, 0);
            for (int b = 0; b < B; ++b) {
                who[b] = ids[rng.below((int)ids.size())];
                cnt[b] = rng.below(3) == 0 ? 0 : rng.range(1, 45);
                extra[who[b]] += cnt[b];
            }
            long want = 0;
            for (int s = 0; s < max_seqs && want >= 0; ++s)
                if (extra[s]) {
                    const int np = pages_for((long)m.len[s] + extra[s]);
                    if (np > max_pp) want = -1 - s; else want += np - (int)m.pt[s].size();
                }
            const long need = t.pages_needed(extra);
            REQUIRE(need == want, "append: pages needed");
            if (need >= 0 && need <= (long)t.free_pages.size()) {
                for (int b = 0; b < B; ++b) {
                    t.grow(who[b], cnt[b]);
                    m.add_rows(who[b], cnt[b]);
                    changed = changed || cnt[b] > 0;
                }
                queued_pages = true;
            }
        } else if (kind < 80 && !ids.empty()) {   // a segment replaced by memory rows, the rows after it kept
            const int s = ids[rng.below((int)ids.size())];
            const int L = m.len[s];
            const int begin = rng.range(0, L), seg = rng.range(0, L - begin), n_mem = rng.range(0, 12);
            const int tail = L - begin - seg, new_len = L - seg + n_mem;
            const int keep = pages_for(begin), np = pages_for(new_len);
            const long free_after = (long)t.free_pages.size() + (long)t.pt[s].size() - keep - (np - keep);
            if (np <= max_pp && free_after >= 0) {
                t.cut_to(s, begin);
                t.grow(s, n_mem);
                t.grow(s, tail);
                t.note_len(s);
                m.cut(s, begin);
                m.add_rows(s, n_mem + tail);
                changed = queued_pages = true;
            }
        } else if (!ids.empty()) {   // device-side commits replayed: a few steps, then the host catches up
            flush(t, mir, "before device commits");
            std::vector<int> free_list(t.free_pages.begin(), t.free_pages.end());
            std::vector<int> who, dev_len = t.len;
            int cursor = 0;
            const int steps = rng.range(1, 5), n_max = rng.range(1, MS_PAGE_SIZE);
            for (int st = 0; st < steps; ++st) {
                std::vector<int> batch = ids;
                for (size_t i = batch.size(); i > 1; --i) std::swap(batch[i - 1], batch[rng.below((int)i)]);
                batch.resize(rng.range(1, (int)batch.size()));
                // the host's admission test: room for one page per listed sequence, page count within bounds
                bool fits = cursor + (int)batch.size() <= (int)free_list.size();
                for (int s : batch) fits = fits && pages_for((long)dev_len[s] + n_max) <= max_pp;
                if (!fits) break;
                for (int s : batch) {   // the kernel: sequences in argument order, the next listed page when a row opens one
                    const int acc = rng.range(0, n_max), old_pages = pages_for(dev_len[s]);
                    dev_len[s] += acc;
                    if (pages_for(dev_len[s]) > old_pages) {
                        REQUIRE(pages_for(dev_len[s]) == old_pages + 1, "device commit takes at most one page");
                        mir.pt[(size_t)s * max_pp + old_pages] = free_list[cursor];
                        who.push_back(s);
                        ++cursor;
                    }
                    mir.len[s] = dev_len[s];
                    m.add_rows(s, acc);
                }
            }
            REQUIRE(t.apply_device_commits(who.data(), cursor, free_list, dev_len.data()), "device commits");
            changed = true;   // (the version is bumped even when nothing was taken)
            // corrupt logs are refused: a count beyond the list, a dead sequence
            ms::HostTables copy = t;
            REQUIRE(!copy.apply_device_commits(who.data(), (int)free_list.size() + 1, free_list, dev_len.data()), "corrupt log");
            if (!free_list.empty() && cursor < (int)free_list.size()) {
                int dead = -1;
                for (int s = 0; s < max_seqs && dead < 0; ++s)
                    if (!m.live[s]) dead = s;
                if (dead >= 0) {
                    copy = t;
                    std::vector<int> fl(free_list.begin() + cursor, free_list.end());
                    REQUIRE(!copy.apply_device_commits(&dead, 1, fl, dev_len.data()), "corrupt log");
                }
            }
        }
        if (changed) REQUIRE(t.version != version_before, "version bump");
        compare(t, m, "after an operation");
        peak = std::max(peak, n_pages - m.n_free());
        REQUIRE(t.peak_pages >= peak, "peak pages");
        if (queued_pages || rng.below(4) == 0) flush(t, mir, "mirror");
    }
    flush(t, mir, "mirror at the end");
}

// ---------------------------------------------------------------------------------------------
// plan
// ---------------------------------------------------------------------------------------------
void fuzz_plan(Rng& rng) {
    using ms::Seg;
    const int B = rng.below(8) == 0 ? rng.range(65, MS_MAX_BATCH) : rng.range(1, 64);
    const int max_seqs = B + rng.below(5);
    const int style = rng.below(5);
    std::vector<int> ids(max_seqs);
    for (int i = 0; i < max_seqs; ++i) ids[i] = i;
    for (size_t i = ids.size(); i > 1; --i) std::swap(ids[i - 1], ids[rng.below((int)i)]);
    ids.resize(B);
    std::vector<int> lens(B);
    std::vector<std::vector<int>> pt(max_seqs);
    int next_page = 0;
    for (int b = 0; b < B; ++b) {
        int L;
        switch (style) {
            case 0: L = rng.below(200); break;                          // tiny, many empty or single-tile
            case 1: L = 8192 + rng.below(64); break;                    // the metric point and a little more
            case 2: L = rng.range(1000, 16384); break;                  // the ragged mix
            case 3: L = rng.below(4) ? rng.below(40) : rng.range(20000, 140000); break;   // one giant among dwarfs
            default: L = 32 * rng.below(300) + (rng.below(2) ? 0 : rng.below(32)); break; // tile boundaries
        }
        if (rng.below(10) == 0) L = 0;
        if (B > 64 && L > 3000) L = L % 3000;
        lens[b] = L;
        pt[ids[b]].resize(pages_for(L));
        for (int& p : pt[ids[b]]) p = next_page++;
        for (size_t i = pt[ids[b]].size(); i > 1; --i) std::swap(pt[ids[b]][i - 1], pt[ids[b]][rng.below((int)i)]);
    }
    const int target = rng.below(4) == 0 ? rng.range(1, ms::kMaxMfmaItems) : 64;
    const long min_tiles = rng.below(3) == 0 ? 24L * rng.range(1, 8) : 16;
    std::vector<int> blob;
    int n_items = 0, n_segs = 0;
    ms::build_plan(pt, ids.data(), lens.data(), B, target, min_tiles, blob, &n_items, &n_segs);

    REQUIRE(n_items >= 1 && n_items <= target, "plan: number of shares");
    REQUIRE(n_segs <= n_items + B, "plan: one partial per share plus one per sequence bounds the segments");
    REQUIRE((long)blob.size() == (long)(n_items + n_segs) * ms::kSegInts + B + 1, "plan: blob size");
    REQUIRE((int)blob.size() <= ms::mfma_plan_ints(B), "plan: fits the device buffer");
    REQUIRE(blob.size() * sizeof(int) <= 256 * 1024, "plan: fits one staging slot");
    const Seg* firsts = reinterpret_cast<const Seg*>(blob.data());
    const Seg* segs = reinterpret_cast<const Seg*>(blob.data() + (size_t)n_items * ms::kSegInts);
    const int* part_begin = blob.data() + (size_t)(n_items + n_segs) * ms::kSegInts;

    // the shares' segment ranges tile the list in order
    int at = 0;
    long max_cost = 0, total_tiles = 0;
    for (int it = 0; it < n_items; ++it) {
        REQUIRE(firsts[it].seg_begin == at && firsts[it].seg_end >= at && firsts[it].seg_end <= n_segs, "plan: share ranges");
        long cost = 0;
        for (int k = firsts[it].seg_begin; k < firsts[it].seg_end; ++k)   // (segments of empty sequences are dealt out round robin)
            if (segs[k].t1 > segs[k].t0) cost += ms::kSegOverheadTiles + (segs[k].t1 - segs[k].t0 + ms::kTile - 1) / ms::kTile;
        max_cost = std::max(max_cost, cost);
        if (firsts[it].seg_end > at) {   // the share's first record repeats its first segment
            const Seg& f = firsts[it];
            const Seg& s = segs[at];
            REQUIRE(f.b == s.b && f.seq == s.seq && f.t0 == s.t0 && f.t1 == s.t1 && f.part == s.part && f.len == s.len, "plan: first record");
            REQUIRE(std::equal(f.pages, f.pages + 2 * ms::kWaves, s.pages), "plan: first record's pages");
        }
        at = firsts[it].seg_end;
    }
    REQUIRE(at == n_segs, "plan: share ranges cover every segment");

    // every tile of every sequence in exactly one segment; segments of a sequence in rising order
    REQUIRE(part_begin[0] == 0 && part_begin[B] == n_segs, "plan: partial ranges");
    std::vector<int> next_token(B, 0), seen_parts(B, 0);
    std::vector<char> closed(B, 0);
    for (int k = 0; k < n_segs; ++k) {
        const Seg& s = segs[k];
        REQUIRE(s.b >= 0 && s.b < B && s.seq == ids[s.b] && s.len == lens[s.b], "plan: segment's sequence");
        REQUIRE(s.t0 % ms::kTile == 0 && s.t0 <= s.t1 && s.t1 <= s.len, "plan: segment bounds");
        REQUIRE(!closed[s.b], "plan: a segment after the sequence's last");
        if (s.len > 0) {
            REQUIRE(s.t0 == next_token[s.b] && s.t1 > s.t0, "plan: segments leave no gap and no overlap");
            REQUIRE(s.t1 == s.len || s.t1 % ms::kTile == 0, "plan: only the last segment ends inside a tile");
        } else {
            REQUIRE(s.t0 == 0 && s.t1 == 0, "plan: the empty sequence's one segment");
        }
        next_token[s.b] = s.t1;
        if (s.t1 == s.len) closed[s.b] = 1;
        REQUIRE(s.part == part_begin[s.b] + seen_parts[s.b], "plan: partial slots count up within the sequence");
        seen_parts[s.b]++;
        total_tiles += (s.t1 - s.t0 + ms::kTile - 1) / ms::kTile;
        // page ids of every wave's first tile, clamped to the sequence's last page
        const int n_tiles = (s.t1 - s.t0 + ms::kTile - 1) / ms::kTile, last_page = (s.len - 1) >> 4;
        for (int w = 0; w < ms::kWaves; ++w) {
            if (n_tiles == 0) {
                REQUIRE(s.pages[2 * w] == 0 && s.pages[2 * w + 1] == 0, "plan: pages of an empty segment");
                continue;
            }
            const int tc = std::min(w, n_tiles - 1), pg0 = (s.t0 >> 4) + 2 * tc;
            REQUIRE(s.pages[2 * w] == pt[s.seq][std::min(pg0, last_page)], "plan: first page of a wave's first tile");
            REQUIRE(s.pages[2 * w + 1] == pt[s.seq][std::min(pg0 + 1, last_page)], "plan: second page of a wave's first tile");
        }
    }
    long want_tiles = 0;
    for (int b = 0; b < B; ++b) {
        REQUIRE(closed[b] && seen_parts[b] >= 1, "plan: every sequence has a segment that reaches its end");
        REQUIRE(part_begin[b + 1] - part_begin[b] == seen_parts[b], "plan: partial range of a sequence");
        want_tiles += (lens[b] + ms::kTile - 1) / ms::kTile;
    }
    REQUIRE(total_tiles == want_tiles, "plan: tile count");
    // balance: no share costs more than an even split plus one segment's overhead per sequence boundary it may hold
    if (want_tiles > 0) {
        const long even = (want_tiles + (long)ms::kSegOverheadTiles * (n_items + B) + n_items - 1) / n_items;
        REQUIRE(max_cost <= even + ms::kSegOverheadTiles + 1, "plan: balance");
    }
}

}  // namespace

int main(int argc, char** argv) {
    const uint64_t seed = argc > 1 ? strtoull(argv[1], nullptr, 10) : 1;
    const int table_ops = argc > 2 ? atoi(argv[2]) : 20000, plans = argc > 3 ? atoi(argv[3]) : 2000;
    Rng rng(seed);
    int done = 0;
    while (done < table_ops) {
        const int n = std::min(table_ops - done, 400);
        fuzz_tables(rng, n);
        done += n;
    }
    for (int i = 0; i < plans; ++i) fuzz_plan(rng);
    printf("host_fuzz: seed %llu: %d table operations and %d plans held\n", (unsigned long long)seed, table_ops, plans);
    return 0;
}
