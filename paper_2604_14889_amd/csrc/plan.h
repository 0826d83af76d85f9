// Work plan of the streaming attention kernel: which workgroup walks which tokens of which sequence
// (MemoSight paper, Section 2.3: one pass over each sequence's cached rows per step; the pass of a
// batch is divided into equal shares so that every compute unit streams the same number of bytes).
// Plain C++ without any GPU call: the library builds it into the launch path, and the same code
// builds for the CPU alone with the address and undefined-behaviour sanitizers.
#pragma once

#include <string.h>

#include <vector>

namespace ms {

constexpr int kTile = 32;            // tokens per MFMA tile
constexpr int kWaves = 8;            // waves per workgroup (2 per SIMD: at most 256 registers each)
constexpr int kMaxMfmaItems = 256;   // stream-kernel workgroups per KV head

struct Seg {
    int b;          // index in the call's batch
    int seq;        // sequence id
    int t0;         // first token (multiple of 32); 0 marks the sequence's first segment
    int t1;         // one past the last token
    int part;       // partial slot (per KV head)
    int len;        // sequence length
    int seg_begin;  // in an item's first record: the item's segment range in the full list
    int seg_end;
    int pages[2 * kWaves];  // page ids of the first tile of every wave (clamped like tile_pages)
};

constexpr int kSegInts = (int)(sizeof(Seg) / sizeof(int));
constexpr int kSegOverheadTiles = 16;   // set-up + merge of a segment, in units of one tile of streaming (12 to 20 measured alike, 8 and 24 slower)

// plan blob: [first segment of every item][all segments][partial range of every sequence]
inline int mfma_plan_ints(int B) { return kMaxMfmaItems * kSegInts + (kMaxMfmaItems + B) * kSegInts + (B + 1); }

// Splits the batch's 32-token tiles into equal contiguous shares (work items) and lists each share's
// segments.  Every sequence gets at least one segment (an empty one if it has no cached tokens): the
// first segment's workgroup also runs the sequence's in-flight tile.
inline void build_plan(const std::vector<std::vector<int>>& page_tables, const int* seq_ids, const int* lens, int B, int n_items_target,
                       long min_tiles, std::vector<int>& blob, int* n_items_out, int* n_parts_out) {
    std::vector<long> tile_prefix(B + 1, 0);
    for (int b = 0; b < B; ++b) tile_prefix[b + 1] = tile_prefix[b] + (lens[b] + kTile - 1) / kTile;
    const long nt = tile_prefix[B];
    int n_items = n_items_target;
    if ((long)n_items * min_tiles > nt) n_items = (int)(nt / min_tiles);
    if (n_items < 1) n_items = 1;
    std::vector<std::vector<Seg>> per_item(n_items);
    std::vector<int> part_count(B, 0);
    auto make_seg = [&](int b, int t0, int t1) {
        Seg s;
        s.b = b;
        s.seq = seq_ids[b];
        s.t0 = t0;
        s.t1 = t1;
        s.part = part_count[b]++;   // rebased below
        s.len = lens[b];
        s.seg_begin = s.seg_end = 0;
        const std::vector<int>& pt = page_tables[seq_ids[b]];
        const int n_tiles = (t1 - t0 + kTile - 1) / kTile, last_page = (lens[b] - 1) >> 4;
        for (int w = 0; w < kWaves; ++w) {
            if (n_tiles == 0) {
                s.pages[2 * w] = s.pages[2 * w + 1] = 0;
                continue;
            }
            const int tc = w < n_tiles ? w : n_tiles - 1;
            const int pg0 = (t0 >> 4) + 2 * tc;
            s.pages[2 * w] = pt[pg0 < last_page ? pg0 : last_page];
            s.pages[2 * w + 1] = pt[pg0 + 1 < last_page ? pg0 + 1 : last_page];
        }
        return s;
    };
    // Shares are cut so that the largest cost, tiles + kSegOverheadTiles per segment, is as small
    // as n_items shares allow (every segment costs a set-up and a merge phase worth about that many
    // tiles of streaming): greedy packing under a cost cap, the cap found by bisection.
    auto pack = [&](long cap, bool emit) {
        int it = 0;
        long cost = 0;
        for (int b = 0; b < B; ++b) {
            long left = tile_prefix[b + 1] - tile_prefix[b], at = 0;
            while (left > 0) {
                if (cost + kSegOverheadTiles + 1 > cap) {
                    ++it;
                    cost = 0;
                }
                long take = cap - cost - kSegOverheadTiles;
                if (take > left) take = left;
                if (emit) {
                    int t1 = (int)(at + take) * kTile;
                    if (t1 > lens[b]) t1 = lens[b];
                    per_item[it].push_back(make_seg(b, (int)at * kTile, t1));
                }
                cost += kSegOverheadTiles + take;
                left -= take;
                at += take;
            }
        }
        return it + 1;
    };
    if (nt > 0) {
        long lo = kSegOverheadTiles + 1, hi = nt + (long)kSegOverheadTiles * (B + 1);
        while (lo < hi) {
            const long mid = (lo + hi) / 2;
            if (pack(mid, false) <= n_items) hi = mid; else lo = mid + 1;
        }
        pack(lo, true);
    }
    for (int e = 0; e < B; ++e)
        if (lens[e] == 0) per_item[e % n_items].push_back(make_seg(e, 0, 0));
    std::vector<int> part_begin(B + 1, 0);
    for (int i = 0; i < B; ++i) part_begin[i + 1] = part_begin[i] + part_count[i];
    std::vector<Seg> firsts(n_items), segs;
    for (int it = 0; it < n_items; ++it) {
        const int begin = (int)segs.size();
        for (Seg s : per_item[it]) {
            s.part += part_begin[s.b];
            segs.push_back(s);
        }
        firsts[it] = per_item[it].empty() ? Seg{} : segs[begin];
        firsts[it].seg_begin = begin;
        firsts[it].seg_end = (int)segs.size();
    }
    // compact blob: [first segment of every item][all segments][partial range of every sequence]
    blob.assign((size_t)(n_items + segs.size()) * kSegInts + part_begin.size(), 0);
    memcpy(blob.data(), firsts.data(), firsts.size() * sizeof(Seg));
    memcpy(blob.data() + (size_t)n_items * kSegInts, segs.data(), segs.size() * sizeof(Seg));
    memcpy(blob.data() + (size_t)(n_items + segs.size()) * kSegInts, part_begin.data(), part_begin.size() * sizeof(int));
    *n_items_out = n_items;
    *n_parts_out = (int)segs.size();
}

}  // namespace ms
