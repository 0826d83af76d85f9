// Host side of the paged cache: which page belongs to which sequence, the free pages, the sequences'
// lengths and the list of changes the device copies still have to receive (MemoSight paper,
// Section 2.1.2: the cache is a list of rows that grows by appends and shrinks when a segment is
// replaced by its memory tokens; Algorithm 1, UpdateCache).  Plain C++ without any GPU call, so that
// the same code also builds for the CPU with the address and undefined-behaviour sanitizers.
//
// Allocation rule: a sequence that needs a page takes the lowest-numbered free page; sequences are
// served in the order of the call's arguments.  The device-side commit reproduces exactly this order
// from an ascending list of free pages, and apply_device_commits() replays its log here.
#pragma once

#include <set>
#include <string>
#include <vector>

#include "memosight.h"

namespace ms {

struct HostTables {
    int n_pages = 0, max_seqs = 0, max_pages_per_seq = 0;
    std::set<int> free_pages;    // ordered: *begin() is the lowest free page
    std::vector<std::vector<int>> pt;
    std::vector<int> len;
    std::vector<char> live;
    int peak_pages = 0;
    // (seq, index, page) triples not yet sent to the device mirror; index -1: the entry is the
    // sequence's length.  The device applies a batch of entries in no particular order, so a batch
    // never holds two entries for one slot: length entries are updated in place, and a call that
    // queues page entries sends the batch before it returns (creates and frees queue lengths only).
    std::vector<int> pending_pt;
    unsigned version = 0;        // bumped by every change of lengths or page tables

    static int pages_for(long n) { return (int)((n + MS_PAGE_SIZE - 1) / MS_PAGE_SIZE); }

    void init_tables(int n_pages_, int max_seqs_, int max_pages_per_seq_) {
        n_pages = n_pages_;
        max_seqs = max_seqs_;
        max_pages_per_seq = max_pages_per_seq_;
        free_pages.clear();
        for (int p = 0; p < n_pages; ++p) free_pages.insert(free_pages.end(), p);
        pt.assign(max_seqs, {});
        len.assign(max_seqs, 0);
        live.assign(max_seqs, 0);
        peak_pages = 0;
        pending_pt.clear();
    }

    void note_peak() {
        const int in_use = n_pages - (int)free_pages.size();
        if (in_use > peak_pages) peak_pages = in_use;
    }

    // The lowest free page becomes the sequence's next page.  The caller has verified capacity.
    int take_page(int seq) {
        version++;
        const int page = *free_pages.begin();
        free_pages.erase(free_pages.begin());
        pending_pt.push_back(seq);
        pending_pt.push_back((int)pt[seq].size());
        pending_pt.push_back(page);
        pt[seq].push_back(page);
        note_peak();
        return page;
    }

    // Queues the sequence's current length for the device copy of the lengths.
    void note_len(int seq) {
        for (size_t i = 0; i + 2 < pending_pt.size(); i += 3)
            if (pending_pt[i] == seq && pending_pt[i + 1] == -1) {
                pending_pt[i + 2] = len[seq];
                return;
            }
        pending_pt.push_back(seq);
        pending_pt.push_back(-1);
        pending_pt.push_back(len[seq]);
    }

    // Grows `seq` by n rows; the caller has verified capacity.
    void grow(int seq, int n) {
        version++;
        for (int j = 0; j < n; ++j) {
            if (len[seq] % MS_PAGE_SIZE == 0) take_page(seq);
            len[seq]++;
        }
        if (n > 0) note_len(seq);
    }

    // Lowest unused sequence id, or -1.
    int create_seq() {
        for (int s = 0; s < max_seqs; ++s)
            if (!live[s]) {
                version++;
                live[s] = 1;
                len[s] = 0;
                pt[s].clear();
                note_len(s);
                return s;
            }
        return -1;
    }

    // Every page in range, free and listed once?
    bool pages_importable(const int* pages, int n) const {
        std::set<int> seen;
        for (int i = 0; i < n; ++i)
            if (pages[i] < 0 || pages[i] >= n_pages || !free_pages.count(pages[i]) || !seen.insert(pages[i]).second) return false;
        return true;
    }

    // Gives the (new, empty) sequence s the listed pages and the length; pages_importable() held.
    void import_seq(int s, const int* pages, int n, int length) {
        for (int i = 0; i < n; ++i) {
            free_pages.erase(pages[i]);
            pending_pt.push_back(s);
            pending_pt.push_back(i);
            pending_pt.push_back(pages[i]);
            pt[s].push_back(pages[i]);
        }
        len[s] = length;
        note_len(s);
        version++;
        note_peak();
    }

    void free_seq(int s) {
        version++;
        for (int p : pt[s]) free_pages.insert(p);
        pt[s].clear();
        len[s] = 0;
        note_len(s);
        live[s] = 0;
    }

    // Keeps the first `rows` rows: pages past them go back to the free set.
    void cut_to(int s, int rows) {
        version++;
        const int keep = pages_for(rows);
        for (size_t i = keep; i < pt[s].size(); ++i) free_pages.insert(pt[s][i]);
        pt[s].resize(keep);
        len[s] = rows;
    }

    // Pages an append of extra[s] rows per sequence would take from the free set; -1 - s if
    // sequence s would pass max_pages_per_seq.
    long pages_needed(const std::vector<int>& extra) const {
        long need = 0;
        for (int s = 0; s < max_seqs; ++s) {
            if (!extra[s]) continue;
            const int np = pages_for((long)len[s] + extra[s]);
            if (np > max_pages_per_seq) return -1 - s;
            need += np - (int)pt[s].size();
        }
        return need;
    }

    // Replays a device-side commit log: the k-th page of free_list went to sequence who[k]
    // (k < used); lens are the device's lengths.  False (nothing half-applied matters: the caller
    // reports corruption) if the log names a dead sequence or a page that is not free.
    bool apply_device_commits(const int* who, int used, const std::vector<int>& free_list, const int* lens) {
        if (used < 0 || used > (int)free_list.size()) return false;
        for (int k = 0; k < used; ++k) {
            const int seq = who[k], page = free_list[k];
            if (seq < 0 || seq >= max_seqs || !live[seq] || !free_pages.count(page)) return false;
            free_pages.erase(page);
            pt[seq].push_back(page);
        }
        for (int s = 0; s < max_seqs; ++s)
            if (live[s]) len[s] = lens[s];
        note_peak();
        version++;
        return true;
    }

    // Every page owned exactly once or free, page counts matching lengths; empty string if sound.
    std::string check_tables() const {
        std::vector<char> owner(n_pages, 0);
        for (int s = 0; s < max_seqs; ++s) {
            if (!live[s]) {
                if (!pt[s].empty()) return "dead sequence " + std::to_string(s) + " owns pages";
                continue;
            }
            if ((int)pt[s].size() != pages_for(len[s]))
                return "sequence " + std::to_string(s) + " has " + std::to_string(pt[s].size()) + " pages for " + std::to_string(len[s]) + " rows";
            for (int p : pt[s]) {
                if (p < 0 || p >= n_pages) return "page id " + std::to_string(p) + " out of range";
                if (owner[p]++) return "page " + std::to_string(p) + " owned twice";
            }
        }
        for (int p : free_pages) {
            if (p < 0 || p >= n_pages) return "free page id " + std::to_string(p) + " out of range";
            if (owner[p]++) return "page " + std::to_string(p) + " both free and owned";
        }
        for (int p = 0; p < n_pages; ++p)
            if (!owner[p]) return "page " + std::to_string(p) + " leaked";
        return "";
    }
};

}  // namespace ms
