// Host model of the control flow of the matrix-core decode kernel (paper Sec. 3.2 step 5: attention over the
// selected rounds; here only who streams which key tiles and which partial results exist afterwards): one OS
// thread per wavefront, the same schedule functions as the kernel (range_schedule.hpp), std::atomic in place of the
// GPU's memory where threads meet.
//
// Two launches in a row per random batch (work item = wave, wave + n_waves, ...).  Checked:
//   * every wave terminates: no wave reads anything another wave writes (there is no loop on shared state);
//   * the segments handed out cover every key tile of every (KV head, row block) exactly once;
//   * record indices stay below record_capacity() and no record is written twice;
//   * a sequence that lies in one range is written directly, exactly once, and leaves no record;
//   * for a sequence cut into n parts the merge step (a second kernel, after all waves have exited) finds exactly
//     the n records first .. first + n - 1 that the streaming kernel announced, and they add up to the sequence.
//
// Built with -DPLANT_RECORD_BY_RANGE or -DPLANT_SKIP_LAST_ITEM the model carries a planted mistake and must fail:
// that is how the test shows that the checks can fail at all.
//
// usage: decode_schedule [seed] [cases]     exit status 0 = every check passed
#include <atomic>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <thread>
#include <vector>

#include "range_schedule.hpp"

using namespace ra;

struct Launch {
    int B, inner, max_ranges, min_units, n_waves, skew;
    std::vector<int> U;      // tiles per sequence
    std::vector<int> begin;  // prefix, begin[B] = total
    std::vector<int> rec_val;  // [records][inner] tiles the record stands for (plain memory)
    std::vector<std::atomic<int>> rec_writes, out_writes, tiles_seen;  // [records][inner], [B][inner], [inner]
    std::atomic<int> errors{0};
    Launch(int records, int B_, int inner_)
        : rec_val(records * inner_, -1), rec_writes(records * inner_), out_writes(B_ * inner_), tiles_seen(inner_) {}
};

static void fail(Launch& L, const char* what, int a, int b) {
    if (L.errors.fetch_add(1) < 5) std::fprintf(stderr, "  model check failed: %s (%d, %d)\n", what, a, b);
}

// What one wavefront does after the kernel's prologue.
static void wave(Launch& L, int w, unsigned jitter) {
    const unsigned total = (unsigned)L.begin[L.B];
    if (total == 0) return;
    const RangeCut cut = range_cut(total, L.min_units, L.max_ranges, L.skew);
    int n_items = (int)cut.n_ranges * L.inner;
#ifdef PLANT_SKIP_LAST_ITEM
    n_items -= 1;  // planted mistake: the last work item is never handed out
#endif
    std::minstd_rand rng(jitter);
    for (int item = w; item < n_items; item += L.n_waves) {
        const int range = item / L.inner, gi = item - range * L.inner;
        int t_lo = (int)range_begin(cut, range);
        const int t_hi = (int)range_begin(cut, range + 1);
        int b = upper_slot(L.begin.data(), L.B, t_lo);
        for (; t_lo < t_hi; ++b) {
            if (b >= L.B) { fail(L, "walked past the last sequence", range, b); return; }
            const int seq_lo = L.begin[b], seq_hi = L.begin[b + 1];
            const int seg_hi = t_hi < seq_hi ? t_hi : seq_hi;
            if (seg_hi <= t_lo) continue;
            const int tiles = seg_hi - t_lo;
            t_lo = seg_hi;
            L.tiles_seen[gi].fetch_add(tiles, std::memory_order_relaxed);
            if (rng() & 1) std::this_thread::yield();
            const SeqParts parts = seq_parts(cut, seq_lo, seq_hi);
            if (range < parts.first_range || range >= parts.first_range + parts.n_parts) fail(L, "range outside the sequence's parts", range, b);
            if (parts.n_parts == 1) {
                if (tiles != L.U[b]) fail(L, "uncut sequence streamed in part", b, tiles);
                L.out_writes[b * L.inner + gi].fetch_add(1, std::memory_order_relaxed);
                continue;
            }
#ifdef PLANT_RECORD_BY_RANGE
            const int rec = range;  // planted mistake: two sequences of one range would share a record
#else
            const int rec = record_index(range, b);
#endif
            if (rec < 0 || rec >= record_capacity(L.max_ranges, L.B)) { fail(L, "record index out of bounds", rec, b); return; }
            if (L.rec_writes[rec * L.inner + gi].fetch_add(1, std::memory_order_relaxed) != 0) fail(L, "record written twice", rec, gi);
            L.rec_val[rec * L.inner + gi] = tiles;  // the partial result
        }
    }
}

// The merge kernel, after the streaming kernel has ended: one work item per (sequence, KV head, row block).
static void merge_step(Launch& L) {
    const unsigned total = (unsigned)L.begin[L.B];
    if (total == 0) return;
    const RangeCut cut = range_cut(total, L.min_units, L.max_ranges, L.skew);
    for (int b = 0; b < L.B; ++b) {
        if (L.U[b] == 0) continue;
        const SeqParts parts = seq_parts(cut, L.begin[b], L.begin[b + 1]);  // what block 0 of the kernel announces
        if (parts.n_parts <= 1) continue;
        const int rec0 = record_index(parts.first_range, b);
        for (int gi = 0; gi < L.inner; ++gi) {
            int sum = 0;
            for (int p = 0; p < parts.n_parts; ++p) {
                if (L.rec_writes[(rec0 + p) * L.inner + gi].load() != 1) fail(L, "a record of a cut sequence is missing", b, p);
                sum += L.rec_val[(rec0 + p) * L.inner + gi];
            }
            if (sum != L.U[b]) fail(L, "the records of a sequence do not add up to it", b, sum);
            L.out_writes[b * L.inner + gi].fetch_add(1, std::memory_order_relaxed);
        }
    }
}

int main(int argc, char** argv) {
    const unsigned seed = argc > 1 ? (unsigned)std::atoi(argv[1]) : 1u;
    const int cases = argc > 2 ? std::atoi(argv[2]) : 200;
    std::mt19937 rng(seed);
    int bad = 0;
    for (int c = 0; c < cases; ++c) {
        // mostly small batches; every tenth case a batch beyond one wavefront's lanes, up to the library's limit
        const int B = c % 10 == 9 ? 65 + (int)(rng() % 960) : 1 + (int)(rng() % 24);
        const int inner = 1 + (int)(rng() % 4), n_waves = 1 + (int)(rng() % 48);
        const int min_units = 1 + (int)(rng() % 4);
        int max_ranges = n_waves * (1 + (int)(rng() % 3)) / inner;  // also more ranges than waves: several items per wave
        if (max_ranges < 1) max_ranges = 1;
        const int style = (int)(rng() % 5);
        const int skew = c % 3 == 0 ? 0 : 1 + (int)(rng() % 200);  // two thirds of the cases with unequal halves
        for (int launch = 0; launch < 2; ++launch) {
            Launch L(record_capacity(max_ranges, B), B, inner);
            L.B = B; L.inner = inner; L.max_ranges = max_ranges; L.min_units = min_units; L.n_waves = n_waves; L.skew = skew;
            L.U.resize(B);
            for (int b = 0; b < B; ++b) {
                int u = (int)(rng() % 40);
                if (style == 1) u = (rng() % 3) ? 0 : (int)(rng() % 300);  // many empty sequences
                if (style == 2) u = b == 0 ? 2000 : (int)(rng() % 3);      // one long, many tiny
                if (style == 3) u = 1;                                      // one tile each
                if (style == 4) u = 200 + (int)(rng() % 800);               // long ranges: the skew is in force
                L.U[b] = u;
            }
            L.begin.assign(B + 1, 0);
            for (int b = 0; b < B; ++b) L.begin[b + 1] = L.begin[b] + L.U[b];
            std::vector<std::thread> th;
            for (int w = 0; w < n_waves; ++w) th.emplace_back(wave, std::ref(L), w, (unsigned)rng());
            for (auto& t : th) t.join();
            merge_step(L);
            for (int gi = 0; gi < inner; ++gi)
                if (L.tiles_seen[gi].load() != L.begin[B]) fail(L, "tiles not covered exactly once", gi, L.tiles_seen[gi].load());
            for (int b = 0; b < B; ++b)
                for (int gi = 0; gi < inner; ++gi)
                    if (L.out_writes[b * inner + gi].load() != (L.U[b] > 0 ? 1 : 0)) fail(L, "output written a wrong number of times", b, gi);
            bad += L.errors.load();
        }
    }
    // range arithmetic on its own: the ranges tile [0, total); without skew they differ by at most one tile; with
    // skew each half does, the first half is the longer one and holds its share of the tiles; none is shorter than
    // min_units (unless there is only one); range_of_tile inverts range_begin
    for (int c = 0; c < 4000; ++c) {
        const bool big = c % 2 == 1;
        const unsigned total = 1 + (unsigned)(rng() % (big ? 4000000 : 100000));
        const int min_units = 1 + (int)(rng() % 8), max_ranges = 1 + (int)(rng() % 300);
        const int skew = c % 4 < 2 ? 0 : 1 + (int)(rng() % 200);
        const RangeCut cut = range_cut(total, min_units, max_ranges, skew);
        if (range_begin(cut, 0) != 0 || range_begin(cut, cut.n_ranges) != total || (int)cut.n_ranges > max_ranges) { ++bad; continue; }
        unsigned lo[2] = {total, total}, hi[2] = {0, 0};
        for (unsigned r = 0; r < cut.n_ranges; ++r) {
            const unsigned len = range_begin(cut, r + 1) - range_begin(cut, r);
            const int k = r < cut.n_a ? 0 : 1;
            lo[k] = len < lo[k] ? len : lo[k];
            hi[k] = len > hi[k] ? len : hi[k];
        }
        const bool skewed = cut.n_a != cut.n_ranges;
        if (hi[0] - lo[0] > 1 || (skewed && hi[1] - lo[1] > 1)) ++bad;
        if (skew == 0 && skewed) ++bad;
        if (skewed) {
            if (cut.n_a * 2 != cut.n_ranges || lo[0] < lo[1] || hi[0] < hi[1] || lo[1] < kSkewMinTiles / 2) ++bad;
            const double share = (double)cut.total_a / total, want = (1000.0 + skew) / 2000.0;
            if (share > want + 1e-9 || share < want - 2.0 / total - 1e-9) ++bad;
        }
        const unsigned shortest = skewed && lo[1] < lo[0] ? lo[1] : lo[0];
        if (cut.n_ranges > 1 && (int)shortest < min_units) ++bad;
        for (int k = 0; k < 20; ++k) {
            const unsigned t = (unsigned)(rng() % total);
            const unsigned r = range_of_tile(cut, t);
            if (!(r < cut.n_ranges && range_begin(cut, r) <= t && t < range_begin(cut, r + 1))) ++bad;
        }
    }
    std::printf("%s: %d cases x 2 launches, seed %u, %d failed checks\n", bad ? "FAILED" : "ok", cases, seed, bad);
    return bad ? 1 : 0;
}
