// Schedule of the matrix-core decode kernel: an equal split of the batch's key tiles over wavefronts, and the
// hand-over of the partial results of a sequence that was cut (round-sparse decode, paper Sec. 3.2 step 5).
//
// The key tiles (32 tokens, never crossing a round) of all sequences of the batch form one list per KV head:
// sequence 0's tiles, then sequence 1's, ...; tile_begin[b] is the index of sequence b's first tile and
// tile_begin[B] = total.  The list is cut into n_ranges ranges of equal size (to within one tile; see RangeCut for
// the one exception): with total = n_ranges * q + rem, the first rem ranges have q + 1 tiles and the others q,
//     range r = [ r * q + min(r, rem) , (r + 1) * q + min(r + 1, rem) ),
// and one wavefront streams one range for one (KV head, block of 16 query rows).  A range may end inside a
// sequence and may cover the tails and heads of several: the part of sequence b inside range r is a SEGMENT, and
// a sequence that lies in more than one range has one partial result ("record") per segment.  Along the list
// both r and b only grow, so  record(r, b) = r + b  is unique over all segments, and the records of one
// sequence are consecutive: record_first(b) .. + n_parts(b) - 1.
//
// Hand-over without waiting: a wave stores the record of its segment and is done; a second, small kernel, launched
// behind the first on the same stream, reads the n_parts records of every sequence that was cut and writes its
// output.  No wave ever waits for another, so every wave exits whatever the order of execution.
//
// Everything here is plain 32-bit integer arithmetic usable on host and device (the GPU has no fast 64-bit
// divide); the host model in tests/host_model/ runs the same functions with one thread per wave.
#pragma once

#ifndef RA_HD
#ifdef __HIPCC__
#define RA_HD __host__ __device__
#else
#define RA_HD
#endif
#endif

namespace ra {

// Number of ranges for a batch of `total` tiles: never more than `max_ranges` (the wavefronts of the launch
// divided by the work items per range) and no range shorter than `min_units` tiles.
RA_HD inline unsigned range_count(unsigned total, int min_units, int max_ranges) {
    unsigned n = total / (unsigned)(min_units > 0 ? min_units : 1);
    if (n > (unsigned)max_ranges) n = (unsigned)max_ranges;
    return n < 1 ? 1 : n;
}

// The cut of a batch, prepared once.  total < 2^30.
//
// With skew = 0 all ranges are equal to within one tile.  With skew > 0 (in 1/1000) and a launch that fills the
// chip (as many ranges as it may have, an even number, and long ones) the first half of the ranges, which the
// workgroups dispatched first stream, get (1 + skew/1000) / 2 of the tiles and the second half the rest: the
// hardware serves the waves that came first on a compute unit a little faster for the whole kernel, and ranges
// in proportion let both halves end together.  Inside each half the ranges are again equal to within one tile:
// the first rem_x ranges of a half have q_x + 1 tiles, the others q_x.
struct RangeCut {
    unsigned total, n_ranges;
    unsigned n_a, total_a, q_a, rem_a;  // first class: ranges 0 .. n_a - 1 cover tiles [0, total_a)
    unsigned q_b, rem_b;                // second class: ranges n_a .. n_ranges - 1 cover the rest
};
constexpr unsigned kSkewMinTiles = 16;  // ranges shorter than this are not skewed: their start dominates
RA_HD inline RangeCut range_cut(unsigned total, int min_units, int max_ranges, int skew = 0) {
    RangeCut c;
    c.total = total;
    c.n_ranges = range_count(total, min_units, max_ranges);
    c.n_a = c.n_ranges;
    c.total_a = total;
    if (skew > 0 && c.n_ranges == (unsigned)max_ranges && c.n_ranges >= 2 && (c.n_ranges & 1) == 0 &&
        total / c.n_ranges >= kSkewMinTiles) {
        const unsigned w = 1000u + (unsigned)(skew > 500 ? 500 : skew);
        c.n_a = c.n_ranges / 2;
        c.total_a = total / 2000u * w + total % 2000u * w / 2000u;  // total * w / 2000 without leaving 32 bits
    }
    const unsigned n_b = c.n_ranges - c.n_a, total_b = total - c.total_a;
    c.q_a = c.total_a / c.n_a;
    c.rem_a = c.total_a - c.q_a * c.n_a;
    c.q_b = n_b ? total_b / n_b : 1;
    c.rem_b = n_b ? total_b - c.q_b * n_b : 0;
    return c;
}
RA_HD inline unsigned range_begin(const RangeCut& c, unsigned r) {
    if (r <= c.n_a) return r * c.q_a + (r < c.rem_a ? r : c.rem_a);
    const unsigned k = r - c.n_a;
    return c.total_a + k * c.q_b + (k < c.rem_b ? k : c.rem_b);
}

// The range that holds tile t, 0 <= t < total.
RA_HD inline unsigned range_of_tile(const RangeCut& c, unsigned t) {
    if (t < c.total_a) {
        const unsigned big = c.rem_a * (c.q_a + 1);  // tiles in the ranges of q_a + 1
        return t < big ? t / (c.q_a + 1) : c.rem_a + (t - big) / c.q_a;
    }
    const unsigned u = t - c.total_a, big = c.rem_b * (c.q_b + 1);
    return c.n_a + (u < big ? u / (c.q_b + 1) : c.rem_b + (u - big) / c.q_b);
}

// Records of a sequence with tiles [t_lo, t_hi), t_hi > t_lo.
struct SeqParts {
    int first_range, n_parts;
};
RA_HD inline SeqParts seq_parts(const RangeCut& c, unsigned t_lo, unsigned t_hi) {
    SeqParts p;
    p.first_range = (int)range_of_tile(c, t_lo);
    p.n_parts = (int)range_of_tile(c, t_hi - 1) - p.first_range + 1;
    return p;
}
RA_HD inline int record_index(int r, int b) { return r + b; }
// Upper bound of record_index + 1 for a launch.
RA_HD inline int record_capacity(int max_ranges, int B) { return max_ranges + B; }

// Largest b in [0, n) with begin[b] <= t, for begin[0] <= t < begin[n] (begin non-decreasing).
template <typename T>
RA_HD inline int upper_slot(const T* begin, int n, long long t) {
    int lo = 0, hi = n;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if ((long long)begin[mid] <= t) lo = mid; else hi = mid;
    }
    return lo;
}

}  // namespace ra
