// Schedule of the matrix-core decode kernel: an equal split of the batch's key tiles over wavefronts, and the
// hand-over of the partial results of a sequence that was cut (round-sparse decode, paper Sec. 3.2 step 5).
//
// The key tiles (32 tokens, never crossing a round) of all sequences of the batch form one list per KV head:
// sequence 0's tiles, then sequence 1's, ...; tile_begin[b] is the index of sequence b's first tile and
// tile_begin[B] = total.  The list is cut into n_ranges ranges of equal size (to within one tile): with
// total = n_ranges * q + rem, the first rem ranges have q + 1 tiles and the others q,
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
struct RangeCut {
    unsigned total, n_ranges, q, rem;
};
RA_HD inline RangeCut range_cut(unsigned total, int min_units, int max_ranges) {
    RangeCut c;
    c.total = total;
    c.n_ranges = range_count(total, min_units, max_ranges);
    c.q = total / c.n_ranges;
    c.rem = total - c.q * c.n_ranges;
    return c;
}
RA_HD inline unsigned range_begin(const RangeCut& c, unsigned r) { return r * c.q + (r < c.rem ? r : c.rem); }

// The range that holds tile t, 0 <= t < total.
RA_HD inline unsigned range_of_tile(const RangeCut& c, unsigned t) {
    const unsigned big = c.rem * (c.q + 1);  // tiles in the ranges of q + 1
    return t < big ? t / (c.q + 1) : c.rem + (t - big) / c.q;
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
