// The dense key stream of one query tile (used by the forward and the dQ kernels).
//
// For query positions [i0, i0+TP) the visible keys are enumerated as one stream
//     [ initial tokens j < min(a, bs) | separators in [min(a,bs), bs) | band keys bs .. i0+TP-1 ]
// with bs = max(0, i0-n+1), the first key of the first row's neighbour window (Sec. 3.1).  Elements
// of the first two parts are visible to every row of the tile; a band key j is visible to query i
// iff  j <= i  and  (i-j < n  or  j is an initial token or a separator)  (Eq. 2).  Each stream
// element carries the inclusive query range [lo, hi] that sees it, so the test is lo <= i <= hi.
#pragma once

#include "common.h"
#include "mfma_common.h"

namespace sepattn {

constexpr int kBN = 64;  // keys per LDS tile

// XCD-aware decomposition of a 1-D grid of n_tiles * n_groups workgroups into (tile rank, group),
// where a group is one (batch, KV head, packed query-head group) and owns its own K/V rows.
// Consecutive workgroup ids are dealt round-robin to the 8 XCDs, each with a private L2.  When the
// number of groups is a multiple of 8, XCD x only ever sees groups congruent to x, so the K/V rows
// of a group stay in one L2 instead of being streamed through all eight.
struct TileGroup {
    int rank, group;
};
__device__ inline TileGroup xcd_tile_group(int id, int n_tiles, int n_groups) {
    TileGroup r;
    if (n_groups % 8 == 0) {
        r.group = (id % 8) + 8 * (id / (8 * n_tiles));
        r.rank = (id / 8) % n_tiles;
    } else {
        r.group = id % n_groups;
        r.rank = id / n_groups;
    }
    return r;
}

struct Stream {
    int n_init, n_dense, n_total, sep_lo, bs;
};

__device__ inline Stream make_stream(const sepattn_params &p, const int32_t *__restrict__ prefix, int i0,
                                     int tile_positions) {
    Stream st;
    st.bs = max(0, i0 - p.n + 1);
    st.n_init = min(p.a, st.bs);
    st.sep_lo = prefix[st.n_init];
    st.n_dense = st.n_init + (prefix[st.bs] - st.sep_lo);
    st.n_total = st.n_dense + (min(p.L, i0 + tile_positions) - st.bs);
    return st;
}

// Packed documents: the row holds several documents and a query sees nothing outside its own.  The
// first tokens of every document are marked like separators beforehand (the kernels then run with
// a = 0), so the keys of the first row's document that are older than its window are still one
// contiguous range of the compacted list, now starting at that document's first position `ds`; the
// band starts no earlier than `ds`.  Rows of later documents in the same tile find all their keys in
// the band part; who sees what is decided by the per-key range [lo, hi] with hi cut at the end of
// the key's document.
__device__ inline Stream make_stream_docs(const sepattn_params &p, const int32_t *__restrict__ prefix, int i0,
                                          int tile_positions, int ds) {
    Stream st;
    st.bs = max(ds, i0 - p.n + 1);
    st.n_init = 0;
    st.sep_lo = prefix[ds];
    st.n_dense = prefix[st.bs] - st.sep_lo;
    st.n_total = st.n_dense + (min(p.L, i0 + tile_positions) - st.bs);
    return st;
}
// key position of stream element k, and the query range [lo, hi] that sees it
__device__ inline int stream_key(const Stream &s, int k, const sepattn_params &p,
                                 const int32_t *__restrict__ idx, const int32_t *__restrict__ prefix,
                                 int &lo, int &hi) {
    if (k >= s.n_total) {  // padding of the last tile: never visible, any valid row to load
        lo = kIntMax;
        hi = -1;
        return 0;
    }
    int j;
    if (k < s.n_init) {
        j = k;
        hi = kIntMax;
    } else if (k < s.n_dense) {
        // the clamps keep a stale list tail (caller broke sep_count <= cap) from faulting
        j = min(max(idx[min(s.sep_lo + k - s.n_init, p.cap - 1)], 0), p.L - 1);
        hi = kIntMax;
    } else {
        j = s.bs + (k - s.n_dense);
        bool always = (j < p.a) || (prefix[j + 1] != prefix[j]);
        hi = always ? kIntMax : j + p.n - 1;
    }
    lo = j;
    return j;
}

// how a wave treats a block of 32 stream elements starting at k0, given its rows [pw, pw+31]:
// 0 = skip (nothing visible), 1 = everything visible, 2 = test each pair
__device__ inline int block_mode(const Stream &st, int k0, int pw, int n) {
    int pmax = pw + 31;
    if (k0 + 32 <= st.n_dense) return 1;
    if (k0 >= st.n_dense) {
        int jmin = st.bs + (k0 - st.n_dense), jmax = jmin + 31;
        if (k0 >= st.n_total || jmin > pmax) return 0;
        if (k0 + 32 <= st.n_total && jmax <= pw && jmin + n - 1 >= pmax) return 1;
        return 2;
    }
    return 2;
}

// The same decision for "every pair of the block is visible" (mode 1), reduced to three comparisons
// against thresholds that are computed once per wave: a block of 32 stream elements starting at k0
// needs no mask test iff it lies in the dense part (k0 <= dense_last) or is a band block whose keys
// are inside every row's window and not in any row's future (band_first <= k0 <= band_last).
struct FullBlocks {
    int dense_last, band_first, band_last;
};
__device__ inline FullBlocks full_blocks(const Stream &st, int pw, int n) {
    FullBlocks f;
    const int pmax = pw + 31;
    f.dense_last = st.n_dense - 32;
    f.band_first = max(st.n_dense, st.n_dense + (pmax - n + 1) - st.bs);  // jmin + n - 1 >= pmax
    f.band_last = min(st.n_dense + (pw - 31) - st.bs, st.n_total - 32);   // jmax <= pw, no padding
    return f;
}
// no block of the tile is free of the mask test (a wave whose rows reach into the next document)
__device__ inline FullBlocks no_full_blocks() {
    FullBlocks f;
    f.dense_last = -(1 << 30);
    f.band_first = 1 << 30;
    f.band_last = -1;
    return f;
}
__device__ inline bool block_is_full(const FullBlocks &f, int k0) {
    return (k0 <= f.dense_last) | ((k0 >= f.band_first) & (k0 <= f.band_last));
}

}  // namespace sepattn
