// Geometry shared by the backward kernels: the compacted list of "far" keys (initial tokens and
// separators, the only keys a query can see beyond its neighbour window, Sec. 3.1) and the split of
// the far pass of dK/dV among persistent workgroups.
#pragma once

#include "common.h"

namespace sepattn {

constexpr int kDkvWaves = 4;              // key blocks of 32 keys per dK/dV workgroup (two waves each)
constexpr int kDkvThreads = 2 * 64 * kDkvWaves;
constexpr int kBK = 32 * kDkvWaves;  // keys per dK/dV workgroup
constexpr int kBQ = 64;              // queries per LDS tile in the dK/dV kernels

__host__ __device__ inline int align_down32(int x) { return x & ~31; }

// The far work of one (batch, KV head): for list tile ft (128 consecutive list entries) the
// "items" (query tile of 64 rows, query head) from the first query that can see the tile's first key
// to the end of the sequence.  The items of all list tiles, in this order, are cut into `wpg` slices
// of equal length, one per workgroup; the part of a slice that lies in one list tile is a "piece" and
// produces one fp32 partial of that tile's dK / dV rows.  Piece (w, ft) uses partial slot w + ft
// (along the pieces either w or ft grows, so the slot numbers are distinct).
struct FarGeom {
    int wpg;     // workgroups per (batch, KV head)
    int NFcap;   // capacity of the far list, a multiple of kBK
    int NFTcap;  // list tiles at full capacity
    int NP;      // partial slots per (batch, KV head)
    long rows;   // fp32 partial rows per (batch, KV head): NP slots of kBK rows, then one band row per list entry
};
inline int dkv_workgroups_per_head(const sepattn_params &p) {
    const long n_bkv = (long)p.B * p.Hkv;
    const long w = compute_units() / n_bkv;
    return (int)(w < 1 ? 1 : w);
}
__host__ __device__ inline FarGeom far_geom(const sepattn_params &p, int wpg) {
    FarGeom g;
    g.wpg = wpg;
    g.NFcap = (p.a + p.cap + kBK - 1) / kBK * kBK;
    g.NFTcap = g.NFcap / kBK;
    g.NP = wpg + g.NFTcap;
    g.rows = (long)g.NP * kBK + g.NFcap;
    return g;
}

// backward workspace: D_i [B,Hq,L] fp32 | LSE_i * log2(e) [B,Hq,L] fp32 | dK partials | dV partials |
// first and last workgroup of every list tile [B,Hkv,NFTcap,2] int32
struct BwdWorkspace {
    size_t d_bytes, far_bytes, tab_bytes, total;
};
inline BwdWorkspace bwd_workspace(const sepattn_params &p) {
    FarGeom fg = far_geom(p, dkv_workgroups_per_head(p));
    BwdWorkspace w;
    w.d_bytes = align_up((size_t)p.B * p.Hq * p.L * sizeof(float), 256);
    w.far_bytes = align_up((size_t)p.B * p.Hkv * fg.rows * p.d * sizeof(float), 256);
    w.tab_bytes = align_up((size_t)p.B * p.Hkv * fg.NFTcap * 2 * sizeof(int32_t), 256);
    w.total = 2 * w.d_bytes + 2 * w.far_bytes + w.tab_bytes;
    return w;
}

struct FarList {
    int a_eff, sep_base, NF;
};
__device__ inline FarList far_list(const sepattn_params &p, const int32_t *__restrict__ prefix) {
    FarList f;
    f.a_eff = p.a;  // already clamped to L by the host
    f.sep_base = prefix[f.a_eff];
    int cnt = min(prefix[p.L], p.cap);
    f.NF = f.a_eff + max(cnt - f.sep_base, 0);
    return f;
}
__device__ inline int far_pos(const FarList &fl, int f, const int32_t *__restrict__ idx, int L) {
    if (f < fl.a_eff) return f;
    return min(max(idx[fl.sep_base + f - fl.a_eff], 0), L - 1);
}
// index of key position j on the far list, -1 if it is neither an initial token nor a listed separator
__device__ inline int far_index(const FarList &fl, const int32_t *__restrict__ prefix, int j) {
    int f = -1;
    if (j < fl.a_eff)
        f = j;
    else if (prefix[j + 1] != prefix[j])
        f = fl.a_eff + prefix[j] - fl.sep_base;
    return f < fl.NF ? f : -1;
}
// first query row the far pieces of list entry f's tile cover (>= L: the entry has no far piece)
__device__ inline int far_first_query(const FarList &fl, int f, const int32_t *__restrict__ idx,
                                      const sepattn_params &p) {
    return align_down32(far_pos(fl, (f / kBK) * kBK, idx, p.L) + p.n);
}

// one past the last query row the far pieces of list entry f's tile cover: the end of the sequence,
// or, with packed documents (dend: one past the last position of each position's document, else
// nullptr), the end of the document of the tile's last entry.  A tile whose first query row
// (far_first_query) is not below this has no far piece.
__device__ inline int far_last_query(const FarList &fl, int f, const int32_t *__restrict__ idx,
                                     const sepattn_params &p, const int32_t *__restrict__ dend) {
    if (!dend) return p.L;
    const int last = min((f / kBK + 1) * kBK, fl.NF) - 1;
    return min(max(dend[far_pos(fl, last, idx, p.L)], 0), p.L);
}

// doc_end: packed documents ([B, L], p.a == 0), or nullptr
int launch_dkv_bf16(const sepattn_params &p, const HeadWin &hw, const uint16_t *Q, const uint16_t *K, const uint16_t *V,
                    const float *lse2, const uint16_t *dO, const float *Dws, const int32_t *sep_idx,
                    const int32_t *sep_prefix, const int32_t *doc_end, uint16_t *dK, uint16_t *dV, float *farK,
                    float *farV, int32_t *piece_tab, hipStream_t st);

}  // namespace sepattn
