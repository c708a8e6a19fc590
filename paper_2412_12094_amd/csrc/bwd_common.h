// Geometry shared by the backward kernels: the compacted list of "far" keys (initial tokens and
// separators, the only keys a query can see beyond its neighbour window, Sec. 3.1) and the split of
// the far pass of dK/dV among persistent workgroups.
#pragma once

#include "common.h"

namespace sepattn {

// A dK/dV workgroup holds KW key blocks of 32 keys, two waves each (32 KW keys, 128 KW threads), in one
// of two shapes:
//   KW = 4: 8 waves, one workgroup per compute unit.  Fewest tile loads per matrix instruction; the
//           better shape when a workgroup's pieces are long: d = 128, sequences from 8K on with
//           grouped heads (by 3-5 % there; at L = 4096, or with one head per KV head at 8K, the other
//           shape is 1-13 % ahead, at 16K with one head per KV head the two are level).
//   KW = 2: 4 waves, two workgroups per compute unit (three at d = 64, where the registers and the ring
//           of query tiles allow it) that run independently: one's piece start-up and partial stores
//           overlap the others' matrix work, the split of a (batch, KV head) is finer (it fills the
//           chip where 256 / (B Hkv) is not a whole number), and the workgroups' barriers do not lock
//           each other's phases.
// With packed documents the far pieces end with their documents, so the pieces are short at any
// length.  The launcher chooses (docs: the call has document bounds) and hands KW to both kernels;
// the workspace is laid out for the larger of the two shapes' needs, so its size does not depend
// on the choice.
inline int dkv_key_blocks(const sepattn_params &p, bool docs) {
    const long G = p.Hq / p.Hkv;
    return (p.d == 128 && !docs && p.L >= 8192 && G * p.L >= 32768) ? 4 : 2;
}
// workgroups of a shape that share a compute unit
inline int dkv_workgroups_per_cu(const sepattn_params &p, int kw) { return kw == 4 ? 1 : (p.d == 64 ? 3 : 2); }

__host__ __device__ inline int align_down32(int x) { return x & ~31; }

// The far work of one (batch, KV head): for list tile ft (bk = 32 KW consecutive list entries) the
// "items" (query tile, query head) from the first query that can see the tile's first key
// to the end of the sequence.  The items of all list tiles, in this order, are cut into `wpg` slices
// of equal length, one per workgroup; the part of a slice that lies in one list tile is a "piece" and
// produces one fp32 partial of that tile's dK / dV rows.  Piece (w, ft) uses partial slot w + ft
// (along the pieces either w or ft grows, so the slot numbers are distinct).
struct FarGeom {
    int wpg;     // workgroups per (batch, KV head)
    int bk;      // keys per workgroup and entries per list tile: 32 KW
    int NFcap;   // capacity of the far list, a multiple of bk
    int NFTcap;  // list tiles at full capacity
    int NP;      // partial slots per (batch, KV head)
    long rows;   // fp32 partial rows per (batch, KV head): NP slots of bk rows, then one band row per list entry
};
inline int dkv_workgroups_per_head(const sepattn_params &p, int kw) {
    const long n_bkv = (long)p.B * p.Hkv;
    const long w = dkv_workgroups_per_cu(p, kw) * (long)compute_units() / n_bkv;
    return (int)(w < 1 ? 1 : w);
}
__host__ __device__ inline FarGeom far_geom(const sepattn_params &p, int wpg, int kw) {
    FarGeom g;
    g.wpg = wpg;
    g.bk = 32 * kw;
    g.NFcap = (p.a + p.cap + g.bk - 1) / g.bk * g.bk;
    g.NFTcap = g.NFcap / g.bk;
    g.NP = wpg + g.NFTcap;
    g.rows = (long)g.NP * g.bk + g.NFcap;
    return g;
}

// backward workspace: D_i [B,Hq,L] fp32 | LSE_i * log2(e) [B,Hq,L] fp32 | dK partials | dV partials |
// first and last workgroup of every list tile [B,Hkv,NFTcap,2] int32
struct BwdWorkspace {
    size_t d_bytes, far_bytes, tab_bytes, total;
};
inline BwdWorkspace bwd_workspace(const sepattn_params &p) {
    BwdWorkspace w;
    w.d_bytes = align_up((size_t)p.B * p.Hq * p.L * sizeof(float), 256);
    w.far_bytes = w.tab_bytes = 0;
    // the eight-wave shape exists at d = 128 only
    for (int kw = 2; kw <= (p.d == 128 ? 4 : 2); kw += 2) {
        const FarGeom fg = far_geom(p, dkv_workgroups_per_head(p, kw), kw);
        const size_t far = align_up((size_t)p.B * p.Hkv * fg.rows * p.d * sizeof(float), 256);
        const size_t tab = align_up((size_t)p.B * p.Hkv * fg.NFTcap * 2 * sizeof(int32_t), 256);
        w.far_bytes = far > w.far_bytes ? far : w.far_bytes;
        w.tab_bytes = tab > w.tab_bytes ? tab : w.tab_bytes;
    }
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
                                      const sepattn_params &p, int bk) {
    return align_down32(far_pos(fl, (f / bk) * bk, idx, p.L) + p.n);
}

// one past the last query row the far pieces of list entry f's tile cover: the end of the sequence,
// or, with packed documents (dend: one past the last position of each position's document, else
// nullptr), the end of the document of the tile's last entry.  A tile whose first query row
// (far_first_query) is not below this has no far piece.
__device__ inline int far_last_query(const FarList &fl, int f, const int32_t *__restrict__ idx,
                                     const sepattn_params &p, const int32_t *__restrict__ dend, int bk) {
    if (!dend) return p.L;
    const int last = min((f / bk + 1) * bk, fl.NF) - 1;
    return min(max(dend[far_pos(fl, last, idx, p.L)], 0), p.L);
}

// doc_end: packed documents ([B, L], p.a == 0), or nullptr
int launch_dkv_bf16(const sepattn_params &p, const HeadWin &hw, const uint16_t *Q, const uint16_t *K, const uint16_t *V,
                    const float *lse2, const uint16_t *dO, const float *Dws, const int32_t *sep_idx,
                    const int32_t *sep_prefix, const int32_t *doc_end, uint16_t *dK, uint16_t *dV, float *farK,
                    float *farV, int32_t *piece_tab, hipStream_t st);

}  // namespace sepattn
