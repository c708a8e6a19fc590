// Geometry shared by the backward kernels: the compacted list of "far" keys (initial tokens and
// separators, the only keys a query can see beyond its neighbour window, Sec. 3.1) and the split of
// the query range into chunks for the far pass of dK/dV.
#pragma once

#include "common.h"

namespace sepattn {

constexpr int kFarChunks = 16;  // at most this many query chunks for the far pass
constexpr int kFarChunkMin = 512;
constexpr int kDkvWaves = 4;              // key blocks of 32 keys per dK/dV workgroup (two waves each)
constexpr int kDkvThreads = 2 * 64 * kDkvWaves;
constexpr int kBK = 32 * kDkvWaves;  // keys per dK/dV workgroup
constexpr int kBQ = 64;              // queries per LDS tile in the dK/dV kernels

__host__ __device__ inline int align_down32(int x) { return x & ~31; }

struct FarGeom {
    int CQ, NCH, NFcap;
};
__host__ __device__ inline FarGeom far_geom(const sepattn_params &p) {
    FarGeom g;
    int cq = (p.L + kFarChunks - 1) / kFarChunks;
    cq = (cq + 31) / 32 * 32;
    g.CQ = cq < kFarChunkMin ? kFarChunkMin : cq;
    g.NCH = (p.L + g.CQ - 1) / g.CQ;
    g.NFcap = (p.a + p.cap + kBK - 1) / kBK * kBK;
    return g;
}

// backward workspace: D_i [B,Hq,L] fp32 | LSE_i * log2(e) [B,Hq,L] fp32 | far dK partials | far dV partials
struct BwdWorkspace {
    size_t d_bytes, far_bytes, total;
};
inline BwdWorkspace bwd_workspace(const sepattn_params &p) {
    FarGeom fg = far_geom(p);
    BwdWorkspace w;
    w.d_bytes = align_up((size_t)p.B * p.Hq * p.L * sizeof(float), 256);
    w.far_bytes = align_up((size_t)p.B * p.Hkv * (fg.NCH + 1) * fg.NFcap * p.d * sizeof(float), 256);
    w.total = 2 * w.d_bytes + 2 * w.far_bytes;
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
// first query row the far units of list entry f's tile cover (>= L: the entry has no far unit)
__device__ inline int far_first_query(const FarList &fl, int f, const int32_t *__restrict__ idx,
                                      const sepattn_params &p) {
    return align_down32(far_pos(fl, (f / kBK) * kBK, idx, p.L) + p.n);
}

int launch_dkv_bf16(const sepattn_params &p, const uint16_t *Q, const uint16_t *K, const uint16_t *V,
                    const float *lse2, const uint16_t *dO, const float *Dws, const int32_t *sep_idx,
                    const int32_t *sep_prefix, uint16_t *dK, uint16_t *dV, float *farK, float *farV,
                    hipStream_t st);

}  // namespace sepattn
