// SepAttention backward, bf16 MFMA: the analytic gradient of Eq. 1 under the mask of Eq. 2.
//
//   D_i = <dO_i, O_i>,  P_ij = exp(scale*<Q_i,K_j> - LSE_i),  dP_ij = <dO_i, V_j>,
//   dS_ij = P_ij (dP_ij - D_i),  dQ_i = scale sum_j dS_ij K_j,  dK_j = scale sum_i dS_ij Q_i,
//   dV_j = sum_i P_ij dO_i   (dK, dV summed over the query heads of the KV head).
//
// Three launches, no floating-point atomics (results are bit-reproducible):
//  1. dq_kernel (this file): persistent workgroups over the query tiles, same dense key stream as the forward
//     [initial | separators older than the window | band].  Also writes -D_i and LSE_i*log2(e).
//  2. dkv_kernel (bwd_dkv_bf16.hip): the visible pairs split into band pairs (i-j < n) and far
//     pairs (i-j >= n, j an initial token or a separator); far units work on the COMPACTED list of
//     such keys and write fp32 partials, band units finish the keys that are not on that list.
//  3. dkv_combine_kernel: adds, in fixed order, the partials of every far-list key and rounds once.
#include "bwd_common.h"
#include "mfma_common.h"
#include "key_stream.h"

namespace sepattn {

namespace {

__device__ inline float bf16_dot8(u32x4 a, u32x4 b) {
    float s = 0.f;
    const uint32_t *x = reinterpret_cast<const uint32_t *>(&a);
    const uint32_t *y = reinterpret_cast<const uint32_t *>(&b);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        s = fmaf(__uint_as_float(x[k] << 16), __uint_as_float(y[k] << 16), s);
        s = fmaf(__uint_as_float(x[k] & 0xFFFF0000u), __uint_as_float(y[k] & 0xFFFF0000u), s);
    }
    return s;
}

// ---------------------------------------------------------------------------------------------
// dQ
//
// Same workgroup shapes and key stream as the forward: NW = 8 or 4 waves, each with 32 query rows (one
// head, 32 positions) whose Q and dO rows stay in registers as B operands; K/V tiles of 64 stream
// elements pass through LDS (global->LDS loads two tiles ahead, one workgroup barrier per tile).
// Per block of 32 keys a wave runs
//     S^T = K Q^T,  dP^T = V dO^T   (16 matrix instructions, operands row-major from LDS)
//     dS = exp2(S*scale*log2e - LSE*log2e) * (dP - D), masked pairs zero, rounded to bf16
//     dQ^T += K^T dS^T              (8 matrix instructions, K read transposed from the same tile)
// with the operand fragments requested a few matrix instructions ahead.  K tiles are stored with
// the XOR permutation that serves both kinds of read (V tiles too, so that one set of per-lane
// offsets addresses both); four stages each (tile X+2 is requested while tile X is multiplied, by
// the first four waves only).  The two waves that share a SIMD (of one workgroup, or of the two
// workgroups on the compute unit) drift apart by themselves, so that one wave's exponentials overlap
// the other's matrix work.
// ---------------------------------------------------------------------------------------------
// DOCS: packed documents, as in the forward kernel (doc_start / doc_end [B, L]; p.a == 0).
template <int D, int GP, bool DOCS, int NW>
__global__ __launch_bounds__(64 * NW, 2) void dq_kernel(
    sepattn_params p, const uint16_t *__restrict__ Q, const uint16_t *__restrict__ K,
    const uint16_t *__restrict__ V, const uint16_t *__restrict__ O, const float *__restrict__ LSE,
    const uint16_t *__restrict__ dO, const int32_t *__restrict__ sep_idx,
    const int32_t *__restrict__ sep_prefix, const int32_t *__restrict__ doc_start,
    const int32_t *__restrict__ doc_end, uint16_t *__restrict__ dQ, float *__restrict__ Dws,
    float *__restrict__ Lws, int wpg, HeadWin hw) {
    constexpr int TP = 32 * NW / GP;
    constexpr int CH = D / 8;
    constexpr int RPL = 64 / CH;
    // the tile loads are issued by the first NLW waves only (all of them when NW = 4): of the two waves
    // of a workgroup that share a SIMD the older one (w < 4) is served first and reaches every barrier
    // long before its partner
    constexpr int NLW = 4;
    constexpr int LOADS = kBN / (RPL * NLW);
    constexpr int KSTEPS = D / 16;
    constexpr int DB = D / 32;
    // LDS stages of K, of V, and of the visibility ranges: powers of two, so that a stage number is
    // a mask of the tile number (the kernels spend their time issuing instructions, scalar ones too)
    constexpr int KST = 4, VST = 4, MKS = 4;
    constexpr int TILE = kBN * D;
    static_assert(LOADS >= 1 && LOADS * RPL * NLW == kBN, "tile must divide among the loading waves");

    __shared__ __attribute__((aligned(1024))) uint16_t Ks[KST][TILE];
    __shared__ __attribute__((aligned(1024))) uint16_t Vs[VST][TILE];
    __shared__ __attribute__((aligned(16))) int lo_s[MKS][kBN];
    __shared__ __attribute__((aligned(16))) int hi_s[MKS][kBN];
    // staging of one 32-column block of a wave's 32 dQ rows (see the end of a segment)
    __shared__ __attribute__((aligned(16))) uint16_t ostage[NW][32 * 32];
    constexpr int MR = LOADS * RPL;  // rows per wave and tile
    constexpr int MST = 4;           // ring stages of the index entries
    __shared__ __attribute__((aligned(256))) int meta_s[MST][NLW][64];  // 3 * MR <= 48 entries per wave and stage

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool loader = NW == NLW || wave < NLW;
    const int qi = lane & 31, hh = lane >> 5;
    // Persistent workgroups as in the forward kernel: a workgroup belongs to one (batch, KV head, head
    // group) and walks through several query tiles of it ("segments") in zig-zag order, `wpg`
    // workgroups per group; rank 0 is the last tile, the one with the longest key stream.
    const int G = p.Hq / p.Hkv, groups = G / GP;
    const int n_pos_tiles = (p.L + TP - 1) / TP;
    const TileGroup tg = xcd_tile_group(blockIdx.x, wpg, p.B * p.Hkv * groups);
    int y = tg.group;
    const int hg = y % groups;
    const int kv = (y / groups) % p.Hkv;
    const int b = y / (groups * p.Hkv);
    const int head = kv * G + hg * GP + (wave % GP);
    const int hdelta = head_delta(hw, head);  // head-wise windows: see the forward kernel

    const int32_t *prefix = sep_prefix + (long)b * (p.L + 1);
    const int32_t *idx = sep_idx + (long)b * p.cap;
    const int32_t *dstart = DOCS ? doc_start + (long)b * p.L : nullptr;
    const int32_t *dend = DOCS ? doc_end + (long)b * p.L : nullptr;
    const uint16_t *Kh = K + ((long)b * p.Hkv + kv) * (long)p.L * D;
    const uint16_t *Vh = V + ((long)b * p.Hkv + kv) * (long)p.L * D;

    // state of the segment being multiplied (the lambdas below refer to it)
    int iq = 0, iq_h = 0;
    FullBlocks fullb = {};
    bf16x8 qreg[KSTEPS], doreg[KSTEPS];
    float Di = 0.f, lse2 = 0.f;
    const float sl2 = p.scale * kLog2e_f;
    f32x16 acc[DB];

    // ---- tile loads (see the forward kernel: same scheme, other LDS layouts)
    const int my_pc = lane % CH, my_sub = lane / CH;
    const int row0 = LOADS * wave * RPL + my_sub;  // first of the rows of a tile this lane helps to fill (+ u * RPL)
    const char *Kb = reinterpret_cast<const char *>(Kh), *Vb = reinterpret_cast<const char *>(Vh);
    auto tile_class = [&](const Stream &ss, int t) {
        const int k0 = t * kBN;
        return (k0 + kBN <= ss.n_dense) ? 0 : (k0 >= ss.n_dense ? 1 : 2);
    };
    // A tile is named by the stream of its segment (ss), its number in that stream (t) and its
    // number in the concatenation of all segments of this workgroup (g), which selects the LDS stage.
    const int m_part = lane / MR, m_row = wave * MR + lane % MR;  // lanes 0 .. 3*MR-1 are used
    auto issue_meta = [&](const Stream &ss, int t, int g) __attribute__((always_inline)) {
        const int k = t * kBN + m_row;
        const int e = min(max(ss.sep_lo - ss.n_init + k, 0), p.cap - 1);
        const int j = min(max(ss.bs - ss.n_dense + k, 0), p.L - 1);
        const int32_t *src = m_part == 0 ? idx + e : prefix + j + (m_part - 1);
        if constexpr (DOCS) src = m_part == 3 ? dend + j : src;  // fourth part: where the key's document ends
        if (lane < (DOCS ? 4 : 3) * MR) dma_to_lds_4_addr(src, lds_addr(&meta_s[(unsigned)g % MST][wave % NLW][0]));
    };
    // One row of the tile at a time (the loading waves have time to spare, registers are scarce): read
    // the row's index entries, work out its key position and visibility range, request the row.
    // de: end of the document of the segment's first row; straddle: the segment's rows reach beyond it
    auto load_row = [&](const Stream &ss, int de, bool straddle, int t, int g, auto U) __attribute__((always_inline)) {
        constexpr int u = decltype(U)::value;
        const int *mt = &meta_s[(unsigned)g % MST][wave % NLW][0];
        const int rawi = mt[u * RPL + my_sub], raw0 = mt[MR + u * RPL + my_sub], raw1 = mt[2 * MR + u * RPL + my_sub];
        const int ms_ = (unsigned)g % MKS;
        const int r = row0 + u * RPL;
        const int k = t * kBN + r;
        // the clamp keeps a stale list tail (caller broke sep_count <= cap) from faulting
        const int jl = min(max(rawi, 0), p.L - 1);
        int jrow;
        if (tile_class(ss, t) == 0 && !(DOCS && straddle)) {
            jrow = k < ss.n_init ? k : jl;
        } else {
            const bool init = k < ss.n_init, dense = k < ss.n_dense, pad = k >= ss.n_total;
            const int jb = ss.bs + (k - ss.n_dense);
            const bool always = dense | (jb < p.a) | (raw1 != raw0);
            int j = init ? k : (dense ? jl : jb);
            j = pad ? 0 : j;
            const int lo = pad ? kIntMax : j;
            int hi = always ? kIntMax : jb + p.n - 1;
            if constexpr (DOCS) hi = min(hi, (dense ? de : mt[3 * MR + u * RPL + my_sub]) - 1);
            hi = pad ? -1 : hi;
            if (my_pc == 0) {
                lo_s[ms_][r] = lo;
                hi_s[ms_][r] = hi;
            }
            jrow = j;
        }
        const uint32_t kst = lds_addr(&Ks[(unsigned)g % KST][0]), vst = lds_addr(&Vs[(unsigned)g % VST][0]);
        const uint32_t wave_off = (uint32_t)((LOADS * wave + u) * RPL * D * 2);
        const uint32_t off = (uint32_t)jrow * (uint32_t)(D * 2) + swz_chunk<kSwzBoth, D>(my_pc, r) * 16;
        dma_to_lds_16(Kb, off, kst + wave_off);
        dma_to_lds_16(Vb, off, vst + wave_off);
    };

    // ---- segments of this workgroup and the load cursor: the tiles of all segments form one stream
    // of loads; the cursor (segment lcur, tile l_t, global number l_g) points at the next tile whose
    // rows are to be requested, two tiles ahead of the tile being multiplied, also across segment
    // borders.  Past the last segment the stream is empty: its tiles are "loaded" too (row 0, never
    // visible), which keeps the count of outstanding loads exact.
    struct Seg {
        Stream st;
        int n_tiles, i0, de;
    };
    auto open_segment = [&](int round) {
        Seg g;
        const int rank = round * wpg + ((round & 1) ? wpg - 1 - tg.rank : tg.rank);
        if (rank >= n_pos_tiles) {
            g.st = Stream{0, 0, 0, 0, 0};
            g.n_tiles = kIntMax;
            g.i0 = -1;
            g.de = kIntMax;
        } else {
            g.i0 = (n_pos_tiles - 1 - rank) * TP;
            if constexpr (DOCS) {
                // the clamps keep inconsistent bounds (caller error) from faulting
                const int ds = min(max(dstart[g.i0], 0), g.i0);
                g.de = min(max(dend[g.i0], g.i0 + 1), p.L);
                g.st = make_stream_docs(p, prefix, g.i0, TP, ds);
            } else {
                g.de = kIntMax;
                g.st = make_stream(p, prefix, g.i0, TP);
            }
            g.n_tiles = (g.st.n_total + kBN - 1) / kBN;
        }
        return g;
    };
    Seg lcur = open_segment(0), lnext = open_segment(1);
    int l_round = 0, l_t = 0, l_g = 0;
    auto advance_cursor = [&]() __attribute__((always_inline)) {
        ++l_g;
        if (++l_t == lcur.n_tiles) {
            lcur = lnext;
            ++l_round;
            l_t = 0;
            lnext = open_segment(l_round + 1);
        }
    };
    auto issue_meta_after_cursor = [&]() __attribute__((always_inline)) {
        if (l_t + 1 < lcur.n_tiles)
            issue_meta(lcur.st, l_t + 1, l_g + 1);
        else
            issue_meta(lnext.st, 0, l_g + 1);
    };
    // a tile step issues [1 entry load][2*LOADS row loads], in this order; loads complete in order
    auto wait_vmcnt = [&](auto N) __attribute__((always_inline)) {
        constexpr int n = decltype(N)::value;
        static_assert(n == 2 || n == 3 || n == 4 || n == 5 || n == 8 || n == 9, "add the count");
        if constexpr (n == 2) asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
        if constexpr (n == 3) asm volatile("s_waitcnt vmcnt(3)" ::: "memory");
        if constexpr (n == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
        if constexpr (n == 5) asm volatile("s_waitcnt vmcnt(5)" ::: "memory");
        if constexpr (n == 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        if constexpr (n == 9) asm volatile("s_waitcnt vmcnt(9)" ::: "memory");
    };
    auto entries_landed = [&]() __attribute__((always_inline)) { wait_vmcnt(IntC<2 * LOADS>{}); };
    // (a wave that loads nothing has nothing in flight: the wait falls through)
    auto wait_older_loads = [&]() __attribute__((always_inline)) { wait_vmcnt(IntC<1 + 2 * LOADS>{}); };
    auto wg_barrier = [&]() __attribute__((always_inline)) {
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };

    // per-lane byte offsets of the operand fragments inside a tile
    const int a_row = pi_row(qi);
    const uint32_t ks_base = lds_addr(&Ks[0][0]), vs_base = lds_addr(&Vs[0][0]);
    // Row-major fragments: the XOR permutation acts on the 16-byte chunk index 2*ks + hh, and the
    // k-step only enters through bits 1..3 of it, so fragment ks sits at (fragment 0) ^ (32 * ks):
    // one register instead of KSTEPS.  (Tile bases are multiples of 1 KB, so the XOR commutes with
    // adding the base.)  K and V tiles share one layout and therefore these offsets.
    const uint32_t koff0 = lds_off_a<kSwzBoth, D>(a_row, hh);
    uint32_t ktr0[DB], ktr1[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) {
        ktr0[db] = lds_off_a_tr<kSwzBoth, D>(db * 32, lane);
        ktr1[db] = lds_off_a_tr_second<kSwzBoth, D>(db * 32, lane);
    }
    // for d = 128 the second transposed read is the first with chunk bit 0 flipped, four rows on
    auto tr_second = [&](uint32_t first, int db) __attribute__((always_inline)) {
        if constexpr (D == 128)
            return (first ^ 16u) + 4u * D * 2u;
        else
            return first - ktr0[db] + ktr1[db];
    };

    // ---- one block of 32 keys: tile X of the current segment (global number gbase + X), block HB
    int gbase = 0;
    constexpr int LA = 4;
    constexpr int NS1 = 2 * KSTEPS, NS2 = 2 * DB;  // matrix instructions: scores, then the dQ update
    auto block_step = [&](int X, auto HB_, auto LD_) __attribute__((always_inline)) {
        constexpr int HB = decltype(HB_)::value;
        constexpr bool DO_LD = decltype(LD_)::value != 0;
        const uint32_t kst = ks_base + ((unsigned)(gbase + X) % KST) * (TILE * 2) + HB * 32 * D * 2;
        const uint32_t vst = vs_base + ((unsigned)(gbase + X) % VST) * (TILE * 2) + HB * 32 * D * 2;
        f32x16 sacc, pacc;
        bf16x8 frag[LA];
        auto request1 = [&](auto S) __attribute__((always_inline)) {
            constexpr int s = decltype(S)::value;
            if constexpr (s < NS1) {
                constexpr int ks = s / 2;
                frag[s % LA] = lds_read_b128_at(((s % 2 == 0 ? kst : vst) + koff0) ^ (32u * ks));
            }
        };
        static_for<LA>([&](auto S) { request1(S); });
        __builtin_amdgcn_sched_barrier(0);
        static_for<NS1>([&](auto S) {
            constexpr int s = decltype(S)::value, ks = s / 2;
            const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            if constexpr (s % 2 == 0)
                sacc = mfma_bf16(frag[s % LA], qreg[ks], ks == 0 ? zero : sacc);
            else
                pacc = mfma_bf16(frag[s % LA], doreg[ks], ks == 0 ? zero : pacc);
            request1(IntC<s + LA>{});
            // the load path of the tile at the cursor (two tiles ahead) rides along with the first
            // block of the tile
            if constexpr (DO_LD) {
                static_assert(NS1 / 4 + 2 * (LOADS - 1) < NS1 - 1, "the row slots must come before the cursor moves");
                // order of the requests: [entries of the tile after the cursor] [rows of the tile at it]
                if (loader) {
                    if constexpr (s == 0) {
                        entries_landed();
                        issue_meta_after_cursor();
                    } else if constexpr (s >= NS1 / 4 && (s - NS1 / 4) % 2 == 0 && (s - NS1 / 4) / 2 < LOADS) {
                        load_row(lcur.st, lcur.de, lcur.i0 + TP > lcur.de, l_t, l_g, IntC<(s - NS1 / 4) / 2>{});
                    } else if constexpr (s == NS1 - 1) {
                        advance_cursor();
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        });
        // transposed K fragments of the first half of the dQ update are requested before the dS
        // arithmetic, those of the second half while the first half multiplies
        bf16x8 tfr[DB];
#pragma unroll
        for (int db = 0; db < DB; ++db) tfr[db] = lds_read_tr_at2(kst + ktr0[db], tr_second(kst + ktr0[db], db));
        // dS = P (dP - D), zero where masked
        if (!block_is_full(fullb, X * kBN + HB * 32)) {
            const int ms_ = (unsigned)(gbase + X) % MKS;
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const int base = HB * 32 + 16 * half + 8 * hh;
                const int4 lo0 = *reinterpret_cast<const int4 *>(&lo_s[ms_][base]);
                const int4 lo1 = *reinterpret_cast<const int4 *>(&lo_s[ms_][base + 4]);
                const int4 hi0 = *reinterpret_cast<const int4 *>(&hi_s[ms_][base]);
                const int4 hi1 = *reinterpret_cast<const int4 *>(&hi_s[ms_][base + 4]);
                const int los[8] = {lo0.x, lo0.y, lo0.z, lo0.w, lo1.x, lo1.y, lo1.z, lo1.w};
                const int his[8] = {hi0.x, hi0.y, hi0.z, hi0.w, hi1.x, hi1.y, hi1.z, hi1.w};
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const bool vis = (los[k] <= iq) & (iq_h <= his[k]);
                    sacc[8 * half + k] = vis ? sacc[8 * half + k] : -INFINITY;
                }
            }
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float pr = __builtin_amdgcn_exp2f(fmaf(sacc[i], sl2, -lse2));
            sacc[i] = pr * (pacc[i] - Di);
        }
        const bf16x8 dsb0 = pack_bf16x8(sacc, 0), dsb1 = pack_bf16x8(sacc, 8);
        // dQ^T += K^T dS^T
        bf16x8 tfr2[DB];
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            acc[db] = mfma_bf16(tfr[db], dsb0, acc[db]);
            tfr2[db] = lds_read_tr_at2(kst + ktr0[db] + 16 * D * 2, tr_second(kst + ktr0[db], db) + 16 * D * 2);
        }
#pragma unroll
        for (int db = 0; db < DB; ++db) acc[db] = mfma_bf16(tfr2[db], dsb1, acc[db]);
    };

    // ---- start-up, once per workgroup: the first two tiles of the concatenated stream on their way
    // into LDS, the index entries of the third requested
    if (loader) {
        issue_meta(lcur.st, 0, 0);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
        for (int rep = 0; rep < 2; ++rep) {
            issue_meta_after_cursor();
            static_for<LOADS>([&](auto U) { load_row(lcur.st, lcur.de, lcur.i0 + TP > lcur.de, l_t, l_g, U); });
            advance_cursor();
            entries_landed();  // the entries just requested (the rows after them may be in flight)
        }
    }

    const IntC<1> yes;
    const IntC<0> no;
    // The wave's 32 rows of Q, dO and O of a segment.  The operand layout wants, per lane, 16-byte pieces
    // of ONE row; fetched that way every load instruction is 64 scattered pieces, and their number (1536
    // per wave and segment) is what such loads cost.  They are fetched instead so that four consecutive
    // lanes cover 64 contiguous bytes of a row (column block cb of 32 columns, rows 16 t + lane / 4,
    // piece lane % 4), and they are requested one segment ahead, before the previous segment's dQ rows
    // are stored, so that the store path hides their latency.  (Past the last segment: row 0, unused.)
    constexpr int CB = D / 32;  // column blocks of 32 columns (64 bytes of a row)
    const long head_row0 = ((long)b * p.Hq + head) * p.L;  // rows of this wave's head
    u32x4 q4[CB][2], do4[CB][2], o4[CB][2];
    auto fetch_rows = [&](const Seg &sg) __attribute__((always_inline)) {
        const char *qb = reinterpret_cast<const char *>(Q + head_row0 * D);
        const char *dob = reinterpret_cast<const char *>(dO + head_row0 * D);
        const char *ob = reinterpret_cast<const char *>(O + head_row0 * D);
        const int pwn = max(sg.i0, 0) + 32 * (wave / GP);
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const uint32_t roff = (uint32_t)min(pwn + 16 * t + (lane >> 2), p.L - 1) * (uint32_t)(D * 2) + 16u * (lane & 3);
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) {
                q4[cb][t] = *reinterpret_cast<const u32x4 *>(qb + (roff + 64u * cb));
                do4[cb][t] = *reinterpret_cast<const u32x4 *>(dob + (roff + 64u * cb));
                o4[cb][t] = *reinterpret_cast<const u32x4 *>(ob + (roff + 64u * cb));
            }
        }
    };
    Seg cseg = open_segment(0);
    fetch_rows(cseg);
    for (int round = 0; cseg.i0 >= 0; ++round) {
        const int pw = cseg.i0 + 32 * (wave / GP);
        iq = pw + qi;
        iq_h = iq + hdelta;
        fullb = full_blocks(cseg.st, pw, p.n - hdelta);
        if (DOCS && pw + 31 >= cseg.de) fullb = no_full_blocks();
        {
            // Q and dO reach their operand layout through the wave's 2 KB staging area, one column block
            // at a time (16-byte piece c of row r at piece position c ^ ((r / 4) % 4); the LDS operations
            // of a wave execute in order).  D_i = sum_k dO_ik O_ik needs no particular layout: partial
            // sums per lane, then over the four lanes of a row, then handed to the lane pair that owns
            // the row.
            float part[2] = {0.f, 0.f};
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) part[t] += bf16_dot8(do4[cb][t], o4[cb][t]);
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                part[t] += __shfl_xor(part[t], 1);
                part[t] += __shfl_xor(part[t], 2);
            }
            // row qi is held by the lanes 4 (qi % 16) .. +3 in part[qi / 16]
            {
                const float d0 = __shfl(part[0], 4 * (qi & 15)), d1 = __shfl(part[1], 4 * (qi & 15));
                Di = qi < 16 ? d0 : d1;
            }
            uint16_t *stg = &ostage[wave][0];
            const int wr0 = (lane >> 2), wc = lane & 3;
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) {
                static_for<2>([&](auto X) {
                    constexpr bool is_q = decltype(X)::value == 0;
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        const int r = 16 * t + wr0;
                        *reinterpret_cast<u32x4 *>(stg + r * 32 + ((wc ^ ((r >> 2) & 3)) * 8)) = is_q ? q4[cb][t] : do4[cb][t];
                    }
#pragma unroll
                    for (int k2 = 0; k2 < 2; ++k2) {
                        const u32x4 v = *reinterpret_cast<const u32x4 *>(stg + qi * 32 + (((2 * k2 + hh) ^ ((qi >> 2) & 3)) * 8));
                        if constexpr (is_q) qreg[2 * cb + k2] = as_bf16x8(v);
                        else doreg[2 * cb + k2] = as_bf16x8(v);
                    }
                });
            }
            const uint32_t soff = (uint32_t)min(iq, p.L - 1) * 4u;
            lse2 = *reinterpret_cast<const float *>(reinterpret_cast<const char *>(LSE + head_row0) + soff) * kLog2e_f;
            if (hh == 0 && iq < p.L) {
                // stored negated: the dK/dV kernel starts its dP accumulator from -D
                *reinterpret_cast<float *>(reinterpret_cast<char *>(Dws + head_row0) + soff) = -Di;
                // the dK/dV kernels work in the log2 domain too
                *reinterpret_cast<float *>(reinterpret_cast<char *>(Lws + head_row0) + soff) = lse2;
            }
        }
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[db][i] = 0.f;

        // Tile step X reads K and V of tile gbase+X (row-major and transposed) and requests the tile
        // two further on, whose stages held tile gbase+X-1: last read in the previous step, which
        // every wave has left when it passes the barrier.  The barrier publishes tile gbase+X: each
        // wave has waited for everything older than the previous step's requests.
        const int n_tiles = cseg.n_tiles;
        // the second block of the last tile is skipped when it is all padding (the same decision in
        // every wave; the tile loads ride on the first block)
        const int n_keys = cseg.st.n_total;
        for (int X = 0; X < n_tiles; ++X) {
            wait_older_loads();
            wg_barrier();
            block_step(X, IntC<0>{}, yes);
            if (X * kBN + 32 < n_keys) block_step(X, IntC<1>{}, no);
        }
        gbase += n_tiles;
        const Seg nseg = open_segment(round + 1);
        fetch_rows(nseg);
        __builtin_amdgcn_sched_barrier(0);

        // A lane holds 4-column pieces of ONE dQ row: stored straight from the accumulators they are 64
        // scattered 8-byte pieces per instruction, and their number is what the stores cost.  Each
        // 32-column block of the wave's 32 rows goes through a 2 KB staging area of the wave instead
        // and leaves as 16-byte pieces of which four consecutive lanes cover 64 contiguous bytes of a
        // row.  8-byte chunk ch of row r sits at chunk position ch ^ (2 * ((r / 4) % 4)); the LDS
        // operations of a wave execute in order, so a block's reads precede the next block's writes.
        {
            uint16_t *stg = &ostage[wave][0];
            const int wsw = ((qi >> 2) & 3) << 1;
#pragma unroll
            for (int db = 0; db < DB; ++db) {
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    const uint2 v = pack_bf16x4(acc[db][4 * i4] * p.scale, acc[db][4 * i4 + 1] * p.scale,
                                                acc[db][4 * i4 + 2] * p.scale, acc[db][4 * i4 + 3] * p.scale);
                    *reinterpret_cast<uint2 *>(stg + qi * 32 + (((2 * i4 + hh) ^ wsw) * 4)) = v;
                }
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    const int r = 16 * t + (lane >> 2), c = lane & 3;
                    const int pos = (2 * c) ^ (((r >> 2) & 3) << 1);
                    const uint4 v = *reinterpret_cast<const uint4 *>(stg + r * 32 + pos * 4);
                    if (pw + r < p.L) *reinterpret_cast<uint4 *>(dQ + (head_row0 + pw + r) * D + db * 32 + c * 8) = v;
                }
                __builtin_amdgcn_sched_barrier(0);  // one block at a time: keeps the register pressure down
            }
        }
        cseg = nseg;
    }
    // the loads of the padding tiles past the last segment must have landed before the workgroup
    // ends and its LDS is handed on
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

template <int D, bool DOCS>
int launch_bwd(const sepattn_params &p, const uint16_t *Q, const uint16_t *K, const uint16_t *V,
               const uint16_t *O, const float *LSE, const uint16_t *dO, const int32_t *sep_idx,
               const int32_t *sep_prefix, const int32_t *doc_start, const int32_t *doc_end, uint16_t *dQ,
               uint16_t *dK, uint16_t *dV, void *ws, const HeadWin &hw, hipStream_t st) {
    const BwdWorkspace w = bwd_workspace(p);
    char *base = static_cast<char *>(ws);
    float *Dws = reinterpret_cast<float *>(base);
    float *Lws = reinterpret_cast<float *>(base + w.d_bytes);
    float *farK = reinterpret_cast<float *>(base + 2 * w.d_bytes);
    float *farV = reinterpret_cast<float *>(base + 2 * w.d_bytes + w.far_bytes);
    int32_t *piece_tab = reinterpret_cast<int32_t *>(base + 2 * w.d_bytes + 2 * w.far_bytes);

    int G = p.Hq / p.Hkv;
    int GP = (G % 4 == 0) ? 4 : (G % 2 == 0) ? 2 : 1;
    // Workgroups of eight waves, one per compute unit (the LDS footprint allows no more).  At d = 64
    // the K/V stages are half as large and two independent workgroups of four waves fit a compute
    // unit: one's segment start and row stores overlap the other's matrix work, their barriers do not
    // lock each other's phases, and the split of a group is twice as fine (it fills the chip where
    // 256 / groups is not a whole number).  A four-wave workgroup has half the query rows per K/V
    // tile, i.e. twice the tile loads per matrix instruction: where four grouped heads share the
    // tile (32 positions per workgroup instead of 64) the eight-wave shape stays the better one
    // (by 2-5 % at any length), with one or two heads per tile the four-wave shape wins (5-25 %).
    const bool narrow = D == 64 && GP <= 2;
    const int NWr = narrow ? 4 : 8;
    int TP = 32 * NWr / GP;
    const int n_pos_tiles = (p.L + TP - 1) / TP;
    const long n_groups = (long)p.B * p.Hkv * (G / GP);
    // persistent workgroups, spread evenly over the groups; never more than a group has tiles
    int wpg = (int)((8 / NWr) * (long)compute_units() / n_groups);
    wpg = wpg < 1 ? 1 : (wpg > n_pos_tiles ? n_pos_tiles : wpg);
    if (n_groups * wpg > 0x7FFFFFFFL) return SEPATTN_ERR_SHAPE;
    dim3 grid((unsigned)(n_groups * wpg)), block(64 * NWr);
    {
    ProfScope prof(SEPATTN_K_BWD_DQ, st);
    auto go = [&](auto NW_) {
        constexpr int NW = decltype(NW_)::value;
        if (GP == 4)
            hipLaunchKernelGGL((dq_kernel<D, 4, DOCS, NW>), grid, block, 0, st, p, Q, K, V, O, LSE, dO, sep_idx, sep_prefix, doc_start, doc_end, dQ, Dws, Lws, wpg, hw);
        else if (GP == 2)
            hipLaunchKernelGGL((dq_kernel<D, 2, DOCS, NW>), grid, block, 0, st, p, Q, K, V, O, LSE, dO, sep_idx, sep_prefix, doc_start, doc_end, dQ, Dws, Lws, wpg, hw);
        else
            hipLaunchKernelGGL((dq_kernel<D, 1, DOCS, NW>), grid, block, 0, st, p, Q, K, V, O, LSE, dO, sep_idx, sep_prefix, doc_start, doc_end, dQ, Dws, Lws, wpg, hw);
    };
    if constexpr (D == 64) {
        if (narrow) go(IntC<4>{});
        else go(IntC<8>{});
    } else {
        go(IntC<8>{});
    }
    }
    if (hipGetLastError() != hipSuccess) return SEPATTN_ERR_HIP;
    return launch_dkv_bf16(p, hw, Q, K, V, Lws, dO, Dws, sep_idx, sep_prefix, doc_end, dK, dV, farK, farV, piece_tab, st);
}

}  // namespace

size_t backward_bf16_workspace(const sepattn_params &p) { return bwd_workspace(p).total; }

int launch_backward_bf16(const sepattn_params &p, const HeadWin &hw, const void *Q, const void *K, const void *V,
                         const void *O, const float *LSE, const void *dO, const int32_t *sep_idx,
                         const int32_t *, const int32_t *sep_prefix, const int32_t *doc_start,
                         const int32_t *doc_end, void *dQ, void *dK, void *dV, void *ws, hipStream_t st) {
    auto u = [](const void *x) { return static_cast<const uint16_t *>(x); };
    auto w = [](void *x) { return static_cast<uint16_t *>(x); };
    if (doc_start) {
        if (p.d == 64)
            return launch_bwd<64, true>(p, u(Q), u(K), u(V), u(O), LSE, u(dO), sep_idx, sep_prefix, doc_start, doc_end,
                                        w(dQ), w(dK), w(dV), ws, hw, st);
        return launch_bwd<128, true>(p, u(Q), u(K), u(V), u(O), LSE, u(dO), sep_idx, sep_prefix, doc_start, doc_end,
                                     w(dQ), w(dK), w(dV), ws, hw, st);
    }
    if (p.d == 64)
        return launch_bwd<64, false>(p, u(Q), u(K), u(V), u(O), LSE, u(dO), sep_idx, sep_prefix, nullptr, nullptr,
                                     w(dQ), w(dK), w(dV), ws, hw, st);
    return launch_bwd<128, false>(p, u(Q), u(K), u(V), u(O), LSE, u(dO), sep_idx, sep_prefix, nullptr, nullptr,
                                  w(dQ), w(dK), w(dV), ws, hw, st);
}

}  // namespace sepattn
