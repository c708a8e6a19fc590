// SepAttention backward, dK and dV (bf16 MFMA): the analytic gradient of Eq. 1 under the mask of Eq. 2,
//   dV_j = sum_i P_ij dO_i,   dK_j = scale sum_i dS_ij Q_i,   dS_ij = P_ij (<dO_i, V_j> - D_i),
//   P_ij = exp(scale <Q_i, K_j> - LSE_i),  summed over the query heads of the KV head.
//
// The visible pairs split into band pairs (i-j < n) and far pairs (i-j >= n, j an initial token or a
// separator, Sec. 3.1).  dkv_kernel runs persistent workgroups, `wpg` per (batch, KV head), each of
// which works through
//   its far pieces: far pairs on the COMPACTED list of such keys.  For list tile ft (128 consecutive
//              list entries, gathered K/V rows) the work is the sequence of items (query tile of 64
//              rows, query head) from the first query that sees the tile's first key to the end of
//              the sequence; the items of all list tiles, concatenated, are cut into wpg equal
//              slices, and the part of a workgroup's slice inside one list tile is a piece.  A piece
//              writes an fp32 partial dK/dV of the tile's rows to the workspace (slot w + ft).
//   its band units: 128 consecutive keys against the queries j <= i < j+n (units w, w+wpg, ...).
//              Keys that are not on the far list are finished here (rounded once to bf16); for the
//              others the band unit writes one more fp32 partial.
// dkv_combine_kernel then adds, in fixed order, the partials of every far-list key and rounds once to
// bf16.  One workgroup owns each partial row: no atomics, results are bit-reproducible.  Every
// workgroup gets the same amount of far work and (up to one) the same number of band units, so the
// compute units finish together.
// A workgroup is 8 waves = 4 key blocks of 32 keys x 2 roles.  The two waves of a key block split
// the four contractions so that each keeps only one operand matrix and one accumulator resident:
//   P-wave :  S = Q K^T   -> P = exp2(.)      -> dV^T += dO^T P     (holds K rows, dV^T)
//   dS-wave:  dP = dO V^T -> dS = P (dP - D)  -> dK^T += Q^T dS     (holds V rows, dK^T)
// P travels from the first to the second through a small LDS buffer (same lane, same register:
// both are 32x32 accumulator layouts), once per block of 32 queries, fenced by the block's
// workgroup barrier (P is exchanged in bf16, the form it has in the second contraction anyway).  Query
// tiles (64 rows of Q and dO, plus LSE*log2e and -D) stream through a ring of four LDS buffers filled
// by direct global->LDS loads issued as soon as a buffer is free; with the ring the block barriers
// are the only barriers.  The tiles are stored unpadded with XOR-permuted 16-byte
// chunks so that both the row-major reads (first contraction) and the transposed reads (second
// contraction) are free of bank conflicts.  The four query heads of a GQA group are just four times
// as many query tiles.
#include "bwd_common.h"
#include "mfma_common.h"


namespace sepattn {

namespace {

__device__ inline int wave_min_i(int v) {
    for (int off = 32; off > 0; off >>= 1) v = min(v, __shfl_xor(v, off));
    return v;
}
__device__ inline int wave_max_i(int v) {
    for (int off = 32; off > 0; off >>= 1) v = max(v, __shfl_xor(v, off));
    return v;
}

// DOCS: packed documents (doc_end [B, L]: one past the last position of each position's document;
// p.a == 0, the documents' initial tokens are list entries): a key's query range ends with its
// document, and the far pieces of a list tile end with the document of the tile's last entry.
// HW: head-wise windows.  p.n is the largest window: it fixes the far / band split and the schedule;
// in a band unit a key that is neither an initial token nor a separator is visible to query i of head
// h only while i <= j + p.n - 1 - delta[h] (a third comparison in the blocks that need the mask test).
template <int D, bool DOCS, bool HW, int KW>
__global__ __launch_bounds__(128 * KW, KW == 4 ? 1 : (D == 64 ? 3 : 2)) void dkv_kernel(
    sepattn_params p, const uint16_t *__restrict__ Q, const uint16_t *__restrict__ K,
    const uint16_t *__restrict__ V, const float *__restrict__ LSE2, const uint16_t *__restrict__ dO,
    const float *__restrict__ Dws, const int32_t *__restrict__ sep_idx,
    const int32_t *__restrict__ sep_prefix, const int32_t *__restrict__ doc_end,
    uint16_t *__restrict__ dK, uint16_t *__restrict__ dV,
    float *__restrict__ farK, float *__restrict__ farV, int32_t *__restrict__ piece_tab, int wpg, int n_band,
    HeadWin hw) {
    constexpr int NW = 2 * KW;               // waves per workgroup
    constexpr int BK = 32 * KW;              // keys per workgroup
    constexpr int CH = D / 8;                // 16-byte chunks per row
    constexpr int RPL = 64 / CH;             // rows covered by one wave-wide 1 KB load
    // Query rows per LDS tile.  Workgroups that share a compute unit (two at d = 128 with 80 KB each,
    // three at d = 64 with 53 KB and 168 registers) stream tiles of 32 rows (one block) through the
    // ring of four, the single workgroup tiles of 64 rows (two blocks).
    constexpr int BQ = KW == 2 ? 32 : 64;
    constexpr int BPT = BQ / 32;             // blocks of 32 query rows per tile
    constexpr int LOADS = BQ / (RPL * NW);   // wave-wide loads per wave per tensor per tile
    constexpr int RVL = (2 * BQ / 16) / NW;  // loads of sixteen row values (LSE*log2e or -D) per wave per tile
    constexpr int KSTEPS = D / 16;
    constexpr int DB = D / 32;
    constexpr int TILE = BQ * D;
    constexpr int NBUF = 4;
    static_assert(LOADS >= 1 && LOADS * RPL * NW == BQ && RVL >= 1 && RVL * 16 * NW == 2 * BQ, "tile must divide among the waves");

    __shared__ __attribute__((aligned(1024))) uint16_t Qs[NBUF][TILE];
    __shared__ __attribute__((aligned(1024))) uint16_t dOs[NBUF][TILE];
    __shared__ __attribute__((aligned(256))) float lse_s[NBUF][BQ];
    __shared__ __attribute__((aligned(256))) float d_s[NBUF][BQ];
    __shared__ __attribute__((aligned(1024))) uint16_t Pex[KW][2][2][64 * 8];  // [key block][step parity][k-half][lane*8], bf16

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int role = wave / KW;  // 0: P-wave (S, dV), 1: dS-wave (dP, dK)
    const int kbw = wave % KW;   // key block of the wave
    const int kj = lane & 31, hh = lane >> 5;
    const int G = p.Hq / p.Hkv;
    // 1-D grid: consecutive workgroups belong to consecutive (batch, KV head) pairs, so with 8 KV heads
    // each head's K, V, Q, dO rows stay in the L2 of one XCD.
    const int n_bkv = p.B * p.Hkv;
    const int bkv = blockIdx.x % n_bkv, w_id = blockIdx.x / n_bkv;
    const int kv = bkv % p.Hkv, b = bkv / p.Hkv;
    const int32_t *prefix = sep_prefix + (long)b * (p.L + 1);
    const int32_t *idx = sep_idx + (long)b * p.cap;
    const int32_t *dend = DOCS ? doc_end + (long)b * p.L : nullptr;
    const long kvrow0 = ((long)b * p.Hkv + kv) * (long)p.L;
    const float sl2 = p.scale * kLog2e_f;
    const FarGeom fg = far_geom(p, wpg, KW);
    const FarList fl = far_list(p, prefix);
    const int a_row = pi_row(kj);
    const int my_pc = lane % CH, my_sub = lane / CH;
    // Per-lane byte offsets of the operand fragments inside a tile, computed once.  The first
    // contraction reads rows of T1 (Q for the P-wave, dO for the dS-wave), the second reads the other
    // tensor (T2) transposed.  Row-major fragments: the XOR permutation acts on the 16-byte chunk
    // index 2*ks + hh and the k-step only enters through bits 1..3 of it, so fragment ks sits at
    // (fragment 0) ^ (32 * ks); tile and block bases are multiples of 1 KB, so the XOR commutes with
    // adding them.
    const uint32_t q_base = lds_addr(&Qs[0][0]), do_base = lds_addr(&dOs[0][0]);
    const uint32_t t1_base = (role == 0 ? q_base : do_base) + lds_off_a<kSwzBoth, D>(a_row, hh);
    const uint32_t t2_base = role == 0 ? do_base : q_base;
    uint32_t ktr0[DB], ktr1[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) {
        ktr0[db] = t2_base + lds_off_a_tr<kSwzBoth, D>(db * 32, lane);
        ktr1[db] = t2_base + lds_off_a_tr_second<kSwzBoth, D>(db * 32, lane);
    }

    // ---- the far work of this (batch, KV head) and this workgroup's slice [s0, s1) of it.
    // Lane t of a group of 64 list tiles describes tile t: first query row and number of items.
    const int NFT = (fl.NF + BK - 1) / BK;
    auto tile_items = [&](int t, int &fq) __attribute__((always_inline)) {
        fq = p.L;
        int qe = p.L;
        if (t < NFT) {
            fq = align_down32(far_pos(fl, t * BK, idx, p.L) + p.n);
            qe = far_last_query(fl, t * BK, idx, p, dend, BK);
        }
        return fq < qe ? G * ((qe - fq + BQ - 1) / BQ) : 0;
    };
    auto inclusive_scan = [&](int v) __attribute__((always_inline)) {
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int u = __shfl_up(v, off);
            if (lane >= off) v += u;
        }
        return v;
    };
    long far_total = 0;
    for (int base = 0; base < NFT; base += 64) {
        int fq;
        far_total += __builtin_amdgcn_readfirstlane(__shfl(inclusive_scan(tile_items(base + lane, fq)), 63));
    }
    // no more slices than items, so that no slice is empty: the pieces of a list tile then belong to
    // consecutive workgroups, which is what the combine kernel relies on
    const long wfar = far_total < wpg ? (far_total > 0 ? far_total : 1) : wpg;
    const long s0 = w_id < wfar ? w_id * far_total / wfar : far_total;
    const long s1 = w_id < wfar ? (w_id + 1) * far_total / wfar : far_total;

    // iteration state over the pieces: first the far pieces of the slice (list tiles in groups of 64,
    // `pend` = tiles of the current group that overlap the slice and are still to be visited), then
    // the band units
    int it_phase = 0, grp_next = 0, grp_base = 0, band_u = w_id;
    long cum_next = 0, grp_cum = 0;
    int g_fq = 0, g_nq = 0, g_excl = 0;
    unsigned long long pend = 0;
    for (;;) {
        bool FAR = false, have = false;
        int ft = 0, fq0 = 0, item0 = 0, n_items = 0, unit = 0, n_qt = 1;
        while (!have) {
            if (it_phase == 0) {
                if (pend == 0) {
                    if (grp_next >= NFT || cum_next >= s1) {
                        it_phase = 1;
                        continue;
                    }
                    grp_base = grp_next;
                    grp_cum = cum_next;
                    g_nq = tile_items(grp_base + lane, g_fq);
                    const int inc = inclusive_scan(g_nq);
                    g_excl = inc - g_nq;
                    pend = __ballot(g_nq > 0 && grp_cum + inc > s0 && grp_cum + g_excl < s1);
                    cum_next = grp_cum + __builtin_amdgcn_readfirstlane(__shfl(inc, 63));
                    grp_next = grp_base + 64;
                    continue;
                }
                const int l = __ffsll(pend) - 1;
                pend &= pend - 1;
                const long first = grp_cum + __builtin_amdgcn_readfirstlane(__shfl(g_excl, l));
                const int nq = __builtin_amdgcn_readfirstlane(__shfl(g_nq, l));
                const long lo_i = s0 > first ? s0 : first, hi_i = s1 < first + nq ? s1 : first + nq;
                ft = grp_base + l;
                fq0 = __builtin_amdgcn_readfirstlane(__shfl(g_fq, l));
                item0 = (int)(lo_i - first);
                n_items = (int)(hi_i - lo_i);
                n_qt = nq / G;
                // the combine kernel finds the pieces of a list tile through its first and last workgroup
                if (tid == 0) {
                    int32_t *tab = piece_tab + ((long)bkv * fg.NFTcap + ft) * 2;
                    if (item0 == 0) tab[0] = w_id;
                    if (item0 + n_items == nq) tab[1] = w_id;
                }
                FAR = true;
                have = true;
            } else {
                if (band_u >= n_band) break;
                unit = band_u;
                band_u += wpg;
                have = true;
            }
        }
        if (!have) break;
        // the previous piece's last LDS reads are done in every wave before its buffers are refilled
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();

        // ---- this wave's 32 keys and the query range of the piece.  Item i of the piece is query tile
        // i % n_qt (64 rows from q_lo on) of query head i / n_qt.
        int j, lo, hi, q_lo, q_hi, fidx = 0;
        int hi2 = 1 << 29;  // HW: last query row of the head with the LARGEST window that sees the key as a neighbour
        bool valid;
        if (FAR) {
            q_lo = fq0;
            q_hi = far_last_query(fl, ft * BK, idx, p, dend, BK);
            fidx = ft * BK + 32 * kbw + kj;
            valid = fidx < fl.NF;
            j = valid ? far_pos(fl, fidx, idx, p.L) : 0;
            lo = j + p.n;
            hi = q_hi - 1;
            if constexpr (DOCS) hi = min(hi, dend[j] - 1);
        } else {
            int j0 = unit * BK;
            j = j0 + 32 * kbw + kj;
            valid = j < p.L;
            q_lo = j0;
            q_hi = min(p.L, j0 + BK + p.n - 1);
            lo = j;
            hi = min(j + p.n - 1, p.L - 1);
            if constexpr (HW) {
                const int jj = valid ? j : 0;
                if (!(jj < p.a || prefix[jj + 1] != prefix[jj])) hi2 = jj + p.n - 1;
            }
            if (!valid) j = 0;
            if constexpr (DOCS) hi = min(hi, dend[j] - 1);
            item0 = 0;
            n_qt = (q_hi - q_lo + BQ - 1) / BQ;
            n_items = G * n_qt;
        }
        if (!valid) {
            lo = kIntMax;
            hi = -1;
        }
        // visibility of query row i for this lane's key: lo <= i <= hi, tested with one comparison as
        // (unsigned)(i - lo) <= hi - lo; an empty range (hi < lo) becomes lo = max int, span 0
        const int lo_m = hi >= lo ? lo : kIntMax;
        const uint32_t span_m = hi >= lo ? (uint32_t)(hi - lo) : 0u;
        // wave-uniform bounds of the keys' query ranges, in scalar registers so that the per-block
        // decisions below are scalar branches
        const int lo_max = __builtin_amdgcn_readfirstlane(wave_max_i(lo));
        const int hi_min = __builtin_amdgcn_readfirstlane(wave_min_i(hi));
        const int hi2_min = HW ? __builtin_amdgcn_readfirstlane(wave_min_i(hi2)) : 0;

        // resident B operand: K rows for the P-wave, V rows for the dS-wave
        bf16x8 breg[KSTEPS];
        {
            const uint16_t *brow = (role == 0 ? K : V) + (kvrow0 + j) * D;
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks)
                breg[ks] = as_bf16x8(*reinterpret_cast<const u32x4 *>(brow + ks * 16 + 8 * hh));
        }
        f32x16 acc[DB];  // dV^T (P-wave) or dK^T (dS-wave) of the wave's keys
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[db][i] = 0.f;

        // The piece as a sequence of steps; in every step a wave works on one block of 32 query rows.
        // Far piece: block s of its tiles in step s.  Band unit: a key block of 32 keys needs only NBK
        // of the nbh blocks of a head (the queries j <= i < j+n of its keys), key block kb the blocks
        // kb .. kb+NBK-1; all waves walk through a head's blocks together, but the last ov = nbh-NBK
        // steps of a head are merged with the first ov steps of the next head: in merged step b the
        // key blocks kb > b finish the old head (block NBK+b, which the others cannot see) while the
        // key blocks kb <= b start the new one (block b, which the others cannot see either: its
        // queries come before their keys).  A head then costs NBK steps instead of nbh.
        const int n_tiles = n_items;
        const int nbh = FAR ? BPT * n_tiles : BPT * n_qt;        // blocks per "head" (a far piece is one run)
        const int NBK = (p.n + 30) / 32 + 1;
        // steps from one head's start to the next's: at least NBK; at most KW-1 merged steps;
        // and more than half a head, so that a head's tail only overlaps the head that follows it and
        // the ring of NBUF tiles always holds what two consecutive steps need
        int st_P = NBK > nbh / 2 + 1 ? NBK : nbh / 2 + 1;
        st_P = st_P > nbh - (KW - 1) ? st_P : nbh - (KW - 1);
        // a tile is requested one barrier before the barrier that waits for it, so the tiles of three
        // consecutive steps must fit the ring: with one block per tile a head's first step needs two
        // plain steps behind it
        if (BPT == 1 && st_P < 3) st_P = 3;
        if (FAR || st_P > nbh) st_P = nbh;
        const int st_ov = nbh - st_P;                            // 0 .. KW-1
        const int st_G = FAR ? 1 : G;
        const int n_blocks = (st_G - 1) * st_P + nbh;            // steps of the piece
        const int tiles_per_head = FAR ? 0 : n_qt;

        // tile tt -> LDS buffer tt%4: wave w fills rows (LOADS*w + u)*RPL .. +RPL-1 with one wave-wide
        // direct load per tensor; a lane owns physical chunk lane%CH of its row and fetches the
        // logical chunk the permutation maps there.  Rows past the sequence end are clamped (they are
        // masked by the [lo, hi] test: hi <= L-1).  Tiles are issued in order; (iss_g, iss_qt) is the
        // (head, query tile) of the next one.
        int iss_tt = 0, iss_g = item0 / n_qt, iss_qt = item0 % n_qt;
        auto issue_tile = [&]() {
            const int buf = iss_tt % NBUF;
            const long hrow0 = ((long)b * p.Hq + kv * G + iss_g) * (long)p.L;
            const int qbase = q_lo + iss_qt * BQ;
            static_for<LOADS>([&](auto U) {
                constexpr int u = U;
                const int r = (LOADS * wave + u) * RPL + my_sub;
                // (uniform base of the head) + 32-bit byte offset; the loads go through inline assembly
                // so that the compiler does not make every LDS read wait for all of them
                const uint32_t off = (uint32_t)min(qbase + r, p.L - 1) * (uint32_t)(D * 2) + swz_chunk<kSwzBoth, D>(my_pc, r) * 16;
                const int wave_off = (LOADS * wave + u) * RPL * D;
                dma_to_lds_16(Q + hrow0 * D, off, lds_addr(&Qs[buf][wave_off]));
                dma_to_lds_16(dO + hrow0 * D, off, lds_addr(&dOs[buf][wave_off]));
            });
            // the BQ + BQ row values (LSE*log2e, -D) in groups of sixteen, dealt to the waves so that every
            // wave issues the same number of loads per tile: group g holds rows 16 (g % (BQ/16)) .. +15
            // of LSE*log2e (g < BQ/16) or of -D
#pragma unroll
            for (int v = 0; v < RVL; ++v) {
                constexpr int GPT = BQ / 16;  // groups per tensor
                const int g = wave * RVL + v, part = g % GPT;
                const float *src = (g < GPT ? LSE2 : Dws) + hrow0;
                float *dst = g < GPT ? &lse_s[buf][16 * part] : &d_s[buf][16 * part];
                if (lane < 16) dma_to_lds_4(src, (uint32_t)min(qbase + 16 * part + lane, p.L - 1) * 4u, lds_addr(dst));
            }
            ++iss_tt;
            if (++iss_qt == n_qt) {
                iss_qt = 0;
                ++iss_g;
            }
        };
        // wait until at most the loads of the n_out newest tiles are still in flight (loads complete in
        // the order they were issued; every wave issues 2*LOADS + 1 loads per tile)
        auto wait_tiles = [&](int n_out) __attribute__((always_inline)) {
            constexpr int LW = 2 * LOADS + RVL;
            static_assert(LW == 3 || LW == 5 || LW == 6, "wait counts below are written for 3, 5 or 6 loads per wave and tile");
            if (n_out <= 0) {
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            } else if (n_out == 1) {
                if constexpr (LW == 3) asm volatile("s_waitcnt vmcnt(3)" ::: "memory");
                else if constexpr (LW == 5) asm volatile("s_waitcnt vmcnt(5)" ::: "memory");
                else asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
            } else if (n_out == 2) {
                if constexpr (LW == 3) asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
                else if constexpr (LW == 5) asm volatile("s_waitcnt vmcnt(10)" ::: "memory");
                else asm volatile("s_waitcnt vmcnt(12)" ::: "memory");
            } else {
                if constexpr (LW == 3) asm volatile("s_waitcnt vmcnt(9)" ::: "memory");
                else if constexpr (LW == 5) asm volatile("s_waitcnt vmcnt(15)" ::: "memory");
                else asm volatile("s_waitcnt vmcnt(18)" ::: "memory");
            }
        };

        // ---- per-step pieces.  What a wave needs to know about a step (the LDS offset of its block, the
        // block's first query row, whether the block needs the mask test, which tiles the step and its
        // successor touch) is computed for 64 steps at a time, one step per lane, and fetched with
        // three v_readlane per step: scalar bookkeeping inside the loop costs issue slots that the
        // matrix instructions need.  Tiles are numbered in load order (head-major).
        struct Blk {
            int dlt;         // HW: how much shorter the window of the block's head is than p.n
            int r0, ps, rv;  // first query row; parity of the step (P exchange slot); float offset of the row values
            uint32_t off;    // byte offset of the block's first row from the start of the ring
            bool full;       // every (query, key) pair of the block is visible: no mask test needed
        };
        const int q0_tile = item0 % n_qt;
        // step s: the tile and block this wave (key block kbw) works on, lowest / highest tile of any wave
        int step_head = 0;  // head (within the group) of the block step_of was last asked about (band units)
        auto step_of = [&](int s, int &tile, int &blk, int &lo_t, int &hi_t) __attribute__((always_inline)) {
            const int g = s / st_P, b = s - g * st_P;
            const int base_t = g * tiles_per_head;
            const bool mg = g > 0 && b < st_ov;
            const int own = base_t + b / BPT, old = base_t - tiles_per_head + (b + st_P) / BPT;
            const bool prev = mg && (kbw > b || g == st_G);
            step_head = prev ? g - 1 : g;
            tile = prev ? old : own;
            blk = prev ? b + st_P : b;
            lo_t = mg ? old : own;
            hi_t = (mg && g == st_G) ? old : own;
        };
        uint32_t sch_off = 0;
        int sch_r0 = 0, sch_t = 0, sch_d = 0;
        auto fill_schedule = [&](int first) __attribute__((always_inline)) {
            const int sidx = first + lane;
            int tile, blk, lo_t, hi_t, tile_n, blk_n, lo_n, hi_n;
            step_of(sidx, tile, blk, lo_t, hi_t);
            int dl = 0;
            if constexpr (HW) {
                // the head's delta: the table is indexed with wave-uniform numbers only
                const int hd = step_head;
                for (int g = 0; g < G; ++g) {
                    const int sd = head_delta(hw, kv * G + g);
                    dl = (!FAR && hd == g) ? sd : dl;
                }
            }
            step_of(sidx + 1, tile_n, blk_n, lo_n, hi_n);
            if (sidx + 1 >= n_blocks) hi_n = n_tiles - 1;
            const int buf = tile % NBUF, qb = blk % BPT;
            const int r0 = q_lo + ((q0_tile + blk / BPT) % n_qt) * BQ + 32 * qb;
            bool full = (r0 >= lo_max) && (r0 + 31 <= hi_min);
            if constexpr (HW) full = full && (r0 + 31 + dl <= hi2_min);
            sch_d = dl;
            sch_off = (uint32_t)buf * (TILE * 2) + (uint32_t)qb * (32 * D * 2);
            sch_r0 = r0 | (buf << 2) | (qb << 1) | (full ? 1 : 0);  // r0 is a multiple of 32
            sch_t = (lo_t << 2) | max(0, min(hi_n - lo_t, 3));
        };
        int st_n = -1;                            // number of the step handed out last
        int lo_cur = 0, hi_next = 0;              // lowest tile of that step; highest tile of the step after it
        int hi_landed = 0;                        // highest tile this wave has waited for
        auto next_block = [&]() __attribute__((always_inline)) {
            ++st_n;
            const int l = st_n & 63;
            if (l == 0) fill_schedule(st_n);
            Blk k;
            k.off = __builtin_amdgcn_readlane(sch_off, l);
            const int r0p = __builtin_amdgcn_readlane(sch_r0, l);
            const int tp = __builtin_amdgcn_readlane(sch_t, l);
            k.r0 = r0p & ~31;
            k.full = r0p & 1;
            k.rv = ((r0p >> 2) & 3) * BQ + ((r0p >> 1) & 1) * 32;
            k.ps = st_n & 1;
            k.dlt = HW ? __builtin_amdgcn_readlane(sch_d, l) : 0;
            lo_cur = tp >> 2;
            hi_next = lo_cur + (tp & 3);
            return k;
        };
        // fragment reads by precomputed address: one vector instruction per read forms the address
        auto rd_row = [&](uint32_t rbase, int ks) __attribute__((always_inline)) {
            return lds_read_b128_at(rbase ^ (32u * ks));
        };
        // rows 16*stp .. +15 of the block, columns 32*db .. +31, transposed.  For d = 128 the second
        // 64-bit read is the first with chunk bit 0 flipped, four rows on.
        auto rd_tr = [&](uint32_t boff, int stp, int db) __attribute__((always_inline)) {
            const uint32_t first = boff + ktr0[db];
            const uint32_t second = D == 128 ? (first ^ 16u) + 4u * D * 2u : boff + ktr1[db];
            return lds_read_tr_at2(first + stp * 16 * D * 2, second + stp * 16 * D * 2);
        };
        auto read_rows = [&](const Blk &k, bf16x8 (&afr)[KSTEPS]) __attribute__((always_inline)) {
            const uint32_t rbase = t1_base + k.off;
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks) afr[ks] = rd_row(rbase, ks);
        };
        auto read_transposed = [&](const Blk &k, bf16x8 (&tfr)[2][DB]) __attribute__((always_inline)) {
#pragma unroll
            for (int stp = 0; stp < 2; ++stp)
#pragma unroll
                for (int db = 0; db < DB; ++db) tfr[stp][db] = rd_tr(k.off, stp, db);
        };
        // The two contractions of one pipeline step, with the LDS reads of the later one placed
        // between the MFMA groups of the earlier one: a fragment is requested four MFMAs (128 cycles)
        // before its use, and at most 32 fragment registers are live.  The scheduling fences keep the
        // compiler from hoisting all reads to the top (which would spill).
        auto zero = [&](f32x16 &x) __attribute__((always_inline)) {
#pragma unroll
            for (int i = 0; i < 16; ++i) x[i] = 0.f;
        };
        // acc += T2^T(cur) x_b(cur), then x = T1(nxt) B        (P-wave order)
        auto gemm2_then_gemm1 = [&](const Blk &cur, const bf16x8 (&xb)[2], const Blk &nxt, f32x16 &x) __attribute__((always_inline)) {
            const uint32_t rbase = t1_base + nxt.off;
            bf16x8 t0[DB], t1[DB], a0[KSTEPS / 2], a1[KSTEPS / 2];
#pragma unroll
            for (int db = 0; db < DB; ++db) t0[db] = rd_tr(cur.off, 0, db);
#pragma unroll
            for (int db = 0; db < DB; ++db) t1[db] = rd_tr(cur.off, 1, db);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int db = 0; db < DB; ++db) acc[db] = mfma_bf16(t0[db], xb[0], acc[db]);
#pragma unroll
            for (int ks = 0; ks < KSTEPS / 2; ++ks) a0[ks] = rd_row(rbase, ks);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int db = 0; db < DB; ++db) acc[db] = mfma_bf16(t1[db], xb[1], acc[db]);
#pragma unroll
            for (int ks = 0; ks < KSTEPS / 2; ++ks) a1[ks] = rd_row(rbase, ks + KSTEPS / 2);
            __builtin_amdgcn_sched_barrier(0);
            zero(x);
#pragma unroll
            for (int ks = 0; ks < KSTEPS / 2; ++ks) x = mfma_bf16(a0[ks], breg[ks], x);
#pragma unroll
            for (int ks = 0; ks < KSTEPS / 2; ++ks) x = mfma_bf16(a1[ks], breg[ks + KSTEPS / 2], x);
            __builtin_amdgcn_sched_barrier(0);
        };
        // xn += T1(nxt) B (fragments a0, a1 already requested; xn comes in holding -D of the block's rows,
        // so that it leaves as dP - D), then acc += T2^T(cur) x_b(cur)   (dS-wave order)
        auto gemm1_then_gemm2 = [&](const Blk &nxt, const bf16x8 (&a0)[KSTEPS / 2], const bf16x8 (&a1)[KSTEPS / 2],
                                    f32x16 &xn, const Blk &cur, const bf16x8 (&xb)[2]) __attribute__((always_inline)) {
            bf16x8 t0[DB], t1[DB];
#pragma unroll
            for (int ks = 0; ks < KSTEPS / 2; ++ks) xn = mfma_bf16(a0[ks], breg[ks], xn);
#pragma unroll
            for (int db = 0; db < DB; ++db) t0[db] = rd_tr(cur.off, 0, db);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int ks = 0; ks < KSTEPS / 2; ++ks) xn = mfma_bf16(a1[ks], breg[ks + KSTEPS / 2], xn);
#pragma unroll
            for (int db = 0; db < DB; ++db) t1[db] = rd_tr(cur.off, 1, db);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int db = 0; db < DB; ++db) acc[db] = mfma_bf16(t0[db], xb[0], acc[db]);
#pragma unroll
            for (int db = 0; db < DB; ++db) acc[db] = mfma_bf16(t1[db], xb[1], acc[db]);
            __builtin_amdgcn_sched_barrier(0);
        };
        auto read_rows_halves = [&](const Blk &k, bf16x8 (&a0)[KSTEPS / 2], bf16x8 (&a1)[KSTEPS / 2]) __attribute__((always_inline)) {
            const uint32_t rbase = t1_base + k.off;
#pragma unroll
            for (int ks = 0; ks < KSTEPS / 2; ++ks) {
                a0[ks] = rd_row(rbase, ks);
                a1[ks] = rd_row(rbase, ks + KSTEPS / 2);
            }
        };
        auto gemm1 = [&](const bf16x8 (&afr)[KSTEPS], f32x16 &x) {  // x += T1 B
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks) x = mfma_bf16(afr[ks], breg[ks], x);
        };
        auto gemm2 = [&](const bf16x8 (&tfr)[2][DB], const bf16x8 (&xb)[2]) {
#pragma unroll
            for (int stp = 0; stp < 2; ++stp)
#pragma unroll
                for (int db = 0; db < DB; ++db) acc[db] = mfma_bf16(tfr[stp][db], xb[stp], acc[db]);
        };
        // the sixteen per-row values (LSE*log2e or D) of the block's rows held by this lane
        auto read_rowvals = [&](const Blk &k, f32x16 &rv) __attribute__((always_inline)) {
            const float *rowval = (role == 0 ? &lse_s[0][0] : &d_s[0][0]) + k.rv;
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const int base = 16 * half + 8 * hh;
                const float4 l0 = *reinterpret_cast<const float4 *>(rowval + base);
                const float4 l1 = *reinterpret_cast<const float4 *>(rowval + base + 4);
                rv[8 * half + 0] = l0.x, rv[8 * half + 1] = l0.y, rv[8 * half + 2] = l0.z, rv[8 * half + 3] = l0.w;
                rv[8 * half + 4] = l1.x, rv[8 * half + 5] = l1.y, rv[8 * half + 6] = l1.z, rv[8 * half + 7] = l1.w;
            }
        };
        // P-wave: P = exp2(S*scale*log2e - LSE*log2e), zero where masked, rounded to bf16 (the form its
        // own second contraction needs) and handed to the dS-wave in that form
        auto softmax_and_publish = [&](const Blk &k, f32x16 &x, bf16x8 (&xb)[2]) __attribute__((always_inline)) {
            f32x16 ls;
            read_rowvals(k, ls);
#pragma unroll
            for (int i = 0; i < 16; ++i) x[i] = __builtin_amdgcn_exp2f(fmaf(x[i], sl2, -ls[i]));
            if (!k.full) {
                const int rel = k.r0 + 8 * hh - lo_m;  // row of element i, relative to lo: rel + 16*(i/8) + i%8
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    bool vis = (uint32_t)(rel + (16 * (i >> 3) + (i & 7))) <= span_m;
                    if constexpr (HW) vis = vis && (k.r0 + 16 * (i >> 3) + 8 * hh + (i & 7) + k.dlt <= hi2);
                    x[i] = vis ? x[i] : 0.f;
                }
            }
            xb[0] = pack_bf16x8(x, 0);
            xb[1] = pack_bf16x8(x, 8);
            *reinterpret_cast<bf16x8 *>(&Pex[kbw][k.ps][0][lane * 8]) = xb[0];
            *reinterpret_cast<bf16x8 *>(&Pex[kbw][k.ps][1][lane * 8]) = xb[1];
        };
        // dS-wave: dS = P (dP - D); x holds dP - D (the accumulator started from -D), the result is
        // rounded to bf16 in the form the second contraction needs
        auto fetch_p_and_form_ds = [&](const Blk &k, const f32x16 &x, bf16x8 (&xb)[2]) __attribute__((always_inline)) {
            f32x16 ds;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const u32x4 pw = *reinterpret_cast<const u32x4 *>(&Pex[kbw][k.ps][h][lane * 8]);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float p_lo = __uint_as_float(pw[e] << 16), p_hi = __uint_as_float(pw[e] & 0xFFFF0000u);
                    ds[8 * h + 2 * e] = p_lo * x[8 * h + 2 * e];
                    ds[8 * h + 2 * e + 1] = p_hi * x[8 * h + 2 * e + 1];
                }
            }
            xb[0] = pack_bf16x8(ds, 0);
            xb[1] = pack_bf16x8(ds, 8);
        };
        // Barrier after the first contraction (and publication of P) of the step handed out last.  The
        // interval after it reads the blocks of that step (second contraction) and of the next one
        // (first contraction): every wave first waits for its share of the tiles the next step needs,
        // and after the barrier the buffers of the tiles below the lowest one still in use are refilled.
        auto block_barrier = [&]() __attribute__((always_inline)) {
            if (hi_next != hi_landed) {
                wait_tiles(iss_tt - 1 - hi_next);
                hi_landed = hi_next;
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();
            while (iss_tt < n_tiles && iss_tt - NBUF < lo_cur) issue_tile();
        };

        // start-up: the ring is filled, step 0 needs tile 0 only
        while (iss_tt < n_tiles && iss_tt < NBUF) issue_tile();
        wait_tiles(iss_tt - 1);
        __builtin_amdgcn_s_barrier();

        // ---- software pipeline over the steps.  Between the barriers of steps s and s+1 a wave runs
        // the second contraction of its block of step s and the first of its block of step s+1, with
        // the LDS operands of both requested up front; the P-wave puts its softmax arithmetic last (it
        // overlaps the other wave's MFMAs on the same SIMD), the dS-wave puts its arithmetic first.
        // A wave also runs the blocks of a far piece or of its head in which its keys see no query
        // (their P is zero through the mask): the waves meet at a barrier per step anyway, and a loop
        // body without alternatives keeps the accumulators in place.
        auto pipeline = [&](auto ROLE) {
            constexpr int R = ROLE;
            f32x16 x, y;  // P-wave: scores (x only); dS-wave: dP - D of the current and of the next block, in turn
            bf16x8 xb[2];
            Blk cur = next_block();
            {
                bf16x8 afr[KSTEPS];
                read_rows(cur, afr);
                if constexpr (R == 0)
                    zero(x);
                else
                    read_rowvals(cur, x);
                gemm1(afr, x);
                if constexpr (R == 0) softmax_and_publish(cur, x, xb);
            }
            block_barrier();
            // one step of the dS-wave: xc holds dP - D of block cur, xn receives that of block nxt
            auto ds_step = [&](f32x16 &xc, f32x16 &xn) __attribute__((always_inline)) {
                const Blk nxt = next_block();
                bf16x8 a0[KSTEPS / 2], a1[KSTEPS / 2];
                read_rows_halves(nxt, a0, a1);  // in flight during the dS arithmetic
                read_rowvals(nxt, xn);
                fetch_p_and_form_ds(cur, xc, xb);
                __builtin_amdgcn_sched_barrier(0);
                gemm1_then_gemm2(nxt, a0, a1, xn, cur, xb);
                block_barrier();
                cur = nxt;
            };
            if constexpr (R == 0) {
                for (int gb = 0; gb + 1 < n_blocks; ++gb) {
                    const Blk nxt = next_block();
                    gemm2_then_gemm1(cur, xb, nxt, x);
                    softmax_and_publish(nxt, x, xb);
                    block_barrier();
                    cur = nxt;
                }
            } else {
                // two steps per trip, so that the two accumulators swap roles without copies
                int gb = 0;
                for (; gb + 2 < n_blocks; gb += 2) {
                    ds_step(x, y);
                    ds_step(y, x);
                }
                if (gb + 1 < n_blocks) {
                    ds_step(x, y);
                    x = y;
                }
            }
            {
                bf16x8 tfr[2][DB];
                read_transposed(cur, tfr);
                if constexpr (R == 1) fetch_p_and_form_ds(cur, x, xb);
                gemm2(tfr, xb);
            }
        };
        if (role == 0)
            pipeline(IntC<0>{});
        else
            pipeline(IntC<1>{});

        // ---- epilogue: the P-wave owns dV, the dS-wave owns dK (times scale).  A far piece writes its
        // partial (slot w + ft, row = entry within the list tile); a band unit finishes keys that are
        // not on the far list and writes the band partial (one row per list entry, after the slots)
        // of those that are.
        const float oscale = role == 0 ? 1.f : p.scale;
        float *farX = role == 0 ? farV : farK;
        long part_row = (long)(w_id + ft) * BK + 32 * kbw + kj;
        bool to_partial = FAR;
        if (!FAR && valid) {
            const int f = far_index(fl, prefix, j);
            if (f >= 0 && far_first_query(fl, f, idx, p, BK) < far_last_query(fl, f, idx, p, dend, BK)) {
                to_partial = true;
                part_row = (long)fg.NP * BK + f;
            }
        }
        if (valid) {
            if (to_partial) {
                const long prow = ((long)bkv * fg.rows + part_row) * D;
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int i4 = 0; i4 < 4; ++i4) {
                        const int col = db * 32 + 8 * i4 + 4 * hh;
                        const float4 a = {acc[db][4 * i4] * oscale, acc[db][4 * i4 + 1] * oscale,
                                          acc[db][4 * i4 + 2] * oscale, acc[db][4 * i4 + 3] * oscale};
                        *reinterpret_cast<float4 *>(farX + prow + col) = a;
                    }
            } else {
                uint16_t *orow = (role == 0 ? dV : dK) + (kvrow0 + j) * D;
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int i4 = 0; i4 < 4; ++i4) {
                        const int col = db * 32 + 8 * i4 + 4 * hh;
                        *reinterpret_cast<uint2 *>(orow + col) =
                            pack_bf16x4(acc[db][4 * i4] * oscale, acc[db][4 * i4 + 1] * oscale,
                                        acc[db][4 * i4 + 2] * oscale, acc[db][4 * i4 + 3] * oscale);
                    }
            }
        }
    }  // pieces
}

// Sum of the partials of every far-list key (the far pieces of its list tile in ascending workgroup
// order, then the band partial), rounded once to bf16.  One thread per (key, 4 consecutive columns).
template <int D>
__global__ __launch_bounds__(256) void dkv_combine_kernel(sepattn_params p, const int32_t *__restrict__ sep_idx,
                                                          const int32_t *__restrict__ sep_prefix,
                                                          const int32_t *__restrict__ doc_end,
                                                          uint16_t *__restrict__ dK, uint16_t *__restrict__ dV,
                                                          const float *__restrict__ farK,
                                                          const float *__restrict__ farV,
                                                          const int32_t *__restrict__ piece_tab, int wpg, int kw) {
    constexpr int TPR = D / 4;  // threads per row
    const int bkv = blockIdx.y, kv = bkv % p.Hkv, b = bkv / p.Hkv;
    const int32_t *prefix = sep_prefix + (long)b * (p.L + 1);
    const int32_t *idx = sep_idx + (long)b * p.cap;
    const FarGeom fg = far_geom(p, wpg, kw);
    const FarList fl = far_list(p, prefix);
    const int f = (blockIdx.x * 256 + threadIdx.x) / TPR, col = ((blockIdx.x * 256 + threadIdx.x) % TPR) * 4;
    if (f >= fl.NF) return;
    const int lt = fg.bk;  // entries per list tile
    const int A = far_first_query(fl, f, idx, p, lt);
    // no far piece for this list tile: the band unit has written the row
    if (A >= far_last_query(fl, f, idx, p, doc_end ? doc_end + (long)b * p.L : nullptr, lt)) return;
    const int j = far_pos(fl, f, idx, p.L);
    const int ft = f / lt;
    const int32_t *tab = piece_tab + ((long)bkv * fg.NFTcap + ft) * 2;
    // the clamps keep a table that the far pass did not write (it always does) from faulting
    const int w0 = min(max(tab[0], 0), wpg - 1), w1 = min(max(tab[1], w0), wpg - 1);
    const long base = (long)bkv * fg.rows;
    float4 sk = {0.f, 0.f, 0.f, 0.f}, sv = {0.f, 0.f, 0.f, 0.f};
    // the band partial and eight pieces at a time (clamped slots) are requested together, so that a
    // list tile with up to eight pieces costs one memory round trip; the sum runs in slot order
    constexpr int NB = 8;
    const long brow = (base + (long)fg.NP * lt + f) * D + col;
    const float4 bk = *reinterpret_cast<const float4 *>(farK + brow);
    const float4 bv = *reinterpret_cast<const float4 *>(farV + brow);
    for (int w = w0; w <= w1; w += NB) {
        float4 pk[NB], pv[NB];
#pragma unroll
        for (int c = 0; c < NB; ++c) {
            const int ww = min(w + c, w1);
            const long prow = (base + (long)(ww + ft) * lt + (f - ft * lt)) * D + col;
            pk[c] = *reinterpret_cast<const float4 *>(farK + prow);
            pv[c] = *reinterpret_cast<const float4 *>(farV + prow);
        }
#pragma unroll
        for (int c = 0; c < NB; ++c) {
            if (w + c <= w1) {
                sk.x += pk[c].x, sk.y += pk[c].y, sk.z += pk[c].z, sk.w += pk[c].w;
                sv.x += pv[c].x, sv.y += pv[c].y, sv.z += pv[c].z, sv.w += pv[c].w;
            }
        }
    }
    sk.x += bk.x, sk.y += bk.y, sk.z += bk.z, sk.w += bk.w;
    sv.x += bv.x, sv.y += bv.y, sv.z += bv.z, sv.w += bv.w;
    const long orow = (((long)b * p.Hkv + kv) * (long)p.L + j) * D + col;
    *reinterpret_cast<uint2 *>(dK + orow) = pack_bf16x4(sk.x, sk.y, sk.z, sk.w);
    *reinterpret_cast<uint2 *>(dV + orow) = pack_bf16x4(sv.x, sv.y, sv.z, sv.w);
}

template <int D, int KW>
void launch_dkv_shape(const sepattn_params &p, const HeadWin &hw, bool headwise, const uint16_t *Q, const uint16_t *K,
                      const uint16_t *V, const float *lse2, const uint16_t *dO, const float *Dws, const int32_t *sep_idx,
                      const int32_t *sep_prefix, const int32_t *doc_end, uint16_t *dK, uint16_t *dV, float *farK,
                      float *farV, int32_t *piece_tab, int wpg, hipStream_t st) {
    const int band_grid = (p.L + 32 * KW - 1) / (32 * KW);
    const dim3 grid((unsigned)((long)wpg * p.B * p.Hkv)), block(128 * KW);
    if (doc_end)
        hipLaunchKernelGGL((dkv_kernel<D, true, false, KW>), grid, block, 0, st, p, Q, K, V, lse2, dO, Dws, sep_idx,
                           sep_prefix, doc_end, dK, dV, farK, farV, piece_tab, wpg, band_grid, hw);
    else if (headwise)
        hipLaunchKernelGGL((dkv_kernel<D, false, true, KW>), grid, block, 0, st, p, Q, K, V, lse2, dO, Dws, sep_idx,
                           sep_prefix, doc_end, dK, dV, farK, farV, piece_tab, wpg, band_grid, hw);
    else
        hipLaunchKernelGGL((dkv_kernel<D, false, false, KW>), grid, block, 0, st, p, Q, K, V, lse2, dO, Dws, sep_idx,
                           sep_prefix, doc_end, dK, dV, farK, farV, piece_tab, wpg, band_grid, hw);
}

template <int D>
int launch_dkv(const sepattn_params &p, const HeadWin &hw, bool headwise, const uint16_t *Q, const uint16_t *K, const uint16_t *V,
               const float *lse2, const uint16_t *dO, const float *Dws, const int32_t *sep_idx,
               const int32_t *sep_prefix, const int32_t *doc_end, uint16_t *dK, uint16_t *dV, float *farK,
               float *farV, int32_t *piece_tab, hipStream_t st) {
    const int kw = dkv_key_blocks(p, doc_end != nullptr);
    const int wpg = dkv_workgroups_per_head(p, kw);
    const FarGeom fg = far_geom(p, wpg, kw);
    if ((long)wpg * p.B * p.Hkv > 0x7FFFFFFFL) return SEPATTN_ERR_SHAPE;
    {
        ProfScope prof(SEPATTN_K_BWD_DKV, st);
        // the eight-wave shape exists for d = 128 only (dkv_key_blocks)
        if (D == 128 && kw == 4)
            launch_dkv_shape<128, 4>(p, hw, headwise, Q, K, V, lse2, dO, Dws, sep_idx, sep_prefix, doc_end, dK, dV, farK, farV, piece_tab, wpg, st);
        else
            launch_dkv_shape<D, 2>(p, hw, headwise, Q, K, V, lse2, dO, Dws, sep_idx, sep_prefix, doc_end, dK, dV, farK, farV, piece_tab, wpg, st);
    }
    if (hipGetLastError() != hipSuccess) return SEPATTN_ERR_HIP;
    ProfScope prof(SEPATTN_K_BWD_COMBINE, st);
    const int rows_per_block = 256 / (D / 4);
    hipLaunchKernelGGL((dkv_combine_kernel<D>), dim3((fg.NFcap + rows_per_block - 1) / rows_per_block, p.B * p.Hkv),
                       dim3(256), 0, st, p, sep_idx, sep_prefix, doc_end, dK, dV, farK, farV, piece_tab, wpg, kw);
    return launch_status();
}

}  // namespace

int launch_dkv_bf16(const sepattn_params &p, const HeadWin &hw, const uint16_t *Q, const uint16_t *K, const uint16_t *V,
                    const float *lse2, const uint16_t *dO, const float *Dws, const int32_t *sep_idx,
                    const int32_t *sep_prefix, const int32_t *doc_end, uint16_t *dK, uint16_t *dV, float *farK,
                    float *farV, int32_t *piece_tab, hipStream_t st) {
    bool headwise = false;
    for (int h = 0; h < kMaxHeadwise; ++h) headwise = headwise || hw.delta[h] != 0;
    if (p.d == 64)
        return launch_dkv<64>(p, hw, headwise, Q, K, V, lse2, dO, Dws, sep_idx, sep_prefix, doc_end, dK, dV, farK, farV, piece_tab, st);
    return launch_dkv<128>(p, hw, headwise, Q, K, V, lse2, dO, Dws, sep_idx, sep_prefix, doc_end, dK, dV, farK, farV, piece_tab, st);
}

}  // namespace sepattn
