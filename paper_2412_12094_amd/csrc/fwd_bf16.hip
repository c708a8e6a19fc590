// SepAttention forward, bf16 MFMA (Eq. 1 with the mask of Eq. 2), flash-style with online softmax.
//
// A workgroup (NW = 8 waves, or 4 where two workgroups share a compute unit: see launch_fwd) owns
// TP = 32 NW / GP consecutive query positions of GP query heads that share one KV
// head (grouped-query attention: the heads are packed into the row dimension, so K/V tiles and the
// mask are shared).  Each wave owns 32 rows: one head, 32 positions.  The keys a tile can see are
// turned into ONE dense stream,
//     [ initial tokens j < min(a, bs) | separators in [min(a,bs), bs) | band keys bs .. i0+TP-1 ]
// with bs = max(0, i0-n+1) the first key of the first row's neighbour window (Sec. 3.1).  The first
// two parts are visible to every row of the tile (they are older than every window and are initial
// tokens / separators) and are gathered through the compacted separator index list; only band keys
// need the per-element test  j <= i and (i-j < n or j is an initial token or a separator).
//
// Schedule: every wave runs the same software pipeline over blocks of 32 keys; the score block of
// the next block, the output update of the previous one and the softmax of the current one are
// interleaved instruction by instruction (the matrix instructions execute while the vector
// instructions issued after them run), one workgroup barrier per tile.  K tiles, V tiles and the
// per-key visibility ranges live in 4 LDS stages each; tiles are filled by direct global->LDS loads
// (global_load_lds_dwordx4, no staging registers) issued two tiles ahead, unpadded with XOR-swizzled
// 16-byte chunks (see mfma_common.h).  V^T operands are read with ds_read_b64_tr_b16.  A wave drops
// the mask test on blocks every one of its rows sees in full.  The running maximum is only raised
// when it grows by more than 2^8 (all terms carry the same stale maximum, so the result is
// unchanged), which removes almost every rescale of the output accumulators.
#include "common.h"
#include "mfma_common.h"
#include "key_stream.h"


namespace sepattn {

namespace {

constexpr float kRescaleThreshold = 8.f;  // log2 units

// DOCS: packed documents (see make_stream_docs); doc_start / doc_end [B, L] give, per position, the
// first position of its document and one past its last.  Requires p.a == 0.
// NW: waves per workgroup (8 or 4); 2 waves per SIMD either way.
template <int D, int GP, bool DOCS, int NW>
__global__ __launch_bounds__(64 * NW, 2) void fwd_bf16_kernel(
    sepattn_params p, const uint16_t *__restrict__ Q, const uint16_t *__restrict__ K,
    const uint16_t *__restrict__ V, const int32_t *__restrict__ sep_idx,
    const int32_t *__restrict__ sep_prefix, const int32_t *__restrict__ doc_start,
    const int32_t *__restrict__ doc_end, uint16_t *__restrict__ O, float *__restrict__ LSE, int wpg, HeadWin hw) {
    constexpr int TP = 32 * NW / GP;  // query positions per workgroup
    constexpr int CH = D / 8;         // 16-byte chunks per row
    constexpr int RPL = 64 / CH;      // rows covered by one wave-wide 1 KB load
    // The tile loads are issued by the first NLW waves only (all of them when NW = 4).  With eight
    // waves, w and w+4 share a SIMD and the arbiter serves the older one (w) first: it reaches every
    // barrier long before its partner, so the load path costs nothing there, while on the younger wave
    // it would lengthen the critical path.
    constexpr int NLW = 4;
    constexpr int LOADS = kBN / (RPL * NLW);  // wave-wide loads per loading wave per tensor per tile
    constexpr int KSTEPS = D / 16;
    constexpr int DB = D / 32;
    // LDS stages of K, and of V and the visibility ranges: powers of two, so that a stage number is a
    // mask of the tile number (the kernel spends its time issuing instructions, scalar ones too)
    constexpr int KST = 4, VST = 4;
    constexpr int TILE = kBN * D;    // elements per LDS tile (unpadded, XOR-swizzled chunks)
    static_assert(LOADS >= 1 && LOADS * RPL * NLW == kBN, "tile must divide among the loading waves");

    __shared__ __attribute__((aligned(1024))) uint16_t Ks[KST][TILE];
    __shared__ __attribute__((aligned(1024))) uint16_t Vs[VST][TILE];
    __shared__ __attribute__((aligned(16))) int lo_s[VST][kBN];
    __shared__ __attribute__((aligned(16))) int hi_s[VST][kBN];
    // staging of one 32-column block of a wave's 32 output rows (see the epilogue)
    __shared__ __attribute__((aligned(16))) uint16_t ostage[NW][32 * 32];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keeps branches scalar
    const int qi = lane & 31, hh = lane >> 5;
    // A workgroup is persistent: it belongs to one (batch, KV head, head group) and walks through
    // several query tiles of it ("segments"), `wpg` workgroups per group sharing the tiles in zig-zag
    // order (round r: rank r*wpg + j for even r, r*wpg + wpg-1-j for odd r; rank 0 = the last tile,
    // the one with the longest key stream), so that with an even spread of separators every
    // workgroup gets about the same number of stream tiles.  Launch gaps, the tail of a grid of
    // unequal workgroups and most of the per-tile start-up cost are paid once per workgroup.
    const int G = p.Hq / p.Hkv, groups = G / GP;
    const int n_pos_tiles = (p.L + TP - 1) / TP;
    const TileGroup tg = xcd_tile_group(blockIdx.x, wpg, p.B * p.Hkv * groups);
    int y = tg.group;
    const int hg = y % groups;
    const int kv = (y / groups) % p.Hkv;
    const int b = y / (groups * p.Hkv);
    const int head = kv * G + hg * GP + (wave % GP);
    // head-wise windows: the stream is that of the largest window p.n; this head's window is shorter by
    // hdelta, which only enters the visibility test of band keys (hi was computed with p.n) and the
    // decision which blocks need no test
    const int hdelta = head_delta(hw, head);

    const int32_t *prefix = sep_prefix + (long)b * (p.L + 1);
    const int32_t *idx = sep_idx + (long)b * p.cap;
    const int32_t *dstart = DOCS ? doc_start + (long)b * p.L : nullptr;
    const int32_t *dend = DOCS ? doc_end + (long)b * p.L : nullptr;
    const uint16_t *Kh = K + ((long)b * p.Hkv + kv) * (long)p.L * D;
    const uint16_t *Vh = V + ((long)b * p.Hkv + kv) * (long)p.L * D;

    // state of the current segment (the lambdas below refer to it)
    int i0 = 0, pw = 0, iq = 0, iq_h = 0, n_tiles = 0;
    Stream st = {};
    FullBlocks fullb = {};
    bf16x8 qreg[KSTEPS];  // this wave's queries as B operands
    const float sl2 = p.scale * kLog2e_f;

    f32x16 oacc[DB];
    float m_run = -INFINITY, l_run = 0.f;  // m_run in the log2 domain (scores times scale*log2e)
    float alpha_pending = 1.f;             // rescale of oacc decided by a softmax, applied before the next output update

    // ---- tile loads: wave w fills rows (LOADS*w + u)*RPL .. +RPL-1 of a tile with one wave-wide
    // direct global->LDS load per tensor; a lane owns physical chunk lane%CH of its row.  Everything
    // about a load except the key position j is a per-lane constant, and the address is formed as
    // (uniform base) + 32-bit byte offset, so issuing a tile costs a handful of vector instructions.
    // Tiles come in three wave-uniform classes: all elements in the dense part (gather through the
    // index list, no visibility ranges needed: every block of such a tile is fully visible), all in
    // the band part (consecutive keys; ranges from the prefix counts), or mixed (general code).
    const int my_pc = lane % CH, my_sub = lane / CH;
    uint32_t kgo[LOADS], vgo[LOADS];  // byte offset of this lane's 16-byte piece inside a K / V row
    int rrow[LOADS];                  // row of the tile this lane helps to fill
#pragma unroll
    for (int u = 0; u < LOADS; ++u) {
        rrow[u] = (LOADS * wave + u) * RPL + my_sub;
        kgo[u] = swz_chunk<kSwzRow, D>(my_pc, rrow[u]) * 16;
        vgo[u] = swz_chunk<kSwzTr, D>(my_pc, rrow[u]) * 16;
    }
    const char *Kb = reinterpret_cast<const char *>(Kh), *Vb = reinterpret_cast<const char *>(Vh);
    auto tile_class = [&](const Stream &ss, int t) {
        const int k0 = t * kBN;
        return (k0 + kBN <= ss.n_dense) ? 0 : (k0 >= ss.n_dense ? 1 : 2);
    };
    // Index stage, one tile ahead of the rows: the list entry (dense part) and the two prefix counts
    // (band part) of each of the MR rows this wave fills, fetched by 3*MR lanes with one 4-byte
    // global->LDS load into the wave's own slot of a small ring; the wave reads them back one tile
    // step later.  All vector-memory traffic of the loop is thus global->LDS, issued through inline
    // assembly and waited for with explicit counts.
    // A tile is named by the stream of its segment (ss), its number in that stream (t) and its
    // number in the concatenation of all segments of this workgroup (g), which selects the LDS stage.
    constexpr int MR = LOADS * RPL;  // rows per wave and tile
    constexpr int MST = 4;           // ring stages
    __shared__ __attribute__((aligned(256))) int meta_s[MST][NLW][64];  // 3 * MR <= 48 entries per wave and stage
    const bool loader = NW == NLW || wave < NLW;
    const int m_part = lane / MR, m_row = wave * MR + lane % MR;  // lanes 0 .. 3*MR-1 are used
    auto issue_meta = [&](const Stream &ss, int t, int g) __attribute__((always_inline)) {
        const int k = t * kBN + m_row;
        const int e = min(max(ss.sep_lo - ss.n_init + k, 0), p.cap - 1);
        const int j = min(max(ss.bs - ss.n_dense + k, 0), p.L - 1);
        const int32_t *src = m_part == 0 ? idx + e : prefix + j + (m_part - 1);
        if constexpr (DOCS) src = m_part == 3 ? dend + j : src;  // fourth part: where the key's document ends
        if (lane < (DOCS ? 4 : 3) * MR) dma_to_lds_4_addr(src, lds_addr(&meta_s[(unsigned)g % MST][wave % NLW][0]));
    };
    // Rows of a tile in two steps, so that the index entries of the NEXT tile can be requested in
    // between: vector-memory results return in issue order, and with the order
    //   [entries of the next tile] [rows of this tile]   the wait for the entries does not wait for
    // the rows.  Past the last segment the stream is empty: its tiles are "loaded" too (row 0, never
    // visible), which keeps the count of outstanding loads exact in a loop body without alternatives.
    int jrow[LOADS], rawi[LOADS], raw0[LOADS], raw1[LOADS], raw2[DOCS ? LOADS : 1];
    auto read_entries = [&](int g) __attribute__((always_inline)) {
        const int *mt = &meta_s[(unsigned)g % MST][wave % NLW][0];
        static_for<LOADS>([&](auto U) {
            constexpr int u = U;
            rawi[u] = mt[u * RPL + my_sub];
            raw0[u] = mt[MR + u * RPL + my_sub];
            raw1[u] = mt[2 * MR + u * RPL + my_sub];
            if constexpr (DOCS) raw2[u] = mt[3 * MR + u * RPL + my_sub];
        });
    };
    // de: end of the document of the segment's first row; straddle: the segment's rows reach beyond it
    auto prepare_row = [&](const Stream &ss, int de, bool straddle, int t, int g, auto U) __attribute__((always_inline)) {
        constexpr int u = decltype(U)::value;
        const int vs_ = (unsigned)g % VST;
        const int r = rrow[u];
        const int k = t * kBN + r;
        // the clamp keeps a stale list tail (caller broke sep_count <= cap) from faulting
        const int jl = min(max(rawi[u], 0), p.L - 1);
        if (tile_class(ss, t) == 0 && !(DOCS && straddle)) {
            jrow[u] = k < ss.n_init ? k : jl;
        } else {
            const bool init = k < ss.n_init, dense = k < ss.n_dense, pad = k >= ss.n_total;
            const int jb = ss.bs + (k - ss.n_dense);
            const bool always = dense | (jb < p.a) | (raw1[u] != raw0[u]);
            int j = init ? k : (dense ? jl : jb);
            j = pad ? 0 : j;
            const int lo = pad ? kIntMax : j;
            int hi = always ? kIntMax : jb + p.n - 1;
            if constexpr (DOCS) hi = min(hi, (dense ? de : raw2[u]) - 1);
            hi = pad ? -1 : hi;
            if (my_pc == 0) {
                lo_s[vs_][r] = lo;
                hi_s[vs_][r] = hi;
            }
            jrow[u] = j;
        }
    };
    auto issue_row = [&](int g, auto U) __attribute__((always_inline)) {
        constexpr int u = decltype(U)::value;
        const uint32_t kst = lds_addr(&Ks[(unsigned)g % KST][0]), vst = lds_addr(&Vs[(unsigned)g % VST][0]);
        const uint32_t wave_off = (uint32_t)((LOADS * wave + u) * RPL * D * 2);  // bytes: 1 KB per wave-wide load
        const uint32_t row_off = (uint32_t)jrow[u] * (uint32_t)(D * 2);
        dma_to_lds_16(Kb, row_off + kgo[u], kst + wave_off);
        dma_to_lds_16(Vb, row_off + vgo[u], vst + wave_off);
    };

    // ---- segments of this workgroup and the load cursor.  The tiles of all segments form ONE stream
    // of loads: the cursor (segment lcur, tile l_t, global number l_g) always points at the next tile
    // whose rows are to be requested, two tiles ahead of the tile being multiplied, also across
    // segment borders, so that only the first segment of a workgroup pays the start-up latencies.
    struct Seg {
        Stream st;
        int n_tiles, i0, de;
    };
    auto open_segment = [&](int round) {
        Seg g;
        const int rank = round * wpg + ((round & 1) ? wpg - 1 - tg.rank : tg.rank);
        if (rank >= n_pos_tiles) {  // no more work: an empty stream of padding tiles
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
    // index entries of the tile after the cursor
    auto issue_meta_after_cursor = [&]() __attribute__((always_inline)) {
        if (l_t + 1 < lcur.n_tiles)
            issue_meta(lcur.st, l_t + 1, l_g + 1);
        else
            issue_meta(lnext.st, 0, l_g + 1);
    };
    // An MFMA phase issues [1 entry load][2*LOADS row loads], in this order; loads complete in order.
    //   entries_landed:    at most the row loads of the previous phase are still in flight
    //   wait_older_loads:  everything older than this phase's loads has landed
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

    const int a_row = pi_row(qi);

    // per-lane byte offsets of the operand fragments inside a tile (constant for the whole kernel)
    const uint32_t ks_base = lds_addr(&Ks[0][0]), vs_base = lds_addr(&Vs[0][0]);
    uint32_t koff[KSTEPS], voff[DB];
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) koff[ks] = lds_off_a<kSwzRow, D>(a_row, 2 * ks + hh);
#pragma unroll
    for (int db = 0; db < DB; ++db) voff[db] = lds_off_a_tr<kSwzTr, D>(db * 32, lane);

    // Workgroup barrier without the memory fence of __syncthreads(): the fence would make every wave
    // wait for ALL of its outstanding global->LDS loads (vmcnt(0)), i.e. for the tiles it has just
    // requested.  What a barrier has to publish here is waited for explicitly: the wave's LDS writes
    // (lgkmcnt) and the tile loads older than the previous tile step (vmcnt).
    auto wg_barrier = [&]() __attribute__((always_inline)) {
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };

    // ---- The pipeline.  Every wave runs the same instruction stream; one workgroup barrier per tile.
    // Work is cut into blocks of 32 keys (block c = 2*tile + half).  Tile step X, entered through the
    // barrier that publishes tile X, consists of two halves:
    //   half 1:  S(2X)   = K_X[ 0..31] Q^T      O^T += V_{X-1}[ 0..31]^T P(2X-2)^T    softmax of block 2X-1
    //   half 2:  S(2X+1) = K_X[32..63] Q^T      O^T += V_{X-1}[32..63]^T P(2X-1)^T    softmax of block 2X
    // In each half the matrix instructions (first the score block, then the output update) are
    // independent of the softmax arithmetic, which works on the scores of the block before; the two
    // are interleaved instruction by instruction: a matrix instruction is issued, then a few vector
    // instructions of the softmax (or of the load path), which execute while the matrix pipe is busy.
    // Operand fragments are requested from LDS LA matrix instructions ahead.  The loads of tile X+2
    // and the index entries of tile X+3 are issued during step X: the stages they overwrite held
    // tiles X-1 (K) and X-2 (V, visibility ranges), whose last readers finished before the barrier.
    f32x16 s_a, s_b;          // scores: first / second block of a tile
    bf16x8 p_a[2], p_b[2];    // probabilities (bf16, B-operand layout) of the first / second block
    constexpr int LA = D == 128 ? 6 : 4;
    constexpr int NQK = KSTEPS, NPV = 2 * DB;  // matrix instructions per half

    // one sixteenth of the softmax of a block: s -> pb, updating (m_run, l_run, alpha_pending)
    struct SmState {
        float m_loc, neg_m, psum;
        bool masked;
    } sm;
    auto softmax_chunk = [&](auto C, f32x16 &s, bf16x8 (&pb)[2], int tile, int gtile, int kb) __attribute__((always_inline)) {
        constexpr int c = decltype(C)::value;
        if constexpr (c == 0) {
            sm.masked = !block_is_full(fullb, tile * kBN + kb * 32);
            if (sm.masked) {
                const int vs_ = (unsigned)gtile % VST;
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    const int base = kb * 32 + 16 * half + 8 * hh;
                    const int4 lo0 = *reinterpret_cast<const int4 *>(&lo_s[vs_][base]);
                    const int4 lo1 = *reinterpret_cast<const int4 *>(&lo_s[vs_][base + 4]);
                    const int4 hi0 = *reinterpret_cast<const int4 *>(&hi_s[vs_][base]);
                    const int4 hi1 = *reinterpret_cast<const int4 *>(&hi_s[vs_][base + 4]);
                    const int los[8] = {lo0.x, lo0.y, lo0.z, lo0.w, lo1.x, lo1.y, lo1.z, lo1.w};
                    const int his[8] = {hi0.x, hi0.y, hi0.z, hi0.w, hi1.x, hi1.y, hi1.z, hi1.w};
#pragma unroll
                    for (int k = 0; k < 8; ++k) {
                        const bool vis = (los[k] <= iq) & (iq_h <= his[k]);
                        s[8 * half + k] = vis ? s[8 * half + k] : -INFINITY;
                    }
                }
            }
            sm.m_loc = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
        } else if constexpr (c < 4) {
            sm.m_loc = fmaxf(fmaxf(sm.m_loc, s[4 * c]), fmaxf(fmaxf(s[4 * c + 1], s[4 * c + 2]), s[4 * c + 3]));
        } else if constexpr (c == 4) {
            const float m_new = fmaxf(m_run, pair_max(sm.m_loc * sl2));
            const bool grow = m_new > m_run + kRescaleThreshold;
            if (__builtin_amdgcn_ballot_w64(grow) != 0ull) {
                const float alpha = grow ? __builtin_amdgcn_exp2f(m_run - m_new) : 1.f;
                m_run = grow ? m_new : m_run;
                l_run *= alpha;
                alpha_pending = alpha;
            }
            sm.neg_m = (m_run == -INFINITY) ? 0.f : -m_run;
            sm.psum = 0.f;
        } else if constexpr (c < 14) {
            // exponentials of two elements; their sum is taken one chunk later, when the results of
            // the transcendental unit have arrived
            if constexpr (c < 13) {
#pragma unroll
                for (int i = 2 * (c - 5); i < 2 * (c - 5) + 2; ++i) s[i] = __builtin_amdgcn_exp2f(fmaf(s[i], sl2, sm.neg_m));
            }
            if constexpr (c > 5) sm.psum += s[2 * (c - 6)] + s[2 * (c - 6) + 1];
            if constexpr (c == 13) pb[0] = pack_bf16x8(s, 0);
        } else if constexpr (c == 14) {
            pb[1] = pack_bf16x8(s, 8);
        } else {
            l_run += sm.psum;
        }
    };
    // one piece of the load path: rows of the tile at the cursor, index entries of the tile after it
    auto load_chunk = [&](auto C) __attribute__((always_inline)) {
        constexpr int c = decltype(C)::value;
        constexpr int PSTEP = LOADS <= 2 ? 2 : 1, PREP0 = LOADS <= 2 ? 2 : 1;  // chunks of the row preparation
        constexpr int ISTEP = LOADS <= 2 ? 2 : 1;                             // chunks 8.. of the row loads
        static_assert(PREP0 + (LOADS - 1) * PSTEP < 6 && 8 + (LOADS - 1) * ISTEP < 12, "chunks overlap");
        if (!loader) return;
        if constexpr (c == 0) {
            entries_landed();
            read_entries(l_g);
        } else if constexpr (c >= PREP0 && c < 6 && (c - PREP0) % PSTEP == 0 && (c - PREP0) / PSTEP < LOADS) {
            prepare_row(lcur.st, lcur.de, lcur.i0 + TP > lcur.de, l_t, l_g, IntC<(c - PREP0) / PSTEP>{});
        } else if constexpr (c == 6) {
            issue_meta_after_cursor();
        } else if constexpr (c >= 8 && c < 12 && (c - 8) % ISTEP == 0 && (c - 8) / ISTEP < LOADS) {
            issue_row(l_g, IntC<(c - 8) / ISTEP>{});
        } else if constexpr (c == 12) {
            advance_cursor();
        }
    };

    // one half of a tile step.  HB: which block of the tile (0 or 1).  DO_QK: S(2X+HB) of tile X into
    // s_new; DO_PV: O^T += V_{X-1}[32 HB ..]^T p_old^T; DO_SM: softmax of the block whose scores are
    // s_old (tile sm_tile, block sm_kb) into p_new; DO_LD: the load path of tile X+2 rides along.
    int gbase = 0;  // global number of tile 0 of the segment being multiplied
    auto half_step = [&](int X, auto HB_, auto DO_QK_, auto DO_PV_, auto DO_SM_, auto DO_LD_, f32x16 &s_new,
                         const bf16x8 (&p_old)[2], f32x16 &s_old, bf16x8 (&p_new)[2], int sm_tile,
                         int sm_kb) __attribute__((always_inline)) {
        constexpr int HB = decltype(HB_)::value;
        constexpr bool DO_QK = decltype(DO_QK_)::value != 0, DO_PV = decltype(DO_PV_)::value != 0;
        constexpr bool DO_SM = decltype(DO_SM_)::value != 0, DO_LD = decltype(DO_LD_)::value != 0;
        constexpr int N1 = DO_QK ? NQK : 0, N2 = DO_PV ? NPV : 0, NS = N1 + N2;
        constexpr int CPS = (16 + NS - 1) / NS;  // softmax / load chunks per matrix instruction
        if (DO_PV && __builtin_amdgcn_ballot_w64(alpha_pending != 1.f) != 0ull) {
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int i = 0; i < 16; ++i) oacc[db][i] *= alpha_pending;
            alpha_pending = 1.f;
        }
        const uint32_t vst = vs_base + ((unsigned)(gbase + X + VST - 1) % VST) * (TILE * 2) + HB * 32 * D * 2;
        const uint32_t kst = ks_base + ((unsigned)(gbase + X) % KST) * (TILE * 2) + HB * 32 * D * 2;
        uint32_t va_[DB], ka_[KSTEPS];
#pragma unroll
        for (int db = 0; db < DB; ++db) va_[db] = vst + voff[db];
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) ka_[ks] = kst + koff[ks];
        bf16x8 frag[LA];
        auto request = [&](auto S) __attribute__((always_inline)) {
            constexpr int s = decltype(S)::value;
            if constexpr (s < N1) {
                frag[s % LA] = lds_read_b128_at(ka_[s]);
            } else if constexpr (s < NS) {
                constexpr int q_ = s - N1, stp = q_ / DB, db = q_ % DB;
                frag[s % LA] = lds_read_tr_at(va_[db] + stp * 16 * D * 2, 4 * D * 2);
            }
        };
        auto multiply = [&](auto S) __attribute__((always_inline)) {
            constexpr int s = decltype(S)::value;
            if constexpr (s < N1) {
                if constexpr (s == 0) {
                    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                    s_new = mfma_bf16(frag[s % LA], qreg[s], zero);
                } else {
                    s_new = mfma_bf16(frag[s % LA], qreg[s], s_new);
                }
            } else {
                constexpr int q_ = s - N1, stp = q_ / DB, db = q_ % DB;
                oacc[db] = mfma_bf16(frag[s % LA], p_old[stp], oacc[db]);
            }
        };
        static_for<(LA < NS ? LA : NS)>([&](auto S) { request(S); });
        __builtin_amdgcn_sched_barrier(0);
        static_for<NS>([&](auto S) {
            constexpr int s_ = decltype(S)::value;
            multiply(S);
            request(IntC<s_ + LA>{});
            static_for<CPS>([&](auto J) {
                constexpr int c = s_ * CPS + decltype(J)::value;
                if constexpr (c < 16) {
                    if constexpr (DO_SM) softmax_chunk(IntC<c>{}, s_old, p_new, sm_tile, gbase + sm_tile, sm_kb);
                    if constexpr (DO_LD) load_chunk(IntC<c>{});
                }
            });
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    // barrier that publishes tile X: this wave's loads of tile X have landed (everything older than
    // the previous step's [1 entry load][2*LOADS row loads])
    auto publish = [&]() __attribute__((always_inline)) {
        wait_older_loads();
        wg_barrier();
    };

    // ---- start-up, once per workgroup: the first two tiles of the concatenated stream on their way
    // into LDS, the index entries of the third requested (three dependent round trips)
    if (loader) {
        issue_meta(lcur.st, 0, 0);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
        for (int rep = 0; rep < 2; ++rep) {
            read_entries(l_g);
            static_for<LOADS>([&](auto U) { prepare_row(lcur.st, lcur.de, lcur.i0 + TP > lcur.de, l_t, l_g, U); });
            issue_meta_after_cursor();
            static_for<LOADS>([&](auto U) { issue_row(l_g, U); });
            advance_cursor();
            entries_landed();  // the entries just requested (the rows after them may be in flight)
        }
    }
    wg_barrier();  // tile 0 is in LDS (its rows were the first loads)

    const IntC<1> yes;
    const IntC<0> no;
    const IntC<0> first_block;
    const IntC<1> second_block;
    Seg cseg = open_segment(0), cnext = open_segment(1);
    auto load_queries = [&](int seg_i0) __attribute__((always_inline)) {
        const int row = min(seg_i0 + 32 * (wave / GP) + qi, p.L - 1);
        const uint16_t *qrow = Q + (((long)b * p.Hq + head) * p.L + row) * D;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks)
            qreg[ks] = as_bf16x8(*reinterpret_cast<const u32x4 *>(qrow + ks * 16 + 8 * hh));
    };
    load_queries(cseg.i0);
    for (int round = 0; cseg.i0 >= 0; ++round) {
    i0 = cseg.i0;
    pw = i0 + 32 * (wave / GP);  // first position of this wave
    iq = pw + qi;                // this lane's query position
    iq_h = iq + hdelta;          // ... as the upper ends of the keys' query ranges (computed with p.n) see it
    st = cseg.st;
    n_tiles = cseg.n_tiles;
    fullb = full_blocks(st, pw, p.n - hdelta);
    if (DOCS && pw + 31 >= cseg.de) fullb = no_full_blocks();
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[db][i] = 0.f;
    m_run = -INFINITY;
    l_run = 0.f;
    alpha_pending = 1.f;

    // step 0: no output update yet, no softmax in the first half.  Tile 0 of the segment has been
    // published already: by the start-up barrier, or by the barrier of the previous segment's last
    // step (its rows were requested two load steps earlier, and each wave waits for everything but
    // its newest load step before a barrier).
    half_step(0, first_block, yes, no, no, yes, s_a, p_a, s_b, p_b, 0, 0);
    half_step(0, second_block, yes, no, yes, no, s_b, p_b, s_a, p_a, 0, 0);
    for (int X = 1; X < n_tiles; ++X) {
        publish();
        half_step(X, first_block, yes, yes, yes, yes, s_a, p_a, s_b, p_b, X - 1, 1);
        half_step(X, second_block, yes, yes, yes, no, s_b, p_b, s_a, p_a, X, 0);
    }
    // last step: output updates of the last tile, softmax of its second block; the queries of the
    // next segment are fetched meanwhile (the registers are free: no score block in this step)
    publish();
    if (cnext.i0 >= 0) load_queries(cnext.i0);
    half_step(n_tiles, first_block, no, yes, yes, no, s_a, p_a, s_b, p_b, n_tiles - 1, 1);
    half_step(n_tiles, second_block, no, yes, no, no, s_b, p_b, s_a, p_a, n_tiles, 0);
    gbase += n_tiles;

    // epilogue: normalise, store O (bf16) and LSE (natural log)
    if (__builtin_amdgcn_ballot_w64(alpha_pending != 1.f) != 0ull) {
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) oacc[db][i] *= alpha_pending;
    }
    float l_tot = pair_sum(l_run);
    float inv = 1.f / l_tot;
    // A lane holds 4-column pieces of ONE output row, so a store straight from the accumulators would
    // write 64 scattered 8-byte pieces per instruction, and the number of such pieces (1024 per wave
    // and segment) is what the stores cost.  Each 32-column block of the wave's 32 rows therefore goes
    // through a 2 KB staging area of the wave and leaves as 16-byte pieces of which four consecutive
    // lanes cover 64 contiguous bytes of a row (16 rows per store instruction).  8-byte chunk ch of
    // row r sits at chunk position ch ^ (2 * ((r / 4) % 4)): 16-byte pairs stay together, and the
    // writes (one chunk of 32 rows) spread over the banks.  The LDS operations of a wave execute in
    // order, so a block's reads are issued before the next block's writes without a wait in between.
    {
        uint16_t *stg = &ostage[wave][0];
        const long orow0 = ((long)b * p.Hq + head) * p.L + pw;  // output row of the wave's first query
        const int wsw = ((qi >> 2) & 3) << 1;
#pragma unroll
        for (int db = 0; db < DB; ++db) {
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const uint2 v = pack_bf16x4(oacc[db][4 * i4] * inv, oacc[db][4 * i4 + 1] * inv,
                                            oacc[db][4 * i4 + 2] * inv, oacc[db][4 * i4 + 3] * inv);
                *reinterpret_cast<uint2 *>(stg + qi * 32 + (((2 * i4 + hh) ^ wsw) * 4)) = v;
            }
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int r = 16 * t + (lane >> 2), c = lane & 3;
                const int pos = (2 * c) ^ (((r >> 2) & 3) << 1);
                const uint4 v = *reinterpret_cast<const uint4 *>(stg + r * 32 + pos * 4);
                if (pw + r < p.L) *reinterpret_cast<uint4 *>(O + (orow0 + r) * D + db * 32 + c * 8) = v;
            }
            __builtin_amdgcn_sched_barrier(0);  // one block at a time: keeps the register pressure of the epilogue down
        }
    }
    if (iq < p.L && hh == 0) LSE[((long)b * p.Hq + head) * p.L + iq] = (m_run + __builtin_amdgcn_logf(l_tot)) * kLn2_f;
    cseg = cnext;
    cnext = open_segment(round + 2);
    }  // segments
    // the loads of the padding tiles past the last segment are still in flight: they must have
    // landed before the workgroup ends and its LDS is handed on
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

template <int D, bool DOCS>
int launch_fwd(const sepattn_params &p, const uint16_t *Q, const uint16_t *K, const uint16_t *V,
               const int32_t *sep_idx, const int32_t *sep_prefix, const int32_t *doc_start, const int32_t *doc_end,
               uint16_t *O, float *LSE, const HeadWin &hw, hipStream_t st) {
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
    ProfScope prof(SEPATTN_K_FORWARD, st);
    auto go = [&](auto NW_) {
        constexpr int NW = decltype(NW_)::value;
        if (GP == 4)
            hipLaunchKernelGGL((fwd_bf16_kernel<D, 4, DOCS, NW>), grid, block, 0, st, p, Q, K, V, sep_idx, sep_prefix, doc_start, doc_end, O, LSE, wpg, hw);
        else if (GP == 2)
            hipLaunchKernelGGL((fwd_bf16_kernel<D, 2, DOCS, NW>), grid, block, 0, st, p, Q, K, V, sep_idx, sep_prefix, doc_start, doc_end, O, LSE, wpg, hw);
        else
            hipLaunchKernelGGL((fwd_bf16_kernel<D, 1, DOCS, NW>), grid, block, 0, st, p, Q, K, V, sep_idx, sep_prefix, doc_start, doc_end, O, LSE, wpg, hw);
    };
    if constexpr (D == 64) {
        if (narrow) go(IntC<4>{});
        else go(IntC<8>{});
    } else {
        go(IntC<8>{});
    }
    }
    return launch_status();
}

}  // namespace

size_t forward_bf16_workspace(const sepattn_params &) { return 0; }

int launch_forward_bf16(const sepattn_params &p, const HeadWin &hw, const void *Q, const void *K, const void *V,
                        const int32_t *sep_idx, const int32_t *sep_prefix, const int32_t *doc_start,
                        const int32_t *doc_end, void *O, float *LSE, void *, hipStream_t st) {
    auto q = static_cast<const uint16_t *>(Q), k = static_cast<const uint16_t *>(K),
         v = static_cast<const uint16_t *>(V);
    auto o = static_cast<uint16_t *>(O);
    if (doc_start) {
        if (p.d == 64) return launch_fwd<64, true>(p, q, k, v, sep_idx, sep_prefix, doc_start, doc_end, o, LSE, hw, st);
        return launch_fwd<128, true>(p, q, k, v, sep_idx, sep_prefix, doc_start, doc_end, o, LSE, hw, st);
    }
    if (p.d == 64) return launch_fwd<64, false>(p, q, k, v, sep_idx, sep_prefix, nullptr, nullptr, o, LSE, hw, st);
    return launch_fwd<128, false>(p, q, k, v, sep_idx, sep_prefix, nullptr, nullptr, o, LSE, hw, st);
}

}  // namespace sepattn
