// Device helpers shared by the bf16 MFMA kernels (gfx950 / CDNA4, wave64).
//
// All contractions use v_mfma_f32_32x32x16_bf16.  Operand layouts (lane l of the wave):
//   A (32 x 16): row l%32, k = 8*(l/32) .. +7        B (16 x 32): column l%32, k = 8*(l/32) .. +7
//   C (32 x 32): column l%32, register i holds row 8*(i/4) + 4*(l/32) + i%4
// The kernels always put the "streamed" matrix (staged in LDS) in A and the wave's own 32 rows
// (queries in forward / dQ, keys in dK/dV) in B, so every softmax quantity of one query (or key)
// lives in one lane pair (l, l+32).
//
// Row permutation pi: the A-operand lane with l%32 = m reads LDS row pi(m).  With it, register i
// of lane half hh = l/32 holds streamed row  rho(hh, i) = 16*(i/8) + 8*hh + i%8,  i.e. registers
// 0..7 and 8..15 are two runs of eight consecutive rows.  Those runs are exactly the k-slots that
// lane needs as the B operand of the following contraction over the streamed rows (P^T, dS^T, ...),
// so scores flow from accumulator registers into the next MFMA without any cross-lane movement.
//
// Transposed A operands (V^T, K^T, Q^T, dO^T) are read from row-major LDS tiles with
// ds_read_b64_tr_b16: within each group of 16 lanes, lane p supplies the address of four
// consecutive 16-bit elements; the 16 x 4 elements, taken as a 4 x 16 matrix (row r = lanes
// 4r..4r+3), are returned column-wise: lane i receives column i.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sepattn {

// compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>).  Used where a
// register array must be indexed by constants only (a rolled loop would push it to scratch memory).
template <int I>
struct IntC {
    static constexpr int value = I;
    constexpr operator int() const { return I; }
};
template <int N, int I = 0, typename F>
__device__ inline void static_for(F &&f) {
    if constexpr (I < N) {
        f(IntC<I>{});
        static_for<N, I + 1>(f);
    }
}

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
// native 16-byte vector for staging registers (HIP's uint4 is a struct the optimiser may keep in
// scratch memory when it sits in an array)
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr float kLog2e_f = 1.4426950408889634f;
constexpr float kLn2_f = 0.6931471805599453f;
constexpr int kIntMax = 0x7FFFFFFF;

__device__ inline int pi_row(int m) {
    // inverse of: register i of lane half hh <-> accumulator row 8*(i/4) + 4*hh + i%4
    int i4 = m >> 3, hh = (m >> 2) & 1, r = m & 3;
    return 16 * (i4 >> 1) + 8 * hh + 4 * (i4 & 1) + r;
}

// streamed row (within a block of 32) held by accumulator register i of lane half hh
__device__ inline int rho_row(int hh, int i) { return 16 * (i >> 3) + 8 * hh + (i & 7); }

__device__ inline f32x16 mfma_bf16(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ inline bf16x8 as_bf16x8(u32x4 u) { return __builtin_bit_cast(bf16x8, u); }

// ---- LDS tiles filled by direct global->LDS loads -------------------------------------------------
// global_load_lds_dwordx4: every lane fetches 16 bytes from its own global address and the wave's
// 64 pieces land contiguously in LDS at (wave-uniform base) + 16*lane.  Tiles are therefore stored
// unpadded, [rows][D] bf16, and bank conflicts are avoided by permuting the 16-byte chunks of a row
// with an XOR that depends on the row; the permutation is applied on the global-address side (lane
// l of a load fills physical chunk l%CH of its row, so it fetches logical chunk phys^swz(row)).
//   kSwzRow: 16 consecutive rows hit 16 different 16-byte bank slots, so row-major 16-byte
//            A-operand reads (32 lanes, one chunk column) are conflict-free
//            (D=128: chunk ^= row%16;  D=64, two rows per 256 bytes: chunk ^= (row/2)%8)
//   kSwzTr : 4 consecutive rows put a 64-byte column window into 4 different 64-byte bank groups,
//            so ds_read_b64_tr_b16 reads (4 rows x 64 bytes per 32 lanes) are conflict-free
//            (D=128: chunk ^= (row%4)*4;  D=64: chunk ^= ((row/2)%2)*4)
//   kSwzBoth: one permutation that serves both kinds of read of the same tile (the dK/dV kernels
//            read Q and dO tiles row-major and transposed): the XOR mask is a bit permutation of the
//            row number that puts row bits 0..1 (bit 1 for D=64) into chunk bits 2..3, as kSwzTr
//            needs, and spreads the 16 rows {0-3, 8-11, 4-7, 12-15} that 16 consecutive lanes of a
//            row-major A-operand read touch over 16 different 16-byte slots
enum { kSwzRow = 0, kSwzTr = 1, kSwzBoth = 2 };
template <int MODE, int D>
__device__ inline int swz_chunk(int chunk, int row) {
    if (MODE == kSwzBoth) {
        if (D == 128) return chunk ^ (((row & 3) << 2) | (((row >> 3) & 1) << 1) | ((row >> 2) & 1));
        return chunk ^ ((((row >> 1) & 1) << 2) | ((row >> 2) & 3));
    }
    if (D == 128) return MODE == kSwzRow ? (chunk ^ (row & 15)) : (chunk ^ ((row & 3) << 2));
    return MODE == kSwzRow ? (chunk ^ ((row >> 1) & 7)) : (chunk ^ (((row >> 1) & 1) << 2));
}

// Direct global->LDS loads, through inline assembly.  For the builtin forms the compiler knows that LDS is
// written asynchronously, and since it cannot tell which LDS bytes a later ds_read touches it makes
// every LDS read wait for ALL outstanding loads (vmcnt(0)), which serialises a prefetch pipeline.
// These forms are opaque to it: the kernels that use them wait explicitly (s_waitcnt vmcnt(n), loads
// complete in issue order) before the data is read, and every such wait carries a memory clobber so
// that no LDS access is moved across it at compile time.
// M0 (the LDS base of such a load) is written inside the statement; the compiler treats M0 as a
// reserved register that it sets itself right before each of its own uses, and the kernels that use
// these helpers contain no other M0 user.
//   base      wave-uniform global pointer        voff   per-lane byte offset from base (32 bits)
//   lds_addr  wave-uniform LDS byte address: lane l's piece lands at lds_addr + 16*l (or 4*l)
__device__ inline void dma_to_lds_16(const void *base, uint32_t voff, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(base)
                 : "memory");
}
// the same with the non-temporal hint: for data that is read once (the decode's cache rows)
__device__ inline void dma_to_lds_16_nt(const void *base, uint32_t voff, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(base)
                 : "memory");
}
__device__ inline void dma_to_lds_4(const void *base, uint32_t voff, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(base)
                 : "memory");
}

// 4-byte form with a full per-lane address (lanes that are switched off fetch and write nothing)
__device__ inline void dma_to_lds_4_addr(const void *lane_addr, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off"
                 :
                 : "s"(lds_addr), "v"(lane_addr)
                 : "memory");
}

// 16-byte A-operand read from a swizzled unpadded tile: row `row`, logical chunk `chunk`
template <int MODE, int D>
__device__ inline bf16x8 lds_read_a_swz(const uint16_t *tile, int row, int chunk) {
    return *reinterpret_cast<const bf16x8 *>(tile + row * D + swz_chunk<MODE, D>(chunk, row) * 8);
}

// transposed A operand from a swizzled unpadded tile: element (m, k) = tile[row0 + k][col0 + m],
// m = l%32, the k-slots of lane half hh are rows row0 + 8*hh .. +7.  Two 64-bit transposed reads.
template <int MODE, int D>
__device__ inline bf16x8 lds_read_a_tr_swz(const uint16_t *tile, int row0, int col0, int lane) {
    int p = lane & 15, g = lane >> 4;
    int r = row0 + 8 * (g >> 1) + (p >> 2);
    int c = col0 + 16 * (g & 1) + 4 * (p & 3);  // element column: chunk c/8, 8-byte half (c/4)%2
    const uint16_t *a0 = tile + r * D + swz_chunk<MODE, D>(c >> 3, r) * 8 + (c & 4);
    const uint16_t *a1 = tile + (r + 4) * D + swz_chunk<MODE, D>(c >> 3, r + 4) * 8 + (c & 4);
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)a0);
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)a1);
    union {
        s16x4 s[2];
        bf16x8 v;
    } x;
    x.s[0] = lo;
    x.s[1] = hi;
    return x.v;
}

// ---- LDS reads by 32-bit byte address ---------------------------------------------------------------
// The kernels precompute, once per lane, the byte offset of every operand fragment inside a tile
// (the XOR swizzle makes it a per-lane constant); per tile only the stage base is added, and the
// block / step within the tile goes into the instruction's immediate offset.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Wint-to-pointer-cast"  // LDS pointers are 32 bits wide on the device
__device__ inline uint32_t lds_addr(const void *p) {
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void *)p;
}
__device__ inline bf16x8 lds_read_b128_at(uint32_t addr) {
    return *(const bf16x8 __attribute__((address_space(3))) *)addr;
}
// two transposed 64-bit reads, `second` bytes apart (the rows r and r+4 of lds_read_a_tr_swz)
__device__ inline bf16x8 lds_read_tr_at(uint32_t addr, uint32_t second) {
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)addr);
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)(addr + second));
    union {
        s16x4 s[2];
        bf16x8 v;
    } x;
    x.s[0] = lo;
    x.s[1] = hi;
    return x.v;
}
__device__ inline bf16x8 lds_read_tr_at2(uint32_t addr0, uint32_t addr1) {
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)addr0);
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)addr1);
    union {
        s16x4 s[2];
        bf16x8 v;
    } x;
    x.s[0] = lo;
    x.s[1] = hi;
    return x.v;
}
#pragma clang diagnostic pop
// byte offset of the 16-byte row-major A fragment (row, logical chunk) in a swizzled unpadded tile
template <int MODE, int D>
__device__ inline uint32_t lds_off_a(int row, int chunk) {
    return (uint32_t)(row * D + swz_chunk<MODE, D>(chunk, row) * 8) * 2u;
}
// byte offset of this lane's first transposed read for rows 0..15, columns col0 + l%32 (see
// lds_read_a_tr_swz); with kSwzTr the second read is exactly 4 rows further on
template <int MODE, int D>
__device__ inline uint32_t lds_off_a_tr(int col0, int lane) {
    int p = lane & 15, g = lane >> 4;
    int r = 8 * (g >> 1) + (p >> 2);
    int c = col0 + 16 * (g & 1) + 4 * (p & 3);
    return (uint32_t)(r * D + swz_chunk<MODE, D>(c >> 3, r) * 8 + (c & 4)) * 2u;
}

// the same for the second transposed read (row r + 4), for layouts in which it is not simply
// 4 rows further on (kSwzBoth)
template <int MODE, int D>
__device__ inline uint32_t lds_off_a_tr_second(int col0, int lane) {
    int p = lane & 15, g = lane >> 4;
    int r = 8 * (g >> 1) + (p >> 2) + 4;
    int c = col0 + 16 * (g & 1) + 4 * (p & 3);
    return (uint32_t)(r * D + swz_chunk<MODE, D>(c >> 3, r) * 8 + (c & 4)) * 2u;
}
// combine a per-lane value with the other half of the lane pair (l, l^32)
__device__ inline float pair_max(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ inline float pair_sum(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// eight fp32 accumulator values -> packed bf16 B operand (round to nearest even)
__device__ inline bf16x8 pack_bf16x8(const f32x16 &v, int first) {
    f32x8 t;
#pragma unroll
    for (int k = 0; k < 8; ++k) t[k] = v[first + k];
    return __builtin_convertvector(t, bf16x8);
}

__device__ inline uint2 pack_bf16x4(float a, float b, float c, float d) {
    f32x4 t = {a, b, c, d};
    bf16x4 r = __builtin_convertvector(t, bf16x4);
    union {
        bf16x4 v;
        uint2 u;
    } x;
    x.v = r;
    return x.u;
}

}  // namespace sepattn
