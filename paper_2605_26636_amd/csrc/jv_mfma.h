// Device helpers for the bf16 matrix-core kernels (gfx950, wavefront 64).
//
// Register layouts of v_mfma_f32_32x32x16_bf16 (D = A*B + C, A is 32x16, B is 16x32), with
// lane = 32*g + i:
//   A operand: lane holds A[i][8g .. 8g+7]            (8 bf16 = 4 VGPRs)
//   B operand: lane holds B[8g .. 8g+7][i]
//   C/D      : lane holds D[8*(v/4) + 4g + v%4][i] in accumulator register v = 0..15
// The contraction index only has to be labelled the same way in A and B, so "k-slot (g, e)"
// may stand for any token as long as both operands agree.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace jv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) short s16x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

__device__ inline f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Loads and stores of data that is touched once per launch (the Q/K/V/O streams of the
// HBM-bound mixers), marked non-temporal so that they do not displace what is reused.  Only for
// accesses that cover whole 128-byte lines within one instruction: a line that several
// non-temporal instructions touch in parts is fetched again for each of them.
// JV_STREAM_HINTS=0 builds the plain forms (for A/B timing).
#ifndef JV_STREAM_HINTS
#define JV_STREAM_HINTS 1
#endif
constexpr int kDmaStreamAux = JV_STREAM_HINTS ? 2 : 0;  // cache-policy bits of the LDS-DMA load: nt
__device__ inline u32x4 ld_stream(const u32x4 *p) {
#if JV_STREAM_HINTS
    return __builtin_nontemporal_load(p);
#else
    return *p;
#endif
}
__device__ inline void st_stream(u32x4 *p, u32x4 v) {
#if JV_STREAM_HINTS
    __builtin_nontemporal_store(v, p);
#else
    *p = v;
#endif
}
__device__ inline void st_stream(f32x4 *p, f32x4 v) {
#if JV_STREAM_HINTS
    __builtin_nontemporal_store(v, p);
#else
    *p = v;
#endif
}

__device__ inline bf16x8 as_bf16x8(u32x4 x) { return __builtin_bit_cast(bf16x8, x); }
__device__ inline u32x4 as_u32x4(bf16x8 x) { return __builtin_bit_cast(u32x4, x); }

// ReLU on two packed bf16: as signed 16-bit integers, negative floats are negative integers.
__device__ inline unsigned relu_bf16x2(unsigned x) {
    s16x2 v = __builtin_bit_cast(s16x2, x);
    s16x2 zero = {0, 0};
    v = __builtin_elementwise_max(v, zero);
    return __builtin_bit_cast(unsigned, v);
}
__device__ inline u32x4 relu_bf16x8(u32x4 x) {
    u32x4 r;
    r[0] = relu_bf16x2(x[0]); r[1] = relu_bf16x2(x[1]);
    r[2] = relu_bf16x2(x[2]); r[3] = relu_bf16x2(x[3]);
    return r;
}

// fp32 pair -> packed bf16 (round to nearest even), low half = a.
__device__ inline unsigned pack_bf16x2(float a, float b) {
    bf16x2 r;
    r[0] = (__bf16)a;
    r[1] = (__bf16)b;
    return __builtin_bit_cast(unsigned, r);
}
__device__ inline float bf16_lo(unsigned x) { return __builtin_bit_cast(float, x << 16); }
__device__ inline float bf16_hi(unsigned x) { return __builtin_bit_cast(float, x & 0xffff0000u); }

// Sum of the two bf16 halves of x added to acc (fp32).
__device__ inline float add_bf16x2(unsigned x, float acc) {
    const unsigned ones = 0x3f803f80u;  // (1.0bf16, 1.0bf16)
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, x),
                                           __builtin_bit_cast(bf16x2, ones), acc, false);
}

// Transposing LDS read (ds_read_b64_tr_b16).  Within each block of 16 lanes, lane n receives
// element e = 0..3 from the 8 bytes addressed by lane 4e + n/4, 16-bit element n%4: if lanes
// 4r..4r+3 of a block address the four 8-byte pieces of a 16-element row r, lane n ends up
// with column n of the 4 x 16 block.
__device__ inline u32x2 lds_read_tr16(const unsigned char *lds_ptr) {
    s16x4 r = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)lds_ptr);
    return __builtin_bit_cast(u32x2, r);
}

// The same read written in assembly, at `addr` + OFF bytes (addr: LDS byte address, OFF: a
// compile-time constant that goes into the instruction's offset field).  The compiler's wait
// insertion treats the builtin above as a read of unknown LDS bytes and puts a wait for ALL
// outstanding vector-memory loads (vmcnt 0) in front of it whenever loads that write LDS
// (global_load_lds) are in flight, which serialises a kernel that keeps such loads in flight
// across its arithmetic.  Written this way the read is invisible to that pass: the caller
// orders it against the loads with its own counted waits and barriers, and must wait for the
// result itself (lds_reads_landed) before using it.
__device__ inline unsigned lds_address(const void *p) {
    return (unsigned)(unsigned long long)(__attribute__((address_space(3))) const unsigned char *)p;
}
template <int OFF>
__device__ inline u32x2 lds_read_tr16_at(unsigned addr) {
    static_assert(OFF >= 0 && OFF < 65536, "offset field is 16 bits");
    u32x2 r;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF));
    return r;
}
// Plain 16-byte LDS read in the same style (ds_read_b128), for kernels whose operand reads
// use run-time addresses: the compiler cannot tell those from the bytes that in-flight loads
// into LDS are writing and waits for all of them.
template <int OFF>
__device__ inline u32x4 lds_read_b128_at(unsigned addr) {
    static_assert(OFF >= 0 && OFF < 65536, "offset field is 16 bits");
    u32x4 r;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF));
    return r;
}
// The same read, ordered after the compiler's own LDS stores that precede it in the source
// (for reading back what the wavefront has just staged in LDS).
__device__ inline u32x4 lds_read_b128_ordered(unsigned addr) {
    u32x4 r;
    asm volatile("ds_read_b128 %0, %1" : "=v"(r) : "v"(addr) : "memory");
    return r;
}
// Wait for every LDS read this wavefront has issued; the operands are tied to the wait so
// that no instruction using them can be scheduled above it.
__device__ inline void lds_reads_landed(u32x4 &a, u32x4 &b, u32x4 &c, u32x4 &d) {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d));
}
__device__ inline void lds_reads_landed(u32x4 (&a)[2], u32x4 (&b)[2], u32x4 (&c)[4]) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(a[0]), "+v"(a[1]), "+v"(b[0]), "+v"(b[1]), "+v"(c[0]), "+v"(c[1]), "+v"(c[2]), "+v"(c[3]));
}

// Workgroup barrier for kernels that order their LDS traffic with their own counted waits:
// this wavefront's LDS operations have completed, then the barrier.  Unlike __syncthreads()
// it carries no memory fence, which the compiler implements by waiting for every outstanding
// vector-memory operation as well: loads into LDS that are meant to stay in flight across
// the barrier, and output stores that no one in the workgroup reads.
__device__ inline void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Exchange between lane l and lane l^32: returns {value of the lower lane, value of the upper
// lane} in both lanes (v_permlane32_swap).
__device__ inline void pair_values(float x, float *lo, float *hi) {
    unsigned u = __builtin_bit_cast(unsigned, x);
    auto s = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    *lo = __builtin_bit_cast(float, (unsigned)s[0]);
    *hi = __builtin_bit_cast(float, (unsigned)s[1]);
}

// Tile of 16-bit rows in LDS, 128 bytes (64 channels) per row.  The 64-byte half a 16-byte
// chunk lands in is flipped from row to row so that the 8 rows one transposing read touches
// spread over all banks.
__device__ inline unsigned tile_off_tr(int row, int chunk16) {
    return (unsigned)(row * 128 + ((chunk16 ^ (((row ^ (row >> 1)) & 1) << 2)) << 4));
}
// Same tile, for row-per-lane 16-byte reads: the chunk index is rotated by the row pair, so
// that the 16 consecutive rows one pass of such a read touches (16 lanes x 16 bytes = all 64
// banks) land on 16 different 16-byte bank groups.
__device__ inline int tile_row_rotation(int row) { return (row >> 1) & 7; }
__device__ inline unsigned tile_off_row(int row, int chunk16) {
    return (unsigned)(row * 128 + ((chunk16 ^ tile_row_rotation(row)) << 4));
}

// Tiles of 256-byte rows (128 channels of 16 bits).  Row-per-lane 16-byte reads: the chunk
// index is rotated by the row, so that 16 consecutive rows land on 16 different bank groups.
__device__ inline unsigned wide_off_row(int row, int chunk16) {
    return (unsigned)(row * 256 + ((chunk16 ^ (row & 15)) << 4));
}
// Transposing reads (V operands) touch 64 bytes of each of four consecutive rows per half
// wavefront: the 64-byte quarter of a row is rotated by the row, which spreads them over all banks.
__device__ inline unsigned wide_off_tr(int row, int chunk16) {
    return (unsigned)(row * 256 + ((((chunk16 >> 2) ^ (row & 3)) << 6) | ((chunk16 & 3) << 4)));
}

// Operand "lane = channel, k-slots = 8 tokens" read from a [token][channel] tile laid out
// with tile_off_tr: channels 32*blk32 .. +31, tokens tok0 + 8g + (0..7).
__device__ inline bf16x8 load_tr_operand(const unsigned char *tile, int tok0, int blk32,
                                         int lane) {
    const int b = lane >> 4, j = lane & 15, g = b >> 1;
    const int chunk16 = blk32 * 4 + (b & 1) * 2 + ((j & 3) >> 1);
    const int half = (j & 1) * 8;
    const int row0 = tok0 + 8 * g + (j >> 2);
    u32x2 r0 = lds_read_tr16(tile + tile_off_tr(row0, chunk16) + half);
    u32x2 r1 = lds_read_tr16(tile + tile_off_tr(row0 + 4, chunk16) + half);
    u32x4 r = {r0[0], r0[1], r1[0], r1[1]};
    return as_bf16x8(r);
}

}  // namespace jv
