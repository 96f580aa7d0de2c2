// Softmax attention for bf16 tensors on the matrix cores (Eq. 1 of the paper; restricted to a
// window of the token grid for window attention, Sec. 3.2.2), fp32 softmax and accumulation.
//
// A wavefront owns 64 query slots of one window (two 32-column blocks) and walks the window's
// key slots in tiles of 32.  Per tile it forms the transposed scores S^T = K_tile Q^T, so that
// a lane holds one query column: row maxima and sums stay inside a lane (plus one exchange
// with lane^32), and the exponentiated tile, rounded to bf16, is already laid out as the B
// operand of O^T += V_tile^T P^T.  K tiles are read from LDS row by row (A operand of the
// first product); V tiles are read with transposing LDS reads (A operand of the second).
// The softmax reference (running maximum) is only raised when a tile's probabilities against
// the current reference come out large (lane sum above 2^8); the common path has no maximum
// search and no rescaling of the accumulators.  The result is unchanged because numerator and
// denominator always use the same reference.
#include <math.h>

#include <type_traits>

#include "jv_common.h"
#include "jv_mfma.h"

#ifndef JV_ATTN_NT
#define JV_ATTN_NT 2   // blocks of 32 query columns per wavefront
#endif
#ifndef JV_ATTN_MINW
#define JV_ATTN_MINW 2  // wavefronts per SIMD the register budget is sized for
#endif

namespace jv {

struct AttnArgs {
    TensorArg q, k, v, o;
    WindowGeom g;
    int heads;
    int contig;  // windows span whole grid rows: token = first token of the window + slot
    int q_slots; // leading query slots of each window to compute (all keys always take part)
    float c;     // logit scale times log2(e)
    int n_bh;    // batch * heads
};

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLazySum = 256.0f;     // largest lane sum of a tile taken without a max pass
constexpr float kMinusHuge = -1.0e30f; // finite stand-in for "no maximum yet"

// Work items of the streaming and ring kernels: (query block, window, batch * head), query block fastest.  The
// hardware deals consecutive workgroups to the eight XCDs in turn; the launch is one-dimensional
// (8 * ceil(items / 8) workgroups) and workgroup w takes item (w % 8) * ceil(items / 8) + w / 8,
// so that an XCD walks a contiguous range of items: the query blocks that stream the same keys
// and values run next to each other on one XCD and find them in its L2 (with a three-dimensional
// grid every XCD streamed every head's keys and values; full attention on 4096 tokens x 128
// heads: 577 -> 555 us, with 128 channels 543 -> 523 us).
struct RingItem { int qblock, win, bh; };
__device__ inline bool ring_item(const AttnArgs &a, int block_slots, RingItem &it) {
    const int nq = (a.q_slots + block_slots - 1) / block_slots;
    const int items = nq * a.g.n_win * a.n_bh, per_xcd = (items + 7) >> 3;
    const int item = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (item >= items) return false;
    it.qblock = item % nq;
    it.win = (item / nq) % a.g.n_win;
    it.bh = item / (nq * a.g.n_win);
    return true;
}
inline dim3 ring_grid(const AttnArgs &a, int block_slots) {
    const long long items = (long long)((a.q_slots + block_slots - 1) / block_slots) * a.g.n_win * a.n_bh;
    return dim3((unsigned)(8 * ((items + 7) / 8)));
}

// slot of window (wy, wx) -> token index, or -1 for padding / past the window.
__device__ inline int slot_token(const AttnArgs &a, int wy, int wx, int slot) {
    const WindowGeom &g = a.g;
    if (slot >= g.slots) return -1;
    if (a.contig) {
        const int tok = wy * g.wh * g.W + slot;
        return tok < g.H * g.W ? tok : -1;
    }
    const int r = wy * g.wh + slot / g.ww, c = wx * g.ww + slot % g.ww;
    return (r < g.H && c < g.W) ? r * g.W + c : -1;
}

// A operands of O^T += V^T P^T for one tile of 32 keys: va[kk][mi] holds channels 32*mi .. +31
// (one per lane) of keys 16*kk .. +15 of the tile, k-slot (g, 4r + e) standing for key
// 16*kk + 8r + 4g + e, the order in which a lane holds its scores.  `vaddr[mi]` is this lane's
// LDS byte address for the tile's first key (vt_lane_address), OFF a compile-time byte offset
// on top of it: because a tile starts at a multiple of 16 rows, the chunk flips of tile_off_tr
// are the same for every 8-row step, so all eight reads are constant offsets from two
// per-lane addresses.  The reads are written in assembly (see lds_read_tr16_at): wait with
// lds_reads_landed before use.
__device__ inline unsigned vt_lane_address(const unsigned char *vrow0, int mi, int lane) {
    const int b = lane >> 4, j = lane & 15, g = b >> 1;
    const int chunk16 = mi * 4 + (b & 1) * 2 + ((j & 3) >> 1);
    return lds_address(vrow0) + tile_off_tr(4 * g + (j >> 2), chunk16) + (j & 1) * 8;
}
template <int OFF>
__device__ inline void load_vt_operands(u32x4 (&va)[2][2], const unsigned (&vaddr)[2]) {
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
        for (int mi = 0; mi < 2; ++mi) {
            u32x2 r0, r1;
            if (kk == 0) {
                r0 = lds_read_tr16_at<OFF>(vaddr[mi]);
                r1 = lds_read_tr16_at<OFF + 1024>(vaddr[mi]);
            } else {
                r0 = lds_read_tr16_at<OFF + 2048>(vaddr[mi]);
                r1 = lds_read_tr16_at<OFF + 3072>(vaddr[mi]);
            }
            u32x4 r = {r0[0], r0[1], r1[0], r1[1]};
            va[kk][mi] = r;
        }
}

// Running softmax state of one wavefront: NT blocks of 32 query columns, 64 channels.
template <int NT>
struct WaveState {
    f32x16 acc[2][NT];  // [channel block][query block]
    float m[NT], l[NT];  // per query block; l is this lane's half of the keys only
};

template <int NT>
__device__ inline void wave_state_init(WaveState<NT> &w) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int v = 0; v < 16; ++v) w.acc[mi][nt][v] = 0.f;
        w.m[nt] = kMinusHuge;
        w.l[nt] = 0.f;
    }
}

// Slow path of the running softmax: find the exact maximum of the (already masked) scores s of
// query block nt, raise the reference to it and rescale that block's accumulators and row sum.
template <int NT>
__device__ inline void raise_reference(WaveState<NT> &w, int nt, const f32x16 &s, float c) {
    float t0 = fmaxf(fmaxf(s[0], s[1]), s[2]);
    float t1 = fmaxf(fmaxf(s[3], s[4]), s[5]);
    float t2 = fmaxf(fmaxf(s[6], s[7]), s[8]);
    float t3 = fmaxf(fmaxf(s[9], s[10]), s[11]);
    float t4 = fmaxf(fmaxf(s[12], s[13]), s[14]);
    t0 = fmaxf(fmaxf(t0, t1), t2);
    t3 = fmaxf(fmaxf(t3, t4), s[15]);
    float a, b;
    pair_values(fmaxf(t0, t3) * c, &a, &b);  // this lane and lane^32 share the query column
    const float m_new = fmaxf(w.m[nt], fmaxf(a, b));
    const float alpha = __builtin_amdgcn_exp2f(w.m[nt] - m_new);
    w.m[nt] = m_new;
    w.l[nt] *= alpha;
    // Multiply in place, register by register: written as an opaque instruction so that the
    // common path (no rescaling) needs no register copies where the two paths meet.  alpha
    // comes out of a transcendental instruction, whose result may not be read by the very
    // next vector instruction; the compiler does not pad inline assembly, so pad here.
    asm volatile("s_nop 1" ::"v"(alpha));
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            float x = w.acc[mi][nt][v];
            asm volatile("v_mul_f32 %0, %0, %1" : "+v"(x) : "v"(alpha));
            w.acc[mi][nt][v] = x;
        }
}

// Probabilities of one query block's tile against the current reference: rounded to bf16 and
// packed in score-register order; returns this lane's sum (fp32, before rounding).
// (Plain adds on purpose: summing the packed pairs with dot-product instructions halves the
// additions but those instructions share the matrix pipeline -- full attention took the same
// time with them and window attention 8 % more.)
__device__ inline float exp_block(const f32x16 &s, unsigned (&pk)[8], float c, float neg_m) {
    float sum0 = 0.f, sum1 = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const float p0 = __builtin_amdgcn_exp2f(fmaf(s[2 * j], c, neg_m));
        const float p1 = __builtin_amdgcn_exp2f(fmaf(s[2 * j + 1], c, neg_m));
        pk[j] = pack_bf16x2(p0, p1);
        sum0 += p0;
        sum1 += p1;
    }
    return sum0 + sum1;
}

__device__ inline void add_key_bias(f32x16 &s, const float *bias, int g) {
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
        const f32x4 bv = *(const f32x4 *)(bias + 8 * q4 + 4 * g);
#pragma unroll
        for (int e = 0; e < 4; ++e) s[4 * q4 + e] += bv[e];
    }
}

// K operands of one tile of 32 keys (A of S^T = K Q^T): lane holds channels 16*ks + 8g .. +7
// of key row lane%32 of the tile.  `kaddr[ks]` is this lane's LDS byte address of that piece in
// a tile that starts at row 0 of a K stage laid out with tile_off_row (k_lane_addresses); a
// tile that starts at another multiple of 16 rows has the same chunk rotation, so it is a
// constant number of bytes (OFF) further on.  Read in assembly, like the V operands: wait with
// lds_reads_landed before use.
__device__ inline void k_lane_addresses(unsigned (&kaddr)[4], const unsigned char *krow0, int lane) {
    const int g = lane >> 5, li = lane & 31;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) kaddr[ks] = lds_address(krow0) + tile_off_row(li, 2 * ks + g);
}
template <int OFF>
__device__ inline void load_k_operands(u32x4 (&ka)[4], const unsigned (&kaddr)[4]) {
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) ka[ks] = lds_read_b128_at<OFF>(kaddr[ks]);
}
__device__ inline void k_operands_landed(u32x4 (&ka)[4]) { lds_reads_landed(ka[0], ka[1], ka[2], ka[3]); }

// One tile of 32 keys.  `ka` holds the tile's K operands on entry (landed); its V rows (laid
// out with tile_off_tr) are addressed by vaddr + VOFF (load_vt_operands).  If KNEXT >= 0 the K
// operands of the tile at kaddr + KNEXT are read into `ka` as soon as the scores are issued, so
// that their LDS latency hides behind the exponentials, like that of the V operands; they have
// landed when the function returns.  bias, if non-null, holds 0 / -inf per key of the tile.
template <int NT, int KNEXT, int VOFF>
__device__ __forceinline__ void attn_tile32(WaveState<NT> &w, const u32x4 (&qreg)[NT][4], u32x4 (&ka)[4],
                                   const unsigned (&kaddr)[4], const unsigned (&vaddr)[2],
                                   const float *bias, float c, int lane) {
    const int g = lane >> 5;
    f32x16 s[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int v = 0; v < 16; ++v) s[nt][v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) s[nt] = mfma32(as_bf16x8(ka[ks]), as_bf16x8(qreg[nt][ks]), s[nt]);
    __builtin_amdgcn_sched_barrier(0);  // the score products are issued before the reads below
    u32x4 va[2][2];
    load_vt_operands<VOFF>(va, vaddr);
    if (KNEXT >= 0) load_k_operands<KNEXT >= 0 ? KNEXT : 0>(ka, kaddr);
    __builtin_amdgcn_sched_barrier(0);  // ... and the reads before the softmax arithmetic
    if (bias) {  // wave-uniform
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) add_key_bias(s[nt], bias, g);
    }
    // Exponentiate against the current reference first; the tile sum tells whether that was
    // safe.  A lane sum of at most 2^8 means every probability is at most 2^8 (the reference
    // is at most 8 binary orders stale), which neither overflows nor costs precision.  Larger
    // sums (or the infinities of the very first tile) take the slow path: raise the reference
    // to the exact maximum and redo the block.  Numerator and denominator always share one
    // reference, so the result does not depend on which path ran.
    unsigned pk[NT][8];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        float tile_sum = exp_block(s[nt], pk[nt], c, -w.m[nt]);
        if (__builtin_amdgcn_ballot_w64(!(tile_sum <= kLazySum)) != 0) {  // also catches inf/NaN
            raise_reference<NT>(w, nt, s[nt], c);
            tile_sum = exp_block(s[nt], pk[nt], c, -w.m[nt]);
        }
        w.l[nt] += tile_sum;
    }
    if (KNEXT >= 0) lds_reads_landed(va[0], va[1], ka);  // (va[kk] is the pair of channel blocks)
    else lds_reads_landed(va[0][0], va[0][1], va[1][0], va[1][1]);
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                u32x4 pb = {pk[nt][4 * kk], pk[nt][4 * kk + 1], pk[nt][4 * kk + 2], pk[nt][4 * kk + 3]};
                w.acc[mi][nt] = mfma32(as_bf16x8(va[kk][mi]), as_bf16x8(pb), w.acc[mi][nt]);
            }
}

// Normalise and store the 32*NT query columns of a wavefront.  `stage` is 4 KB of wave-private
// LDS used to turn the channel-major accumulators into token rows for 16-byte stores.
template <bool O_BF16, int NT>
__device__ inline void wave_store(const WaveState<NT> &w, const AttnArgs &a, int wy, int wx,
                                  int q0, long long obase, unsigned char *stage, int lane) {
    const int g = lane >> 5, li = lane & 31, lrow = lane >> 3, lchunk = lane & 7;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        float lo, hi;
        pair_values(w.l[nt], &lo, &hi);
        const float inv = __builtin_amdgcn_rcpf(lo + hi);
        if (O_BF16) {
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    const f32x16 &x = w.acc[mi][nt];
                    u32x2 pk = {pack_bf16x2(x[4 * q4] * inv, x[4 * q4 + 1] * inv),
                                pack_bf16x2(x[4 * q4 + 2] * inv, x[4 * q4 + 3] * inv)};
                    *(u32x2 *)(stage + tile_off_row(li, 4 * mi + q4) + 8 * g) = pk;
                }
            __bf16 *op = (__bf16 *)a.o.ptr + obase;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int orow = r * 8 + lrow;
                const int tok = slot_token(a, wy, wx, q0 + 32 * nt + orow);
                const u32x4 val = *(const u32x4 *)(stage + tile_off_row(orow, lchunk));
                if (tok >= 0) st_stream((u32x4 *)(op + (long long)tok * a.o.sn + lchunk * 8), val);
            }
        } else {
            float *op = (float *)a.o.ptr + obase;
            const int tok = slot_token(a, wy, wx, q0 + 32 * nt + li);
            if (tok >= 0) {
#pragma unroll
                for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4) {
                        const f32x16 &x = w.acc[mi][nt];
                        f32x4 val = {x[4 * q4] * inv, x[4 * q4 + 1] * inv, x[4 * q4 + 2] * inv,
                                     x[4 * q4 + 3] * inv};
                        *(f32x4 *)(op + (long long)tok * a.o.sn + 32 * mi + 8 * q4 + 4 * g) = val;
                    }
            }
        }
    }
}

// Query operands (B of S^T = K Q^T): lane holds channels 16*ks + 8g .. +7 of query li.  Padding
// slots fetch token 0 of the slice (their columns are computed and never stored).  The loads
// are written in assembly: the compiler, which cannot tell which of the loads in flight write
// LDS, would otherwise wait for all of them before the first use of a query register, inside
// the key loop.  They are the oldest loads of the wavefront, so any wait for a later load
// covers them; the caller puts queries_landed() behind that wait.
template <int NT>
__device__ inline void load_queries(u32x4 (&qreg)[NT][4], const AttnArgs &a, int wy, int wx,
                                    int q0, long long qbase, int lane) {
    const int g = lane >> 5, li = lane & 31;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int tok = max(slot_token(a, wy, wx, q0 + 32 * nt + li), 0);
        const __bf16 *row = (const __bf16 *)a.q.ptr + qbase + (long long)tok * a.q.sn + g * 8;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
            asm volatile("global_load_dwordx4 %0, %1, off offset:%2" : "=v"(qreg[nt][ks]) : "v"(row), "n"(32 * ks));
    }
}
// Nothing that uses the query registers may be scheduled above this point (no instruction).
template <int NT>
__device__ inline void queries_landed(u32x4 (&qreg)[NT][4]) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
        asm volatile("" : "+v"(qreg[nt][0]), "+v"(qreg[nt][1]), "+v"(qreg[nt][2]), "+v"(qreg[nt][3]));
}

// ---------------------------------------------------------------------------------------
// Streaming kernel: any window size, including the whole grid (full attention).
// A workgroup holds 128*NT consecutive query slots of one window (4 waves x 32*NT) and streams
// the window's keys through LDS in double-buffered stages of 64.
// grid ring_grid(a, 128 * NT): one workgroup per (block of 128 * NT query slots, window, batch * head); 256 threads.
// ---------------------------------------------------------------------------------------
constexpr int kStage = 64;
constexpr int kStageBytes = 2 * kStage * 128;  // K rows then V rows

template <bool O_BF16, int NT>
__global__ void __launch_bounds__(256, JV_ATTN_MINW) attn_stream_bf16(AttnArgs a) {
    // the logit scale, fetched (a kernel argument) and waited for here, not inside the key loop
    float c_log2 = a.c;
    asm volatile("" : "+s"(c_log2));
    __shared__ __align__(16) unsigned char smem[2 * kStageBytes];
    __shared__ __align__(16) float bias[2][kStage];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    RingItem it;
    if (!ring_item(a, 128 * NT, it)) return;  // whole workgroup
    const int bh = it.bh, b = bh / a.heads, h = bh % a.heads;
    const int win = it.win, wy = win / a.g.wins_x, wx = win % a.g.wins_x;
    const int q0 = it.qblock * (128 * NT) + wave * (32 * NT);
    const long long qbase = b * a.q.sb + h * a.q.sh, kbase = b * a.k.sb + h * a.k.sh;
    const long long vbase = b * a.v.sb + h * a.v.sh, obase = b * a.o.sb + h * a.o.sh;
    const bool wave_live = q0 < a.q_slots;

    u32x4 qreg[NT][4];
    load_queries<NT>(qreg, a, wy, wx, q0, qbase, lane);
    WaveState<NT> w;
    wave_state_init<NT>(w);

    // Is any key slot of this window padding?  (Stages past the last slot are handled below.)
    const bool ragged = (wy + 1) * a.g.wh > a.g.H || (wx + 1) * a.g.ww > a.g.W;
    const int n_stage = (a.g.slots + kStage - 1) / kStage;
    const int lrow = tid >> 3, lchunk = tid & 7;
    // This thread moves rows lrow and lrow + 32 of every stage.
    const char *kbytes = (const char *)((const __bf16 *)a.k.ptr + kbase);
    const char *vbytes = (const char *)((const __bf16 *)a.v.ptr + vbase);
    u32x4 kreg[2], vreg[2];
    bool live[2];
    auto fetch = [&](int stage) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int tok = slot_token(a, wy, wx, stage * kStage + lrow + 32 * i);
            live[i] = tok >= 0;
            if (live[i]) {
                kreg[i] = *(const u32x4 *)(kbytes + 2 * ((long long)tok * a.k.sn + lchunk * 8));
                vreg[i] = *(const u32x4 *)(vbytes + 2 * ((long long)tok * a.v.sn + lchunk * 8));
            }
        }
    };
    auto stash = [&](int buf) {
        unsigned char *kt = smem + buf * kStageBytes, *vt = kt + kStage * 128;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int row = lrow + 32 * i;
            if (!live[i]) {  // padding rows are zero in LDS and carry a -inf bias
                u32x4 zero = {0u, 0u, 0u, 0u};
                kreg[i] = zero;
                vreg[i] = zero;
            }
            *(u32x4 *)(kt + tile_off_row(row, lchunk)) = kreg[i];
            *(u32x4 *)(vt + tile_off_tr(row, lchunk)) = vreg[i];
            if (lchunk == 0) bias[buf][row] = live[i] ? 0.f : -INFINITY;
        }
    };
    const unsigned vaddr[2] = {vt_lane_address(smem + kStage * 128, 0, lane),
                               vt_lane_address(smem + kStage * 128, 1, lane)};  // V rows of buffer 0
    unsigned kaddr[4];
    k_lane_addresses(kaddr, smem, lane);  // K rows of buffer 0
    // One stage: prefetch the next one, run the two tiles of this one, publish the next one.
    // `buf` is a compile-time constant so that every LDS offset folds into the instruction.
    auto run_stage = [&](int st, auto buf_tag) {
        constexpr int buf = decltype(buf_tag)::value;
        const bool more = st + 1 < n_stage;
        if (more) fetch(st + 1);
        if (wave_live) {
            const bool masked = ragged || (st + 1) * kStage > a.g.slots;
            u32x4 ka[4];
            load_k_operands<buf * kStageBytes>(ka, kaddr);
            k_operands_landed(ka);
            attn_tile32<NT, buf * kStageBytes + 32 * 128, buf * kStageBytes>(
                w, qreg, ka, kaddr, vaddr, masked ? &bias[buf][0] : nullptr, c_log2, lane);
            attn_tile32<NT, -1, buf * kStageBytes + 32 * 128>(
                w, qreg, ka, kaddr, vaddr, masked ? &bias[buf][32] : nullptr, c_log2, lane);
        }
        if (more) stash(buf ^ 1);
        __syncthreads();
    };

    fetch(0);
    stash(0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the queries (the first stage has been waited for already)
    queries_landed<NT>(qreg);
    __syncthreads();
    for (int st = 0; st < n_stage; st += 2) {
        run_stage(st, std::integral_constant<int, 0>());
        if (st + 1 < n_stage) run_stage(st + 1, std::integral_constant<int, 1>());
    }
    if (wave_live) {
        AttnArgs st = a;
        st.g.slots = a.q_slots;  // query slots past the limit are not stored
        wave_store<O_BF16, NT>(w, st, wy, wx, q0, obase, smem + wave * 4096, lane);
    }
}

// ---------------------------------------------------------------------------------------
// Window-resident kernel: windows of at most 64*WPW slots (WPW = wavefronts per window).
// All keys and values of a window are brought into LDS once, then every wavefront runs its 64
// query slots over the resident tiles.  WPW = 4: one workgroup per window (e.g. 16x16
// windows); WPW = 1: one wavefront per window, four windows per workgroup (e.g. 8x8 windows).
// Window attention moves 4 rows of 128 bytes per token and does little arithmetic on them, so
// the point of this kernel is to have many bytes in flight and to start early: the loads of
// the whole window (64 KB for 256 slots) are issued up front, from global memory straight
// into LDS with no register staging, tile by tile; a wavefront starts on key tile j as soon
// as tiles j and j+1 have landed (counted wait, then the barrier of the wavefronts that share
// the window), so the arithmetic of the early tiles runs under the loads of the late ones.
// grid (ceil(n_win * WPW / 4), B*heads), 256 threads, kWindowLds bytes of dynamic LDS.
// ---------------------------------------------------------------------------------------
constexpr int kWindowLds = 4 * (2 * 64 * 128 + 64 * 4);

typedef __attribute__((address_space(1))) const void attn_global_cvoid;
typedef __attribute__((address_space(3))) void attn_lds_void;

// Wait until at most `pending` of this wavefront's vector-memory loads are outstanding
// (the count is an immediate; values are rounded down to a supported one).
__device__ inline void wait_vm_loads(int pending) {
    if (pending >= 24) asm volatile("s_waitcnt vmcnt(24)" ::: "memory");
    else if (pending >= 16) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
    else if (pending >= 12) asm volatile("s_waitcnt vmcnt(12)" ::: "memory");
    else if (pending >= 10) asm volatile("s_waitcnt vmcnt(10)" ::: "memory");
    else if (pending >= 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    else if (pending >= 6) asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
    else if (pending >= 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
    else if (pending >= 2) asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

template <bool O_BF16, int WPW>
__global__ void __launch_bounds__(256, 2) attn_window_bf16(AttnArgs a) {
    // the logit scale, fetched (a kernel argument) and waited for here, not inside the key loop
    float c_log2 = a.c;
    asm volatile("" : "+s"(c_log2));
    extern __shared__ __align__(16) unsigned char wsm[];
    constexpr int R = 64 * WPW;       // LDS rows per window
    constexpr int kIpt = 4 / WPW;     // load instructions per tile, tensor and wavefront (8 rows each)
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int bh = blockIdx.y, b = bh / a.heads, h = bh % a.heads;
    const int win = WPW == 4 ? blockIdx.x : blockIdx.x * 4 + wave;
    const bool win_live = win < a.g.n_win;  // WPW == 1: the last workgroup may have idle waves
    const int wy = win_live ? win / a.g.wins_x : 0, wx = win_live ? win % a.g.wins_x : 0;
    unsigned char *ktile = wsm + (WPW == 4 ? 0 : wave * (2 * 64 * 128));
    unsigned char *vtile = ktile + R * 128;
    float *bias = (float *)(wsm + 4 * 2 * 64 * 128) + (WPW == 4 ? 0 : wave * 64);
    const int ww = WPW == 4 ? wave : 0;  // this wavefront's share of the window's rows
    const int q0 = WPW == 4 ? wave * 64 : 0;
    const long long qbase = b * a.q.sb + h * a.q.sh, kbase = b * a.k.sb + h * a.k.sh;
    const long long vbase = b * a.v.sb + h * a.v.sh, obase = b * a.o.sb + h * a.o.sh;
    const int n_tile = (a.g.slots + 31) >> 5;
    const bool wave_live = win_live && q0 < a.g.slots;

    u32x4 qreg[2][4];
    if (wave_live) load_queries<2>(qreg, a, wy, wx, q0, qbase, lane);

    // Loads, tile by tile: lane = 8 * (row in the group of 8) + 16-byte slot of the LDS row; it
    // fetches the chunk of the token's K (V) row that belongs in that slot under the tile
    // layouts.  Every wavefront issues the same number of loads whatever the padding (the
    // waits below count them): a padding row fetches the window's first token, which is always
    // real, and is kept out of the softmax by its -inf bias (its values meet zero weights).
    if (win_live) {
        const __bf16 *kptr = (const __bf16 *)a.k.ptr + kbase;
        const __bf16 *vptr = (const __bf16 *)a.v.ptr + vbase;
        const int lrow = lane >> 3, lslot = lane & 7;
        const int tok_first = slot_token(a, wy, wx, 0);
        for (int j = 0; j < n_tile; ++j) {
#pragma unroll
            for (int i = 0; i < kIpt; ++i) {
                const int row0 = 32 * j + 8 * (i * WPW + ww), row = row0 + lrow;
                const int tok = slot_token(a, wy, wx, row);
                const int src = tok >= 0 ? tok : tok_first;
                const int kchunk = lslot ^ tile_row_rotation(row);
                const int vchunk = lslot ^ (((row ^ (row >> 1)) & 1) << 2);
                __builtin_amdgcn_global_load_lds(
                    (attn_global_cvoid *)(kptr + (long long)src * a.k.sn + kchunk * 8),
                    (attn_lds_void *)(ktile + row0 * 128), 16, 0, kDmaStreamAux);
                __builtin_amdgcn_global_load_lds(
                    (attn_global_cvoid *)(vptr + (long long)src * a.v.sn + vchunk * 8),
                    (attn_lds_void *)(vtile + row0 * 128), 16, 0, kDmaStreamAux);
                if (lslot == 0) bias[row] = tok >= 0 ? 0.f : -INFINITY;
            }
        }
    }
    // Tiles 0 .. upto have landed for every wavefront of the window.
    auto tiles_ready = [&](int upto) {
        wait_vm_loads(2 * kIpt * max(n_tile - 1 - upto, 0));
        if (WPW == 4) lds_barrier();
        else __builtin_amdgcn_wave_barrier();
    };

    WaveState<2> w;
    wave_state_init<2>(w);
    const bool ragged = (wy + 1) * a.g.wh > a.g.H || (wx + 1) * a.g.ww > a.g.W;
    tiles_ready(0);
    queries_landed<2>(qreg);  // (older than the loads of tile 0)
    const unsigned vaddr[2] = {vt_lane_address(vtile, 0, lane), vt_lane_address(vtile, 1, lane)};
    unsigned kaddr[4];
    k_lane_addresses(kaddr, ktile, lane);
    u32x4 ka[4];
    load_k_operands<0>(ka, kaddr);
    k_operands_landed(ka);
    // The tile loop, unrolled so that every LDS offset is a constant of the instruction.  While
    // tile j is multiplied the K operands of tile j + 1 are read (it has landed); after the
    // window's last tile that read fetches bytes nobody uses (rows of the V tile).
    auto run_tile = [&](auto tile_tag) __attribute__((always_inline)) {
        constexpr int tile = decltype(tile_tag)::value;
        if (tile >= n_tile) return;  // uniform
        if (tile + 1 < n_tile) tiles_ready(tile + 1);  // all wavefronts of the workgroup take part
        if (wave_live) {
            const bool masked = ragged || 32 * (tile + 1) > a.g.slots;
            attn_tile32<2, (tile + 1) * 32 * 128, tile * 32 * 128>(w, qreg, ka, kaddr, vaddr,
                                                                   masked ? bias + 32 * tile : nullptr, c_log2, lane);
        }
    };
    run_tile(std::integral_constant<int, 0>());
    run_tile(std::integral_constant<int, 1>());
    if (WPW == 4) {
        run_tile(std::integral_constant<int, 2>());
        run_tile(std::integral_constant<int, 3>());
        run_tile(std::integral_constant<int, 4>());
        run_tile(std::integral_constant<int, 5>());
        run_tile(std::integral_constant<int, 6>());
        run_tile(std::integral_constant<int, 7>());
    }
    if (WPW == 4) __syncthreads();  // all waves are done with the tiles: reuse them as staging
    else __builtin_amdgcn_wave_barrier();
    if (wave_live)
        wave_store<O_BF16, 2>(w, a, wy, wx, q0, obase, ktile + (WPW == 4 ? wave * 4096 : 0), lane);
}

// ---------------------------------------------------------------------------------------
// Window-resident kernel for 256-slot windows on grids the window divides (e.g. 16x16 windows
// on a 64x64 grid): one window per workgroup at a time, software-pipelined ACROSS windows so
// that loads are in flight the whole time.  A persistent workgroup walks over its windows; the
// two halves of the K/V tiles (key tiles 0-3 = half A, 4-7 = half B) are refilled for the next
// window as soon as the current window is done with them:
//     window start:   loads of half B (this window) are issued; half A is already in LDS
//     tiles 0-3       (half A)
//     middle:         wait for half B; barrier; issue half A of the NEXT window
//     tiles 4-7       (half B)
//     window end:     wait for the next window's half A; barrier; fetch the next window's
//                     queries; normalise and store through staging bytes in half B; barrier
// Both waits are "everything this wavefront has issued" (vmcnt 0): what is outstanding at
// those points beyond the awaited loads are only stores and loads issued half a window
// earlier.  Everything that depends on the lane but not on the window (which token of the
// window a lane loads or stores, as a byte offset from the window's first token) is computed
// once, so that a window switch costs a handful of scalar operations.
// grid (min(windows * B*heads, 512)), 256 threads, 64 KB of dynamic LDS.
// Requires: slots == 256, grid_h % win_h == 0, grid_w % win_w == 0, and byte offsets inside a
// window below 2^31 (checked by the launcher).
// ---------------------------------------------------------------------------------------
constexpr int kWindow8Lds = 2 * 256 * 128;

template <bool O_BF16>
__global__ void __launch_bounds__(256, 2) attn_window8_bf16(AttnArgs a, int n_items) {
    // the logit scale, fetched (a kernel argument) and waited for here, not inside the key loop
    float c_log2 = a.c;
    asm volatile("" : "+s"(c_log2));
    extern __shared__ __align__(16) unsigned char wsm[];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 5, li = lane & 31;
    unsigned char *ktile = wsm, *vtile = wsm + 256 * 128;
    const int lrow = lane >> 3, lslot = lane & 7;
    const int q0 = wave * 64;
    const int esz_o = O_BF16 ? 2 : 4;

    // token of window slot `row`, relative to the window's first token (256 slots: the window
    // width is a power of two)
    const int ww_shift = __builtin_ctz(a.g.ww);
    auto rel_token = [&](int row) { return (row >> ww_shift) * a.g.W + (row & (a.g.ww - 1)); };
    // K/V loads: byte offset of this lane's 16 bytes in key tile 0.  Key tile j starts at window
    // slot 32 j, and a tile never straddles a window row unevenly (the window width is a power of
    // two: either whole rows make up a tile, or a tile lies inside one row), so tile j is tile 0
    // moved by rel_token(32 j) tokens, the same for every lane; the chunk rotations repeat every
    // 16 rows.
    const int row_kv = 8 * wave + lrow;
    const unsigned koff0 = 2u * ((unsigned)rel_token(row_kv) * (unsigned)a.k.sn + (lslot ^ tile_row_rotation(row_kv)) * 8);
    const unsigned voff0 = 2u * ((unsigned)rel_token(row_kv) * (unsigned)a.v.sn + (lslot ^ (((row_kv ^ (row_kv >> 1)) & 1) << 2)) * 8);
    const unsigned ksn2 = 2u * (unsigned)a.k.sn, vsn2 = 2u * (unsigned)a.v.sn;

    struct Item {
        const char *q, *k, *v;
        char *o;
    };
    auto make_item = [&](int item) {
        const int bh = item / a.g.n_win, win = item % a.g.n_win, b = bh / a.heads, h = bh % a.heads;
        const long long origin = (long long)(win / a.g.wins_x) * a.g.wh * a.g.W + (win % a.g.wins_x) * a.g.ww;
        // the bases are the same in every lane: say so, and the loads take them as scalar bases
        auto uniform = [](const char *ptr) {
            const unsigned long long u = (unsigned long long)ptr;
            const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)u);
            const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(u >> 32));
            return (const char *)(((unsigned long long)hi << 32) | lo);
        };
        Item it;
        it.q = uniform((const char *)a.q.ptr + 2 * (b * a.q.sb + h * a.q.sh + origin * a.q.sn));
        it.k = uniform((const char *)a.k.ptr + 2 * (b * a.k.sb + h * a.k.sh + origin * a.k.sn));
        it.v = uniform((const char *)a.v.ptr + 2 * (b * a.v.sb + h * a.v.sh + origin * a.v.sn));
        it.o = (char *)uniform((const char *)a.o.ptr + esz_o * (b * a.o.sb + h * a.o.sh + origin * a.o.sn));
        return it;
    };
    auto issue_half = [&](const Item &it, int half) {
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            const int j = 4 * half + jj, row0 = 32 * j + 8 * wave;
            const unsigned tile_tok = (unsigned)rel_token(32 * j);  // uniform
            __builtin_amdgcn_global_load_lds((attn_global_cvoid *)(it.k + (koff0 + tile_tok * ksn2)),
                                             (attn_lds_void *)(ktile + row0 * 128), 16, 0, kDmaStreamAux);
            __builtin_amdgcn_global_load_lds((attn_global_cvoid *)(it.v + (voff0 + tile_tok * vsn2)),
                                             (attn_lds_void *)(vtile + row0 * 128), 16, 0, kDmaStreamAux);
        }
    };
    u32x4 qreg[2][4];
    // `fresh` is zero, but opaque to the compiler: the offsets are then recomputed per window (a
    // few integer operations) instead of being kept, loop-invariant, in registers that the
    // loop does not have to spare (they were spilled to scratch memory and reloaded per window).
    auto load_q = [&](const Item &it, int fresh) {
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            const unsigned qoff = 2u * ((unsigned)rel_token(q0 + 32 * nt + li + fresh) * (unsigned)a.q.sn + g * 8);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)  // (in assembly, as in load_queries)
                asm volatile("global_load_dwordx4 %0, %1, %2 offset:%3"
                             : "=v"(qreg[nt][ks]) : "v"(qoff), "s"(it.q), "n"(32 * ks)
                             : "memory");  // the stores and loads counted below stay behind it
        }
    };
    // Vector-memory operations a wavefront issues per window after its query loads: the output
    // stores, then the loads of half B.  (Loads and stores complete in issue order.)
    constexpr int kAfterQueries = (O_BF16 ? 8 : 16) + 8;
    auto drain_and_sync = [&]() {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        lds_barrier();
    };

    const unsigned vaddr[2] = {vt_lane_address(vtile, 0, lane), vt_lane_address(vtile, 1, lane)};
    unsigned kaddr[4];
    k_lane_addresses(kaddr, ktile, lane);
    int item = blockIdx.x;
    if (item >= n_items) return;  // whole workgroup
    Item cur = make_item(item);
    load_q(cur, 0);
    issue_half(cur, 0);
    drain_and_sync();
    for (;;) {
        issue_half(cur, 1);
        if (kAfterQueries == 16) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(24)" ::: "memory");
        queries_landed<2>(qreg);
        const int next = item + gridDim.x;
        const bool has_next = next < n_items;
        Item nxt = cur;
        WaveState<2> w;
        wave_state_init<2>(w);
        u32x4 ka[4];
        // (unrolled: every LDS offset is a constant of the instruction)
        auto run_tile = [&](auto tile_tag) __attribute__((always_inline)) {
            constexpr int tile = decltype(tile_tag)::value;
            if (tile == 4) {
                drain_and_sync();  // half B has landed; every wavefront is done with half A
                if (has_next) {
                    nxt = make_item(next);
                    issue_half(nxt, 0);
                }
            }
            if ((tile & 3) == 0) {
                load_k_operands<tile * 32 * 128>(ka, kaddr);
                k_operands_landed(ka);
            }
            attn_tile32<2, (tile & 3) != 3 ? (tile + 1) * 32 * 128 : -1, tile * 32 * 128>(w, qreg, ka, kaddr, vaddr,
                                                                                       nullptr, c_log2, lane);
        };
        run_tile(std::integral_constant<int, 0>());
        run_tile(std::integral_constant<int, 1>());
        run_tile(std::integral_constant<int, 2>());
        run_tile(std::integral_constant<int, 3>());
        run_tile(std::integral_constant<int, 4>());
        run_tile(std::integral_constant<int, 5>());
        run_tile(std::integral_constant<int, 6>());
        run_tile(std::integral_constant<int, 7>());
        drain_and_sync();  // the next window's half A has landed; half B is free
        int fresh = 0;
        asm volatile("" : "+v"(fresh));
        if (has_next) load_q(nxt, fresh);
        unsigned char *stage = ktile + 128 * 128 + wave * 4096;
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            float lo, hi;
            pair_values(w.l[nt], &lo, &hi);
            const float inv = __builtin_amdgcn_rcpf(lo + hi);
            if (O_BF16) {
#pragma unroll
                for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4) {
                        const f32x16 &x = w.acc[mi][nt];
                        u32x2 pk = {pack_bf16x2(x[4 * q4] * inv, x[4 * q4 + 1] * inv),
                                    pack_bf16x2(x[4 * q4 + 2] * inv, x[4 * q4 + 3] * inv)};
                        *(u32x2 *)(stage + tile_off_row(li, 4 * mi + q4) + 8 * g) = pk;
                    }
                // (read back in assembly, so that the compiler does not wait for the query loads
                // of the next window, which it cannot tell from loads that write LDS)
                u32x4 val[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) val[r] = lds_read_b128_ordered(lds_address(stage + tile_off_row(r * 8 + lrow, lslot)));
                lds_reads_landed(val[0], val[1], val[2], val[3]);
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const unsigned ooff = 2u * ((unsigned)rel_token(q0 + 32 * nt + r * 8 + lrow + fresh) * (unsigned)a.o.sn + lslot * 8);
                    st_stream((u32x4 *)(cur.o + ooff), val[r]);
                }
            } else {
                const unsigned ooff = 4u * (unsigned)rel_token(q0 + 32 * nt + li + fresh) * (unsigned)a.o.sn;
#pragma unroll
                for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4) {
                        const f32x16 &x = w.acc[mi][nt];
                        f32x4 val = {x[4 * q4] * inv, x[4 * q4 + 1] * inv, x[4 * q4 + 2] * inv,
                                     x[4 * q4 + 3] * inv};
                        *(f32x4 *)(cur.o + (ooff + 4 * (32 * mi + 8 * q4 + 4 * g))) = val;
                    }
            }
        }
        lds_barrier();  // staging bytes are read out: half B may be refilled (the stores drain on their own)
        if (!has_next) break;
        cur = nxt;
        item = next;
    }
}

// ---------------------------------------------------------------------------------------
// Streaming kernel for windows that span whole grid rows (full attention above all), with
// byte offsets inside one (batch, head) slice below 2^31 (checked by the launcher).
// Same tiling as attn_stream_bf16 (a workgroup holds 256 query slots, keys pass through LDS
// in stages of 64), but built so that the inner loop is nothing but matrix instructions,
// exponentials and LDS operand reads:
//   * K/V stages go from global memory straight into a ring of three LDS stages (no register
//     staging, no LDS stores, no per-row selects), two stages ahead of the arithmetic; a
//     stage costs each wavefront four load instructions, one wait and one barrier, which sit
//     between the stage's two tiles so that the K operands of the next stage's first tile are
//     read under this stage's second tile (a ring of four stages, three in flight and a
//     counted wait, measured 2 % slower);
//   * every full stage runs the unmasked tile code, which is one basic block per tile apart
//     from the (rarely taken) branch that raises the softmax reference; only the last,
//     partial stage of a window masks keys, and it does so by key index, not through LDS.
// grid ring_grid(a, 256): one workgroup per (block of 256 query slots, window, batch * head),
// dealt to the XCDs in contiguous ranges (ring_item); 256 threads.
// ---------------------------------------------------------------------------------------
constexpr int kRing = 3;

// One tile of 32 keys of the ring kernel, as attn_tile32: `ka` holds its K operands, its V rows
// are at vaddr + VOFF, and if KNEXT >= 0 the K operands at kaddr + KNEXT are read into `ka`
// under the exponentials.  MASKED: the tile's keys are keys krow0 .. +31 of their stage, and
// keys with index (inside the stage) >= key_limit are padding.
template <int KNEXT, bool MASKED, int VOFF>
__device__ __forceinline__ void ring_tile32(WaveState<2> &w, const u32x4 (&qreg)[2][4], u32x4 (&ka)[4],
                                   const unsigned (&kaddr)[4], const unsigned (&vaddr)[2],
                                   int krow0, int key_limit, float c, int lane) {
    const int g = lane >> 5;
    f32x16 s[2];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int v = 0; v < 16; ++v) s[nt][v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) s[nt] = mfma32(as_bf16x8(ka[ks]), as_bf16x8(qreg[nt][ks]), s[nt]);
    __builtin_amdgcn_sched_barrier(0);  // the score products are issued before the reads below
    u32x4 va[2][2];
    load_vt_operands<VOFF>(va, vaddr);
    if (KNEXT >= 0) load_k_operands<KNEXT >= 0 ? KNEXT : 0>(ka, kaddr);
    __builtin_amdgcn_sched_barrier(0);  // ... and the reads before the softmax arithmetic
    if (MASKED) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const bool pad = krow0 + 8 * (v / 4) + 4 * g + (v % 4) >= key_limit;
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) s[nt][v] = pad ? -INFINITY : s[nt][v];
        }
    }
    // Lazy softmax reference, as in attn_tile32, with one test for both query blocks.
    unsigned pk[2][8];
    float sum0 = exp_block(s[0], pk[0], c, -w.m[0]);
    float sum1 = exp_block(s[1], pk[1], c, -w.m[1]);
    if (__builtin_amdgcn_ballot_w64(!(sum0 <= kLazySum) || !(sum1 <= kLazySum)) != 0) {  // NaN too
        if (__builtin_amdgcn_ballot_w64(!(sum0 <= kLazySum)) != 0) {
            raise_reference<2>(w, 0, s[0], c);
            sum0 = exp_block(s[0], pk[0], c, -w.m[0]);
        }
        if (__builtin_amdgcn_ballot_w64(!(sum1 <= kLazySum)) != 0) {
            raise_reference<2>(w, 1, s[1], c);
            sum1 = exp_block(s[1], pk[1], c, -w.m[1]);
        }
    }
    w.l[0] += sum0;
    w.l[1] += sum1;
    if (KNEXT >= 0) lds_reads_landed(va[0], va[1], ka);
    else lds_reads_landed(va[0][0], va[0][1], va[1][0], va[1][1]);
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) {
                u32x4 pb = {pk[nt][4 * kk], pk[nt][4 * kk + 1], pk[nt][4 * kk + 2], pk[nt][4 * kk + 3]};
                w.acc[mi][nt] = mfma32(as_bf16x8(va[kk][mi]), as_bf16x8(pb), w.acc[mi][nt]);
            }
}

template <bool O_BF16>
__global__ void __launch_bounds__(256, 2) attn_ring_bf16(AttnArgs a) {
    // the logit scale, fetched (a kernel argument) and waited for here, not inside the key loop
    float c_log2 = a.c;
    asm volatile("" : "+s"(c_log2));
    __shared__ __align__(16) unsigned char smem[kRing * kStageBytes];
    constexpr int WAVES = 4;
    constexpr int kLoads = 8 / WAVES;  // load instructions per stage, tensor and wavefront (8 rows each)
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    RingItem it;
    if (!ring_item(a, 64 * WAVES, it)) return;  // whole workgroup
    const int bh = it.bh, b = bh / a.heads, h = bh % a.heads;
    const int win = it.win, wy = win / a.g.wins_x, wx = win % a.g.wins_x;
    const int q0 = it.qblock * (64 * WAVES) + wave * 64;
    const long long qbase = b * a.q.sb + h * a.q.sh, obase = b * a.o.sb + h * a.o.sh;
    const bool wave_live = q0 < a.q_slots;

    u32x4 qreg[2][4];
    load_queries<2>(qreg, a, wy, wx, q0, qbase, lane);
    WaveState<2> w;
    wave_state_init<2>(w);

    // Key slots of the window that hold tokens: slot s is token tok_first + s.
    const int tok_first = wy * a.g.wh * a.g.W;
    const int tok_limit = min(a.g.slots, a.g.H * a.g.W - tok_first);
    const int n_full = tok_limit / kStage, n_stage = (tok_limit + kStage - 1) / kStage;

    // Loads.  A wavefront moves rows 8 * (WAVES * i + wave) + lane / 8 (i < kLoads) of every
    // stage, K and V: lane = 8 * (row in the group of 8) + 16-byte slot of the LDS row, and it
    // fetches the chunk of the token's row that belongs in that slot under the tile layouts.
    // The number of loads per stage is the same for every wavefront and stage (the waits count
    // them); a row past the last token fetches the window's first token instead.  Stages are
    // issued in order, so the byte offsets just advance by one stage per issue.
    auto uniform = [](const char *ptr) {
        const unsigned long long u = (unsigned long long)ptr;
        const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)u);
        const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(u >> 32));
        return (const char *)(((unsigned long long)hi << 32) | lo);
    };
    const char *kbytes = uniform((const char *)((const __bf16 *)a.k.ptr + b * a.k.sb + h * a.k.sh + (long long)tok_first * a.k.sn));
    const char *vbytes = uniform((const char *)((const __bf16 *)a.v.ptr + b * a.v.sb + h * a.v.sh + (long long)tok_first * a.v.sn));
    const int lrow = lane >> 3, lslot = lane & 7;
    unsigned kcur[kLoads], vcur[kLoads], kpad[kLoads], vpad[kLoads];
#pragma unroll
    for (int i = 0; i < kLoads; ++i) {
        const int row = 8 * (WAVES * i + wave) + lrow;
        kpad[i] = 2u * ((lslot ^ tile_row_rotation(row)) * 8);
        vpad[i] = 2u * ((lslot ^ (((row ^ (row >> 1)) & 1) << 2)) * 8);
        kcur[i] = 2u * (unsigned)row * (unsigned)a.k.sn + kpad[i];
        vcur[i] = 2u * (unsigned)row * (unsigned)a.v.sn + vpad[i];
    }
    const unsigned kstep = 2u * kStage * (unsigned)a.k.sn, vstep = 2u * kStage * (unsigned)a.v.sn;
    auto issue = [&](int stage) {
        unsigned char *kt = smem + (stage % kRing) * kStageBytes, *vt = kt + kStage * 128;
        const bool whole = (stage + 1) * kStage <= tok_limit;  // uniform
#pragma unroll
        for (int i = 0; i < kLoads; ++i) {
            const int row0 = 8 * (WAVES * i + wave);
            unsigned ko = kcur[i], vo = vcur[i];
            if (!whole && stage * kStage + row0 + lrow >= tok_limit) {
                ko = kpad[i];
                vo = vpad[i];
            }
            __builtin_amdgcn_global_load_lds((attn_global_cvoid *)(kbytes + ko),
                                             (attn_lds_void *)(kt + row0 * 128), 16, 0, 0);
            __builtin_amdgcn_global_load_lds((attn_global_cvoid *)(vbytes + vo),
                                             (attn_lds_void *)(vt + row0 * 128), 16, 0, 0);
            kcur[i] += kstep;
            vcur[i] += vstep;
        }
    };
    static_assert(kLoads == 2 && (kRing == 3 || kRing == 4), "the waits below count 2 * kLoads loads per stage in flight");
    // Between the two tiles of stage st: stage st + 1 has landed for every wavefront (with a
    // ring of four, one more stage may be in flight), and every wavefront has left stage st - 1,
    // whose ring slot takes stage st + kRing - 1.  The second tile of stage st may then read the
    // first K operands of stage st + 1, so no tile waits for its operands at a stage boundary.
    auto next_stage_ready = [&](int st) {
        if (st + 1 >= n_stage) return;  // uniform
        if (kRing == 4 && st + 2 < n_stage) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        lds_barrier();
        if (st + kRing - 1 < n_stage) issue(st + kRing - 1);
    };
    const unsigned vaddr[2] = {vt_lane_address(smem + kStage * 128, 0, lane),
                               vt_lane_address(smem + kStage * 128, 1, lane)};  // V rows of ring slot 0
    unsigned kaddr[4];
    k_lane_addresses(kaddr, smem, lane);  // K rows of ring slot 0
    u32x4 ka[4];
    // A full stage in ring slot `slot` (a compile-time constant, so that every LDS offset is a
    // constant of the instruction).
    auto full_stage = [&](int st, auto slot_tag) {
        constexpr int slot = decltype(slot_tag)::value, after = (slot + 1) % kRing;
        if (wave_live)
            ring_tile32<slot * kStageBytes + 32 * 128, false, slot * kStageBytes>(w, qreg, ka, kaddr, vaddr, 0, 0, c_log2, lane);
        next_stage_ready(st);
        if (wave_live)  // (after the window's last stage the K operands read here are not used)
            ring_tile32<after * kStageBytes, false, slot * kStageBytes + 32 * 128>(w, qreg, ka, kaddr, vaddr, 32, 0, c_log2, lane);
    };

    if (n_stage > 0) issue(0);
    if (n_stage > 1) issue(1);
    if (kRing == 4 && n_stage > 2) issue(2);
    if (kRing == 4 && n_stage > 2) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    else if (n_stage > 1) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    lds_barrier();  // stage 0 has landed
    queries_landed<2>(qreg);  // (older than the loads of stage 0)
    load_k_operands<0>(ka, kaddr);
    k_operands_landed(ka);
    int st = 0;
    for (; st + kRing - 1 < n_full; st += kRing) {
        full_stage(st, std::integral_constant<int, 0>());
        full_stage(st + 1, std::integral_constant<int, 1>());
        full_stage(st + 2, std::integral_constant<int, 2>());
        if (kRing == 4) full_stage(st + 3, std::integral_constant<int, 3 % kRing>());
    }
    if (st < n_full) {
        full_stage(st, std::integral_constant<int, 0>());
        ++st;
        if (st < n_full) {
            full_stage(st, std::integral_constant<int, 1>());
            ++st;
            if (st < n_full) {
                full_stage(st, std::integral_constant<int, 2>());
                ++st;
            }
        }
    }
    if (st < n_stage && wave_live) {  // the partial stage that ends the window (its first K operands are in ka)
        const unsigned at = (st % kRing) * kStageBytes;
        const unsigned vlast[2] = {vaddr[0] + at, vaddr[1] + at};
        const unsigned klast[4] = {kaddr[0] + at, kaddr[1] + at, kaddr[2] + at, kaddr[3] + at};
        const int key_limit = tok_limit - st * kStage;  // 1 .. 63
        if (key_limit > 32) {
            ring_tile32<32 * 128, true, 0>(w, qreg, ka, klast, vlast, 0, key_limit, c_log2, lane);
            ring_tile32<-1, true, 32 * 128>(w, qreg, ka, klast, vlast, 32, key_limit, c_log2, lane);
        } else {
            ring_tile32<-1, true, 0>(w, qreg, ka, klast, vlast, 0, key_limit, c_log2, lane);
        }
    }
    __syncthreads();  // every wavefront is done with the ring: reuse it as staging
    if (wave_live) {
        AttnArgs st = a;
        st.g.slots = a.q_slots;  // query slots past the limit are not stored
        wave_store<O_BF16, 2>(w, st, wy, wx, q0, obase, smem + wave * 4096, lane);
    }
}

// ---------------------------------------------------------------------------------------
// A few queries against a whole sequence: the prefix tokens (at most 64, the first query slots
// of a one-window geometry whose slot s is token s) attend to all N tokens.  With so few
// queries the parallelism has to come from the keys: one workgroup of eight wavefronts per
// (batch, head); every wavefront holds all the queries, takes every eighth stage of 64 keys
// into a tile of its own (loads straight into LDS, no barriers in the loop) and keeps its own
// running softmax; at the end the eight partial results are merged through LDS,
//     O = sum_w acc_w 2^(m_w - M) / sum_w l_w 2^(m_w - M),   M = max_w m_w.
// grid (B*heads), 512 threads, kPrefixLds bytes of dynamic LDS.  Requirements as attn_ring_bf16.
// ---------------------------------------------------------------------------------------
constexpr int kPrefixWaves = 8;
constexpr int kPrefixLds = kPrefixWaves * kStageBytes + 2 * kPrefixWaves * 64 * 4;

template <bool O_BF16>
__global__ void __launch_bounds__(512, 1) attn_prefix_bf16(AttnArgs a) {
    // the logit scale, fetched (a kernel argument) and waited for here, not inside the key loop
    float c_log2 = a.c;
    asm volatile("" : "+s"(c_log2));
    extern __shared__ __align__(16) unsigned char psm[];
    const int tid = threadIdx.x, lane = tid & 63, g = lane >> 5, li = lane & 31;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int bh = blockIdx.x, b = bh / a.heads, h = bh % a.heads;
    const long long qbase = b * a.q.sb + h * a.q.sh;
    const int N = a.g.slots;

    u32x4 qreg[2][4];
    load_queries<2>(qreg, a, 0, 0, 0, qbase, lane);
    WaveState<2> w;
    wave_state_init<2>(w);

    auto uniform = [](const char *ptr) {
        const unsigned long long u = (unsigned long long)ptr;
        const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)u);
        const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(u >> 32));
        return (const char *)(((unsigned long long)hi << 32) | lo);
    };
    const char *kbytes = uniform((const char *)((const __bf16 *)a.k.ptr + b * a.k.sb + h * a.k.sh));
    const char *vbytes = uniform((const char *)((const __bf16 *)a.v.ptr + b * a.v.sb + h * a.v.sh));
    unsigned char *kt = psm + wave * kStageBytes, *vt = kt + kStage * 128;
    const int lrow = lane >> 3, lslot = lane & 7;
    const int n_stage = (N + kStage - 1) / kStage;
    for (int st = wave; st < n_stage; st += kPrefixWaves) {
        // (the LDS reads of the previous stage have been waited for before the matrix
        // instructions that used them, so the tile may be overwritten)
#pragma unroll 1
        for (int i = 0; i < 8; ++i) {
            const int row = 8 * i + lrow;
            const int tok = st * kStage + row < N ? st * kStage + row : 0;  // past the end: any valid row
            const unsigned ko = 2u * ((unsigned)tok * (unsigned)a.k.sn + (lslot ^ tile_row_rotation(row)) * 8);
            const unsigned vo = 2u * ((unsigned)tok * (unsigned)a.v.sn + (lslot ^ (((row ^ (row >> 1)) & 1) << 2)) * 8);
            __builtin_amdgcn_global_load_lds((attn_global_cvoid *)(kbytes + ko),
                                             (attn_lds_void *)(kt + 8 * i * 128), 16, 0, 0);
            __builtin_amdgcn_global_load_lds((attn_global_cvoid *)(vbytes + vo),
                                             (attn_lds_void *)(vt + 8 * i * 128), 16, 0, 0);
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        queries_landed<2>(qreg);
        const int key_limit = N - st * kStage;
        // The operand addresses depend on the lane only; `ln` is the lane, but opaque to the
        // compiler, which would otherwise keep every address of every tile variant in a
        // register of its own across the loop (and spill them).
        int ln = lane;
        asm volatile("" : "+v"(ln));
        const unsigned vaddr[2] = {vt_lane_address(vt, 0, ln), vt_lane_address(vt, 1, ln)};
        unsigned kaddr[4];
        k_lane_addresses(kaddr, kt, ln);
        u32x4 ka[4];
        load_k_operands<0>(ka, kaddr);
        k_operands_landed(ka);
        // (one masked tile code for whole and partial stages: this kernel waits for its loads,
        // not for its arithmetic)
        ring_tile32<32 * 128, true, 0>(w, qreg, ka, kaddr, vaddr, 0, key_limit, c_log2, ln);
        if (key_limit > 32) ring_tile32<-1, true, 32 * 128>(w, qreg, ka, kaddr, vaddr, 32, key_limit, c_log2, ln);
    }

    // Partial results into LDS: the accumulators as [query][channel] fp32 in the wavefront's own
    // tile bytes (16-byte pieces rotated by the query to spread the banks), references and sums
    // behind the tiles.
    float *mine = (float *)(psm + wave * kStageBytes);
    float *mbuf = (float *)(psm + kPrefixWaves * kStageBytes), *lbuf = mbuf + kPrefixWaves * 64;
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
        const int qcol = 32 * nt + li;
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const f32x16 &x = w.acc[mi][nt];
                f32x4 val = {x[4 * q4], x[4 * q4 + 1], x[4 * q4 + 2], x[4 * q4 + 3]};
                *(f32x4 *)(mine + qcol * 64 + (((8 * mi + 2 * q4 + g) ^ (qcol & 15)) << 2)) = val;
            }
        float lo, hi;
        pair_values(w.l[nt], &lo, &hi);
        if (g == 0) {
            mbuf[wave * 64 + qcol] = w.m[nt];
            lbuf[wave * 64 + qcol] = lo + hi;
        }
    }
    __syncthreads();
    // Merge: thread = (query, 8 channels).
    const int qcol = tid >> 3, piece = tid & 7;
    if (qcol < a.q_slots && qcol < N) {
        float top = kMinusHuge;
#pragma unroll
        for (int wv = 0; wv < kPrefixWaves; ++wv) top = fmaxf(top, mbuf[wv * 64 + qcol]);
        float den = 0.f;
        f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = s0;
#pragma unroll
        for (int wv = 0; wv < kPrefixWaves; ++wv) {
            const float scale = __builtin_amdgcn_exp2f(mbuf[wv * 64 + qcol] - top);
            den = fmaf(lbuf[wv * 64 + qcol], scale, den);
            const float *row = (const float *)(psm + wv * kStageBytes) + qcol * 64;
            const f32x4 x0 = *(const f32x4 *)(row + (((2 * piece) ^ (qcol & 15)) << 2));
            const f32x4 x1 = *(const f32x4 *)(row + (((2 * piece + 1) ^ (qcol & 15)) << 2));
            s0 += x0 * scale;
            s1 += x1 * scale;
        }
        const float inv = 1.0f / den;
        s0 *= inv;
        s1 *= inv;
        const long long at = b * a.o.sb + h * a.o.sh + (long long)qcol * a.o.sn + 8 * piece;
        if (O_BF16) {
            u32x4 pk = {pack_bf16x2(s0[0], s0[1]), pack_bf16x2(s0[2], s0[3]), pack_bf16x2(s1[0], s1[1]),
                        pack_bf16x2(s1[2], s1[3])};
            *(u32x4 *)((__bf16 *)a.o.ptr + at) = pk;
        } else {
            *(f32x4 *)((float *)a.o.ptr + at) = s0;
            *(f32x4 *)((float *)a.o.ptr + at + 4) = s1;
        }
    }
}

template <bool O_BF16>
static jv_status launch_prefix(const AttnArgs &a, int BH, hipStream_t stream) {
    static LdsLimit lds_limit;
    jv_status st = ensure_lds_limit(lds_limit, (const void *)attn_prefix_bf16<O_BF16>, kPrefixLds);
    if (st != JV_OK) return st;
    hipLaunchKernelGGL((attn_prefix_bf16<O_BF16>), dim3(BH), dim3(512), kPrefixLds, stream, a);
    return launch_status("attn_prefix_bf16");
}

template <bool O_BF16, int WPW>
static jv_status launch_window(const AttnArgs &a, int BH, hipStream_t stream) {
    static LdsLimit lds_limit;
    jv_status st = ensure_lds_limit(lds_limit, (const void *)attn_window_bf16<O_BF16, WPW>, kWindowLds);
    if (st != JV_OK) return st;
    dim3 grid((a.g.n_win * WPW + 3) / 4, BH);
    hipLaunchKernelGGL((attn_window_bf16<O_BF16, WPW>), grid, dim3(256), kWindowLds, stream, a);
    return launch_status("attn_window_bf16");
}

template <bool O_BF16>
static jv_status launch_window8(const AttnArgs &a, int BH, hipStream_t stream) {
    static LdsLimit lds_limit;
    jv_status st = ensure_lds_limit(lds_limit, (const void *)attn_window8_bf16<O_BF16>, kWindow8Lds);
    if (st != JV_OK) return st;
    const long long n_items = (long long)a.g.n_win * BH;
    if (n_items >= (1ll << 31)) return fail(JV_ERR_UNSUPPORTED, "too many windows");
    const int resident = 2 * 256;  // two workgroups per compute unit
    dim3 grid((unsigned)(n_items < resident ? n_items : resident));
    hipLaunchKernelGGL((attn_window8_bf16<O_BF16>), grid, dim3(256), kWindow8Lds, stream, a, (int)n_items);
    return launch_status("attn_window8_bf16");
}

// ---------------------------------------------------------------------------------------
// head_dim 128 (the wide heads of the paper's largest backbones): the streaming kernel that
// handles every geometry -- windows of any size, padded grids, a query-slot limit (and full
// attention; the launcher gives the geometries it can to attn_ring_wide_bf16, further down).
// Same algorithm as above with one block of 32 query columns per wavefront (NT = 1): a
// workgroup holds 128 consecutive query slots of one window (4 wavefronts x 32); the window's
// keys pass through LDS in double-buffered stages of 32 (K rows, then V rows, 256 bytes each;
// register-staged: the next stage is fetched before, and stored after, this stage's
// arithmetic).  Per stage a wavefront issues 8 matrix instructions for the scores (K = 128
// channels in steps of 16) and 8 for O^T += V^T P^T (four 32-channel blocks x two steps of 16
// keys) around the same softmax arithmetic as for 64 channels on half as many columns: the
// vector work per matrix instruction is half that of the 64-channel kernels.
// grid ring_grid(a, 128): one workgroup per (block of 128 query slots, window, batch * head); 256 threads.
// ---------------------------------------------------------------------------------------
constexpr int kStageWide = 32;
constexpr int kTileWideBytes = kStageWide * 256;    // the K rows or the V rows of a stage
constexpr int kStageWideBytes = 2 * kTileWideBytes;

struct WaveStateWide {
    f32x16 acc[4];  // channel blocks of 32
    float m, l;     // l is this lane's half of the keys only
};

__device__ inline void raise_reference_wide(WaveStateWide &w, const f32x16 &s, float c) {
    float t0 = fmaxf(fmaxf(s[0], s[1]), s[2]);
    float t1 = fmaxf(fmaxf(s[3], s[4]), s[5]);
    float t2 = fmaxf(fmaxf(s[6], s[7]), s[8]);
    float t3 = fmaxf(fmaxf(s[9], s[10]), s[11]);
    float t4 = fmaxf(fmaxf(s[12], s[13]), s[14]);
    t0 = fmaxf(fmaxf(t0, t1), t2);
    t3 = fmaxf(fmaxf(t3, t4), s[15]);
    float a, b;
    pair_values(fmaxf(t0, t3) * c, &a, &b);  // this lane and lane^32 share the query column
    const float m_new = fmaxf(w.m, fmaxf(a, b));
    const float alpha = __builtin_amdgcn_exp2f(w.m - m_new);
    w.m = m_new;
    w.l *= alpha;
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int v = 0; v < 16; ++v) w.acc[mi][v] *= alpha;
}

template <bool O_BF16>
__global__ void __launch_bounds__(256, 2) attn_wide_bf16(AttnArgs a) {
    __shared__ __align__(16) unsigned char smem[2 * kStageWideBytes];
    __shared__ __align__(16) float bias[2][kStageWide];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 5, li = lane & 31;
    RingItem it;
    if (!ring_item(a, 128, it)) return;  // whole workgroup
    const int bh = it.bh, b = bh / a.heads, h = bh % a.heads;
    const int win = it.win, wy = win / a.g.wins_x, wx = win % a.g.wins_x;
    const int q0 = it.qblock * 128 + wave * 32;
    const long long qbase = b * a.q.sb + h * a.q.sh, kbase = b * a.k.sb + h * a.k.sh;
    const long long vbase = b * a.v.sb + h * a.v.sh, obase = b * a.o.sb + h * a.o.sh;
    const bool wave_live = q0 < a.q_slots;
    const float c_log2 = a.c;

    // Query operands (B of S^T = K Q^T): channels 16*ks + 8g .. +7 of query li; padding slots
    // fetch token 0 of the slice (their columns are computed and never stored).
    u32x4 qreg[8];
    {
        const int tok = max(slot_token(a, wy, wx, q0 + li), 0);
        const __bf16 *row = (const __bf16 *)a.q.ptr + qbase + (long long)tok * a.q.sn + g * 8;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qreg[ks] = *(const u32x4 *)(row + 16 * ks);
    }
    WaveStateWide w;
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int v = 0; v < 16; ++v) w.acc[mi][v] = 0.f;
    w.m = kMinusHuge;
    w.l = 0.f;

    const bool ragged = (wy + 1) * a.g.wh > a.g.H || (wx + 1) * a.g.ww > a.g.W;
    const int n_stage = (a.g.slots + kStageWide - 1) / kStageWide;
    // This thread moves chunks lchunk and lchunk + 8 of row lrow of every stage's K and V.
    const int lrow = tid >> 3, lchunk = tid & 7;
    const char *kbytes = (const char *)((const __bf16 *)a.k.ptr + kbase);
    const char *vbytes = (const char *)((const __bf16 *)a.v.ptr + vbase);
    u32x4 kreg[2], vreg[2];
    bool live = false;
    auto fetch = [&](int stage) {
        const int tok = slot_token(a, wy, wx, stage * kStageWide + lrow);
        live = tok >= 0;
        if (live) {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                kreg[i] = *(const u32x4 *)(kbytes + 2 * ((long long)tok * a.k.sn + (lchunk + 8 * i) * 8));
                vreg[i] = *(const u32x4 *)(vbytes + 2 * ((long long)tok * a.v.sn + (lchunk + 8 * i) * 8));
            }
        }
    };
    auto stash = [&](int buf) {
        unsigned char *kt = smem + buf * kStageWideBytes, *vt = kt + kTileWideBytes;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            if (!live) {  // padding rows are zero in LDS and carry a -inf bias
                u32x4 zero = {0u, 0u, 0u, 0u};
                kreg[i] = zero;
                vreg[i] = zero;
            }
            *(u32x4 *)(kt + wide_off_row(lrow, lchunk + 8 * i)) = kreg[i];
            *(u32x4 *)(vt + wide_off_tr(lrow, lchunk + 8 * i)) = vreg[i];
        }
        if (lchunk == 0) bias[buf][lrow] = live ? 0.f : -INFINITY;
    };
    // The 32 keys of the stage in buffer `buf`.
    auto tile = [&](int buf, bool masked) {
        const unsigned char *kt = smem + buf * kStageWideBytes, *vt = kt + kTileWideBytes;
        f32x16 s;
#pragma unroll
        for (int v = 0; v < 16; ++v) s[v] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const u32x4 ka = *(const u32x4 *)(kt + wide_off_row(li, 2 * ks + g));
            s = mfma32(as_bf16x8(ka), as_bf16x8(qreg[ks]), s);
        }
        if (masked) add_key_bias(s, &bias[buf][0], g);
        unsigned pk[8];
        float tile_sum = exp_block(s, pk, c_log2, -w.m);
        if (__builtin_amdgcn_ballot_w64(!(tile_sum <= kLazySum)) != 0) {  // also catches inf/NaN
            raise_reference_wide(w, s, c_log2);
            tile_sum = exp_block(s, pk, c_log2, -w.m);
        }
        w.l += tile_sum;
        // A of O^T += V^T P^T: lane = channel of a 32-block, k-slot (g, 4r + e) = key 16*kk + 8r + 4g + e
        const int blk = lane >> 4, j = lane & 15;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            const u32x4 pb = {pk[4 * kk], pk[4 * kk + 1], pk[4 * kk + 2], pk[4 * kk + 3]};
#pragma unroll
            for (int mi = 0; mi < 4; ++mi) {
                const int chunk16 = mi * 4 + (blk & 1) * 2 + ((j & 3) >> 1);
                const int row0 = 16 * kk + 4 * g + (j >> 2);
                const u32x2 r0 = lds_read_tr16(vt + wide_off_tr(row0, chunk16) + (j & 1) * 8);
                const u32x2 r1 = lds_read_tr16(vt + wide_off_tr(row0 + 8, chunk16) + (j & 1) * 8);
                const u32x4 va = {r0[0], r0[1], r1[0], r1[1]};
                w.acc[mi] = mfma32(as_bf16x8(va), as_bf16x8(pb), w.acc[mi]);
            }
        }
    };

    fetch(0);
    stash(0);
    __syncthreads();
    for (int st = 0; st < n_stage; ++st) {
        const int buf = st & 1;
        const bool more = st + 1 < n_stage;
        if (more) fetch(st + 1);
        if (wave_live) tile(buf, ragged || (st + 1) * kStageWide > a.g.slots);
        if (more) stash(buf ^ 1);
        __syncthreads();
    }
    if (!wave_live) return;  // (no barrier follows)

    // Normalise and store this wavefront's 32 query columns.
    float lo, hi;
    pair_values(w.l, &lo, &hi);
    const float inv = __builtin_amdgcn_rcpf(lo + hi);
    if (O_BF16) {
        // channel-major accumulators -> token rows of 256 bytes through 8 KB of wave-private LDS
        unsigned char *stage = smem + wave * kTileWideBytes;
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const f32x16 &x = w.acc[mi];
                u32x2 pk = {pack_bf16x2(x[4 * q4] * inv, x[4 * q4 + 1] * inv),
                            pack_bf16x2(x[4 * q4 + 2] * inv, x[4 * q4 + 3] * inv)};
                *(u32x2 *)(stage + wide_off_row(li, 4 * mi + q4) + 8 * g) = pk;
            }
        __bf16 *op = (__bf16 *)a.o.ptr + obase;
        const int orow = lane >> 4, ochunk = lane & 15;
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int row = 4 * r + orow;
            const int slot = q0 + row;
            const int tok = slot < a.q_slots ? slot_token(a, wy, wx, slot) : -1;
            const u32x4 val = *(const u32x4 *)(stage + wide_off_row(row, ochunk));
            if (tok >= 0) *(u32x4 *)(op + (long long)tok * a.o.sn + ochunk * 8) = val;
        }
    } else {
        float *op = (float *)a.o.ptr + obase;
        const int slot = q0 + li;
        const int tok = slot < a.q_slots ? slot_token(a, wy, wx, slot) : -1;
        if (tok >= 0) {
#pragma unroll
            for (int mi = 0; mi < 4; ++mi)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    const f32x16 &x = w.acc[mi];
                    f32x4 val = {x[4 * q4] * inv, x[4 * q4 + 1] * inv, x[4 * q4 + 2] * inv, x[4 * q4 + 3] * inv};
                    *(f32x4 *)(op + (long long)tok * a.o.sn + 32 * mi + 8 * q4 + 4 * g) = val;
                }
        }
    }
}

// ---------------------------------------------------------------------------------------
// head_dim 128, windows whose key slots are a fixed-step walk through memory -- windows of whole
// grid rows (full attention above all) and unpadded windows whose width divides the 32-key
// stage (a stage is then 32 / ww whole window rows) --: the ring design of attn_ring_bf16 on
// 256-byte rows.  A workgroup holds 128 query slots (4 wavefronts x 32);
// the keys pass through a ring of three LDS stages of one tile each (32 keys: 8 KB of K rows,
// 8 KB of V rows), filled from global memory straight into LDS two stages ahead (four load
// instructions per stage and wavefront, one wait, one barrier).  Inside a tile: the eight
// score products; then -- behind them -- the wait for the next stage, the barrier and the loads
// of the stage after it; the LDS reads of this tile's V operands and of the next tile's K
// operands (in assembly, see lds_read_tr16_at); the softmax arithmetic, which hides their
// latency; one wait; the eight P.V products.  Byte offsets inside one (batch, head) slice
// below 2^31 (checked by the launcher).
// grid ring_grid(a, 128): one workgroup per (block of 128 query slots, window, batch * head),
// dealt to the XCDs in contiguous ranges (ring_item); 256 threads.
// ---------------------------------------------------------------------------------------
#ifndef JV_WIDE_RING
#define JV_WIDE_RING 3  // stages in the ring: 3, or 4 (one more stage in flight; measured the same time)
#endif
constexpr int kWideRing = JV_WIDE_RING;
static_assert(kWideRing == 3 || kWideRing == 4, "the waits of attn_ring_wide_bf16 count the loads of 3 or 4 stages");

// The wavefront's LDS operand addresses for ring slot 0: K pieces (channels 16 ks + 8 g .. +7 of
// key row li) and the first transposing V read of each 32-channel block.
__device__ inline void wide_lane_addresses(unsigned (&kaddr)[8], unsigned (&vaddr)[4], const unsigned char *ring, int lane) {
    const int g = lane >> 5, li = lane & 31, blk = lane >> 4, j = lane & 15;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) kaddr[ks] = lds_address(ring) + wide_off_row(li, 2 * ks + g);
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
        vaddr[mi] = lds_address(ring + kTileWideBytes) + wide_off_tr(4 * g + (j >> 2), mi * 4 + (blk & 1) * 2 + ((j & 3) >> 1)) + (j & 1) * 8;
}

template <int OFF>
__device__ inline void wide_load_k(u32x4 (&ka)[8], const unsigned (&kaddr)[8]) {
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) ka[ks] = lds_read_b128_at<OFF>(kaddr[ks]);
}
// va[kk][mi]: keys 16 kk + 8 r + 4 g + e in k-slot (g, 4 r + e); rows 8 apart keep their rotation,
// so the four reads of a block are constant offsets from one address.
template <int OFF>
__device__ inline void wide_load_v(u32x4 (&va)[2][4], const unsigned (&vaddr)[4]) {
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
        for (int mi = 0; mi < 4; ++mi) {
            u32x2 r0, r1;
            if (kk == 0) {
                r0 = lds_read_tr16_at<OFF>(vaddr[mi]);
                r1 = lds_read_tr16_at<OFF + 2048>(vaddr[mi]);
            } else {
                r0 = lds_read_tr16_at<OFF + 4096>(vaddr[mi]);
                r1 = lds_read_tr16_at<OFF + 6144>(vaddr[mi]);
            }
            const u32x4 r = {r0[0], r0[1], r1[0], r1[1]};
            va[kk][mi] = r;
        }
}
__device__ inline void wide_reads_landed(u32x4 (&va)[2][4], u32x4 (&ka)[8]) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(va[0][0]), "+v"(va[0][1]), "+v"(va[0][2]), "+v"(va[0][3]), "+v"(va[1][0]), "+v"(va[1][1]),
                   "+v"(va[1][2]), "+v"(va[1][3]), "+v"(ka[0]), "+v"(ka[1]), "+v"(ka[2]), "+v"(ka[3]), "+v"(ka[4]),
                   "+v"(ka[5]), "+v"(ka[6]), "+v"(ka[7]));
}

// Running softmax of NT blocks of 32 query columns over 128 channels.
template <int NT>
struct WideState {
    f32x16 acc[4][NT];  // channel blocks of 32
    float m[NT], l[NT]; // l is this lane's half of the keys only
};
template <int NT>
__device__ inline void raise_reference_wide(WideState<NT> &w, int nt, const f32x16 &s, float c) {
    float t0 = fmaxf(fmaxf(s[0], s[1]), s[2]);
    float t1 = fmaxf(fmaxf(s[3], s[4]), s[5]);
    float t2 = fmaxf(fmaxf(s[6], s[7]), s[8]);
    float t3 = fmaxf(fmaxf(s[9], s[10]), s[11]);
    float t4 = fmaxf(fmaxf(s[12], s[13]), s[14]);
    t0 = fmaxf(fmaxf(t0, t1), t2);
    t3 = fmaxf(fmaxf(t3, t4), s[15]);
    float a, b;
    pair_values(fmaxf(t0, t3) * c, &a, &b);  // this lane and lane^32 share the query column
    const float m_new = fmaxf(w.m[nt], fmaxf(a, b));
    const float alpha = __builtin_amdgcn_exp2f(w.m[nt] - m_new);
    w.m[nt] = m_new;
    w.l[nt] *= alpha;
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int v = 0; v < 16; ++v) w.acc[mi][nt][v] *= alpha;
}

// One tile of 32 keys: `ka` holds its K operands; V rows at vaddr + VOFF; KNEXT >= 0: the K
// operands at kaddr + KNEXT are read into `ka` under the exponentials; `mid` is the stage
// hand-over; MASKED: keys with index >= key_limit are padding.  Every operand read from LDS
// feeds NT matrix instructions.
template <int NT, int KNEXT, bool MASKED, int VOFF, class Mid>
__device__ __forceinline__ void wide_ring_tile(WideState<NT> &w, const u32x4 (&qreg)[NT][8], u32x4 (&ka)[8],
                                      const unsigned (&kaddr)[8], const unsigned (&vaddr)[4], int key_limit,
                                      float c, int lane, Mid &&mid) {
    const int g = lane >> 5;
    f32x16 s[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int v = 0; v < 16; ++v) s[nt][v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) s[nt] = mfma32(as_bf16x8(ka[ks]), as_bf16x8(qreg[nt][ks]), s[nt]);
    __builtin_amdgcn_sched_barrier(0);  // the score products are issued before the hand-over and the reads
    mid();
    u32x4 va[2][4];
    wide_load_v<VOFF>(va, vaddr);
    if (KNEXT >= 0) wide_load_k<KNEXT >= 0 ? KNEXT : 0>(ka, kaddr);
    __builtin_amdgcn_sched_barrier(0);  // ... and the reads before the softmax arithmetic
    unsigned pk[NT][8];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        if (MASKED) {
#pragma unroll
            for (int v = 0; v < 16; ++v) s[nt][v] = 8 * (v / 4) + 4 * g + (v % 4) >= key_limit ? -INFINITY : s[nt][v];
        }
        float tile_sum = exp_block(s[nt], pk[nt], c, -w.m[nt]);
        if (__builtin_amdgcn_ballot_w64(!(tile_sum <= kLazySum)) != 0) {  // also catches inf/NaN
            raise_reference_wide<NT>(w, nt, s[nt], c);
            tile_sum = exp_block(s[nt], pk[nt], c, -w.m[nt]);
        }
        w.l[nt] += tile_sum;
    }
    wide_reads_landed(va, ka);
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const u32x4 pb = {pk[nt][4 * kk], pk[nt][4 * kk + 1], pk[nt][4 * kk + 2], pk[nt][4 * kk + 3]};
                w.acc[mi][nt] = mfma32(as_bf16x8(va[kk][mi]), as_bf16x8(pb), w.acc[mi][nt]);
            }
}

// NT: blocks of 32 query columns per wavefront.  The kernel is built with NT = 1: 128 query slots
// per workgroup, two workgroups per compute unit.  (NT = 2 -- 256 query slots, one workgroup per
// compute unit with the whole register file, every operand read from LDS feeding two matrix
// instructions -- was measured 27 % slower: with one wavefront per SIMD nothing runs under its
// softmax arithmetic.)
template <bool O_BF16, int NT>
__global__ void __launch_bounds__(256, 2) attn_ring_wide_bf16(AttnArgs a) {
    static_assert(NT == 1, "two wavefronts per SIMD: the register budget holds one block of query columns");
    float c_log2 = a.c;
    asm volatile("" : "+s"(c_log2));  // fetched and waited for here, not inside the key loop
    __shared__ __align__(16) unsigned char smem[kWideRing * kStageWideBytes];
    static_assert(kWideRing * kStageWideBytes >= 4 * kTileWideBytes, "the ring doubles as output staging");
    const int tid = threadIdx.x, lane = tid & 63, g = lane >> 5, li = lane & 31;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    RingItem it;
    if (!ring_item(a, 128 * NT, it)) return;  // whole workgroup
    const int bh = it.bh, b = bh / a.heads, h = bh % a.heads;
    const int win = it.win, wy = win / a.g.wins_x, wx = win % a.g.wins_x;
    const int q0 = (it.qblock * 4 + wave) * (32 * NT);
    const long long qbase = b * a.q.sb + h * a.q.sh, obase = b * a.o.sb + h * a.o.sh;
    const bool wave_live = q0 < a.q_slots;

    // Query operands, in assembly (they are the wavefront's oldest loads; see load_queries).
    u32x4 qreg[NT][8];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int tok = max(slot_token(a, wy, wx, q0 + 32 * nt + li), 0);
        const __bf16 *row = (const __bf16 *)a.q.ptr + qbase + (long long)tok * a.q.sn + g * 8;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
            asm volatile("global_load_dwordx4 %0, %1, off offset:%2" : "=v"(qreg[nt][ks]) : "v"(row), "n"(32 * ks));
    }
    WideState<NT> w;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
#pragma unroll
            for (int v = 0; v < 16; ++v) w.acc[mi][nt][v] = 0.f;
        w.m[nt] = kMinusHuge;
        w.l[nt] = 0.f;
    }

    // Key slots that hold tokens.  Windows of whole grid rows: slot s is token tok_first + s.
    // Unpadded windows whose width divides the stage: a stage is 32 / ww whole window rows, so
    // slot s is token tok_first + (s / ww) W + s % ww and a stage is still a fixed step on.
    const int tok_first = wy * a.g.wh * a.g.W + (a.contig ? 0 : wx * a.g.ww);
    const int tok_limit = a.contig ? min(a.g.slots, a.g.H * a.g.W - tok_first) : a.g.slots;
    const int n_full = tok_limit / kStageWide, n_stage = (tok_limit + kStageWide - 1) / kStageWide;
    const int stage_tokens = a.contig ? kStageWide : (kStageWide / a.g.ww) * a.g.W;

    // Loads.  A wavefront moves rows 8 * wave .. + 7 of every stage's K and V, four rows (1 KB of
    // LDS) per instruction: lane = 16 * (row in the group of four) + 16-byte slot of the LDS row,
    // and it fetches the chunk of the token's row that belongs in that slot under the tile
    // layouts.  Rows past the last token fetch the window's first token instead.
    auto uniform = [](const char *ptr) {
        const unsigned long long u = (unsigned long long)ptr;
        const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)u);
        const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(u >> 32));
        return (const char *)(((unsigned long long)hi << 32) | lo);
    };
    const char *kbytes = uniform((const char *)((const __bf16 *)a.k.ptr + b * a.k.sb + h * a.k.sh + (long long)tok_first * a.k.sn));
    const char *vbytes = uniform((const char *)((const __bf16 *)a.v.ptr + b * a.v.sb + h * a.v.sh + (long long)tok_first * a.v.sn));
    const int lrow = lane >> 4, lslot = lane & 15;
    unsigned kcur[2], vcur[2], kpad[2], vpad[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int row = 8 * wave + 4 * i + lrow;
        const int row_tok = a.contig ? row : (row / a.g.ww) * a.g.W + row % a.g.ww;
        kpad[i] = 16u * (unsigned)(lslot ^ (row & 15));
        vpad[i] = 16u * (unsigned)((((lslot >> 2) ^ (row & 3)) << 2) | (lslot & 3));
        kcur[i] = 2u * (unsigned)row_tok * (unsigned)a.k.sn + kpad[i];
        vcur[i] = 2u * (unsigned)row_tok * (unsigned)a.v.sn + vpad[i];
    }
    const unsigned kstep = 2u * (unsigned)stage_tokens * (unsigned)a.k.sn, vstep = 2u * (unsigned)stage_tokens * (unsigned)a.v.sn;
    auto issue = [&](int stage) {
        unsigned char *kt = smem + (stage % kWideRing) * kStageWideBytes, *vt = kt + kTileWideBytes;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int row0 = 8 * wave + 4 * i;
            const bool past = stage * kStageWide + row0 + lrow >= tok_limit;  // only in the window's last stage
            __builtin_amdgcn_global_load_lds((attn_global_cvoid *)(kbytes + (past ? kpad[i] : kcur[i])),
                                             (attn_lds_void *)(kt + row0 * 256), 16, 0, 0);
            __builtin_amdgcn_global_load_lds((attn_global_cvoid *)(vbytes + (past ? vpad[i] : vcur[i])),
                                             (attn_lds_void *)(vt + row0 * 256), 16, 0, 0);
            kcur[i] += kstep;
            vcur[i] += vstep;
        }
    };
    // Inside the tile of stage st: stage st + 1 has landed for every wavefront, and every
    // wavefront has left stage st - 1, whose ring slot takes stage st + 2.
    auto hand_over = [&](int st) {
        if (st + 1 >= n_stage) return;  // uniform
        if (kWideRing == 4 && st + 2 < n_stage) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");  // (stage st + 2 stays in flight)
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        lds_barrier();
        if (st + kWideRing - 1 < n_stage) issue(st + kWideRing - 1);
    };
    unsigned kaddr[8], vaddr[4];
    wide_lane_addresses(kaddr, vaddr, smem, lane);
    u32x4 ka[8];
    auto full_stage = [&](int st, auto slot_tag) {
        constexpr int slot = decltype(slot_tag)::value, after = (slot + 1) % kWideRing;
        // (a wavefront whose query slots all lie past the limit computes like the others, on the
        // queries of token 0, and stores nothing: no branch around the tile, whose two sides the
        // compiler would reconcile by moving the accumulators between register files every tile)
        wide_ring_tile<NT, after * kStageWideBytes, false, slot * kStageWideBytes>(w, qreg, ka, kaddr, vaddr, 0, c_log2, lane, [&]() { hand_over(st); });
    };

    if (n_stage > 0) issue(0);
    if (n_stage > 1) issue(1);
    if (kWideRing == 4 && n_stage > 2) issue(2);
    if (kWideRing == 4 && n_stage > 2) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    else if (n_stage > 1) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    lds_barrier();  // stage 0 has landed
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) asm volatile("" : "+v"(qreg[nt][ks]));  // the queries, older than stage 0, have landed too
    wide_load_k<0>(ka, kaddr);
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(ka[0]), "+v"(ka[1]), "+v"(ka[2]), "+v"(ka[3]), "+v"(ka[4]), "+v"(ka[5]), "+v"(ka[6]), "+v"(ka[7]));
    int st = 0;
    while (st < n_full) {  // (one copy of each ring slot's tile: the loop is left from wherever the full stages end)
        full_stage(st, std::integral_constant<int, 0>());
        if (++st >= n_full) break;
        full_stage(st, std::integral_constant<int, 1>());
        if (++st >= n_full) break;
        full_stage(st, std::integral_constant<int, 2>());
        if (kWideRing == 4) {
            if (++st >= n_full) break;
            full_stage(st, std::integral_constant<int, 3 % kWideRing>());
        }
        ++st;
    }
    if (st < n_stage) {  // the partial stage that ends the window (its K operands are in ka)
        const unsigned at = (st % kWideRing) * kStageWideBytes;
        const unsigned vlast[4] = {vaddr[0] + at, vaddr[1] + at, vaddr[2] + at, vaddr[3] + at};
        wide_ring_tile<NT, -1, true, 0>(w, qreg, ka, kaddr, vlast, tok_limit - st * kStageWide, c_log2, lane, [] {});
    }
    __syncthreads();  // every wavefront is done with the ring: reuse it as staging
    if (!wave_live) return;

#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        float lo, hi;
        pair_values(w.l[nt], &lo, &hi);
        const float inv = __builtin_amdgcn_rcpf(lo + hi);
        const int qb = q0 + 32 * nt;
        if (O_BF16) {
            // channel-major accumulators -> token rows of 256 bytes through 8 KB of wave-private LDS
            unsigned char *stage = smem + wave * kTileWideBytes;
#pragma unroll
            for (int mi = 0; mi < 4; ++mi)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    const f32x16 &x = w.acc[mi][nt];
                    u32x2 pk = {pack_bf16x2(x[4 * q4] * inv, x[4 * q4 + 1] * inv),
                                pack_bf16x2(x[4 * q4 + 2] * inv, x[4 * q4 + 3] * inv)};
                    *(u32x2 *)(stage + wide_off_row(li, 4 * mi + q4) + 8 * g) = pk;
                }
            __bf16 *op = (__bf16 *)a.o.ptr + obase;
            const int orow = lane >> 4, ochunk = lane & 15;
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                const int row = 4 * r + orow, slot = qb + row;
                const int tok = slot < a.q_slots ? slot_token(a, wy, wx, slot) : -1;
                const u32x4 val = *(const u32x4 *)(stage + wide_off_row(row, ochunk));
                if (tok >= 0) *(u32x4 *)(op + (long long)tok * a.o.sn + ochunk * 8) = val;
            }
        } else {
            float *op = (float *)a.o.ptr + obase;
            const int slot = qb + li;
            const int tok = slot < a.q_slots ? slot_token(a, wy, wx, slot) : -1;
            if (tok >= 0) {
#pragma unroll
                for (int mi = 0; mi < 4; ++mi)
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4) {
                        const f32x16 &x = w.acc[mi][nt];
                        f32x4 val = {x[4 * q4] * inv, x[4 * q4 + 1] * inv, x[4 * q4 + 2] * inv, x[4 * q4 + 3] * inv};
                        *(f32x4 *)(op + (long long)tok * a.o.sn + 32 * mi + 8 * q4 + 4 * g) = val;
                    }
            }
        }
    }
}

jv_status attn_bf16(const Problem &pr, const WindowGeom &g, float scale, int q_slots, hipStream_t stream) {
    AttnArgs a;
    a.q = pr.q; a.k = pr.k; a.v = pr.v; a.o = pr.o;
    a.g = g;
    a.heads = pr.heads;
    a.contig = g.ww == g.W ? 1 : 0;
    a.q_slots = q_slots < g.slots ? q_slots : g.slots;
    a.c = scale * kLog2e;
    a.n_bh = pr.B * pr.heads;
    if (g.n_win > 65535) return fail(JV_ERR_UNSUPPORTED, "more than 65535 windows");
    // the streaming and ring kernels number their work items (query block, window, batch * head) in 32 bits
    if ((long long)((a.q_slots + 127) / 128) * g.n_win * a.n_bh >= (1ll << 28))
        return fail(JV_ERR_UNSUPPORTED, "more than 2^28 blocks of 128 queries");
    if (pr.D == kHeadDimWide) {
        // windows of whole grid rows, and unpadded windows whose width divides a key stage, with 32-bit
        // byte offsets inside a (batch, head) slice: the ring kernel
        const long long wide_sn = pr.k.sn > pr.v.sn ? pr.k.sn : pr.v.sn;
        const bool whole_windows = g.H % g.wh == 0 && g.W % g.ww == 0 && kStageWide % g.ww == 0;
        if ((a.contig || whole_windows) &&
            ((long long)pr.N + 2ll * kStageWide * g.W) * wide_sn * 2 + 512 < (1ll << 31)) {
            if (pr.o_bf16) hipLaunchKernelGGL((attn_ring_wide_bf16<true, 1>), ring_grid(a, 128), dim3(256), 0, stream, a);
            else hipLaunchKernelGGL((attn_ring_wide_bf16<false, 1>), ring_grid(a, 128), dim3(256), 0, stream, a);
            return launch_status("attn_ring_wide_bf16");
        }
        if (pr.o_bf16) hipLaunchKernelGGL((attn_wide_bf16<true>), ring_grid(a, 128), dim3(256), 0, stream, a);
        else hipLaunchKernelGGL((attn_wide_bf16<false>), ring_grid(a, 128), dim3(256), 0, stream, a);
        return launch_status("attn_wide_bf16");
    }
    const bool all_queries = a.q_slots == g.slots;  // the window-resident kernels compute every slot
    // Windows that fit in LDS whole take the window-resident kernel.
    if (all_queries && g.slots <= 64)
        return pr.o_bf16 ? launch_window<true, 1>(a, pr.B * pr.heads, stream)
                         : launch_window<false, 1>(a, pr.B * pr.heads, stream);
    if (all_queries && g.slots == 256 && g.n_win > 1 && g.H % g.wh == 0 && g.W % g.ww == 0) {
        // byte offsets of a window's tokens from its first one in 32 bits?
        long long max_sn = pr.q.sn;
        for (long long sn : {pr.k.sn, pr.v.sn, pr.o.sn}) max_sn = sn > max_sn ? sn : max_sn;
        if (((long long)(g.wh - 1) * g.W + g.ww) * max_sn * 4 + 256 < (1ll << 31))
            return pr.o_bf16 ? launch_window8<true>(a, pr.B * pr.heads, stream)
                             : launch_window8<false>(a, pr.B * pr.heads, stream);
    }
    if (all_queries && g.slots <= 256 && g.n_win > 1)
        return pr.o_bf16 ? launch_window<true, 4>(a, pr.B * pr.heads, stream)
                         : launch_window<false, 4>(a, pr.B * pr.heads, stream);
    constexpr int NT = JV_ATTN_NT;
    // 32-bit byte offsets inside one (batch, head) slice?
    const long long max_sn = pr.k.sn > pr.v.sn ? pr.k.sn : pr.v.sn;
    const bool fast = a.contig && ((long long)pr.N + 2 * kStage) * max_sn * 2 + 256 < (1ll << 31);
    // a handful of queries against the whole sequence (prefix tokens): split the keys instead
    if (fast && !all_queries && a.q_slots <= 64 && g.n_win == 1)
        return pr.o_bf16 ? launch_prefix<true>(a, pr.B * pr.heads, stream)
                         : launch_prefix<false>(a, pr.B * pr.heads, stream);
    if (fast && NT == 2) {
        if (pr.o_bf16) hipLaunchKernelGGL((attn_ring_bf16<true>), ring_grid(a, 256), dim3(256), 0, stream, a);
        else hipLaunchKernelGGL((attn_ring_bf16<false>), ring_grid(a, 256), dim3(256), 0, stream, a);
        return launch_status("attn_ring_bf16");
    }
    if (pr.o_bf16)
        hipLaunchKernelGGL((attn_stream_bf16<true, NT>), ring_grid(a, 128 * NT), dim3(256), 0, stream, a);
    else
        hipLaunchKernelGGL((attn_stream_bf16<false, NT>), ring_grid(a, 128 * NT), dim3(256), 0, stream, a);
    return launch_status("attn_stream_bf16");
}

}  // namespace jv
