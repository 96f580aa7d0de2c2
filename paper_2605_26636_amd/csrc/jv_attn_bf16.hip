// Softmax attention for bf16 tensors on the matrix cores (Eq. 1 of the paper; restricted to a
// window of the token grid for window attention, Sec. 3.2.2), fp32 softmax and accumulation.
//
// A wavefront owns 64 query slots of one window (two 32-column blocks) and walks the window's
// key slots in tiles of 32.  Per tile it forms the transposed scores S^T = K_tile Q^T, so that
// a lane holds one query column: row maxima and sums stay inside a lane (plus one exchange
// with lane^32), and the exponentiated tile, rounded to bf16, is already laid out as the B
// operand of O^T += V_tile^T P^T.  K tiles are read from LDS row by row (A operand of the
// first product); V tiles are read with transposing LDS reads (A operand of the second).
// The running maximum is only raised when a tile exceeds it by more than 2^8, which keeps the
// rescaling of the accumulators off the common path; the result is unchanged because the
// same reference is used for numerator and denominator.
#include <math.h>

#include <type_traits>

#include "jv_common.h"
#include "jv_mfma.h"

#ifndef JV_ATTN_NT
#define JV_ATTN_NT 2   // blocks of 32 query columns per wavefront
#endif
#ifndef JV_ATTN_SKEW
#define JV_ATTN_SKEW 0  // 1: half-step skew of the two query blocks inside a tile
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
    float c;     // logit scale times log2(e)
};

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLazyRescale = 8.0f;   // log2 units
constexpr float kMinusHuge = -1.0e30f; // finite stand-in for "no maximum yet"

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

// A operand of O^T += V^T P^T: channels 32*blk32 .. +31 (one per lane), k-slot (g, 4r + e)
// stands for key key0 + 8r + 4g + e, the order in which a lane holds its scores.
__device__ inline bf16x8 load_vt_operand(const unsigned char *tile, int key0, int blk32,
                                         int lane) {
    const int b = lane >> 4, j = lane & 15, g = b >> 1;
    const int chunk16 = blk32 * 4 + (b & 1) * 2 + ((j & 3) >> 1);
    const int half = (j & 1) * 8;
    const int row0 = key0 + 4 * g + (j >> 2);
    u32x2 r0 = lds_read_tr16(tile + tile_off_tr(row0, chunk16) + half);
    u32x2 r1 = lds_read_tr16(tile + tile_off_tr(row0 + 8, chunk16) + half);
    u32x4 r = {r0[0], r0[1], r1[0], r1[1]};
    return as_bf16x8(r);
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

// Raise the softmax reference of query block nt if the (already masked) scores s exceed it
// by more than the lazy threshold, rescaling that block's accumulators and row sum.
template <int NT>
__device__ inline void update_reference(WaveState<NT> &w, int nt, const f32x16 &s, float c) {
    float t0 = fmaxf(fmaxf(s[0], s[1]), s[2]);
    float t1 = fmaxf(fmaxf(s[3], s[4]), s[5]);
    float t2 = fmaxf(fmaxf(s[6], s[7]), s[8]);
    float t3 = fmaxf(fmaxf(s[9], s[10]), s[11]);
    float t4 = fmaxf(fmaxf(s[12], s[13]), s[14]);
    t0 = fmaxf(fmaxf(t0, t1), t2);
    t3 = fmaxf(fmaxf(t3, t4), s[15]);
    // This lane sees half of the tile's keys; if no lane of the wave exceeds the threshold,
    // no query column does, and the exchange with the partner lane can be skipped.
    const float own = fmaxf(t0, t3) * c;
    if (__builtin_amdgcn_ballot_w64(own > w.m[nt] + kLazyRescale) != 0) {
        float a, b;
        pair_values(own, &a, &b);
        const float m_new = fmaxf(w.m[nt], fmaxf(a, b));
        const float alpha = __builtin_amdgcn_exp2f(w.m[nt] - m_new);
        w.m[nt] = m_new;
        w.l[nt] *= alpha;
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int v = 0; v < 16; ++v) w.acc[mi][nt][v] *= alpha;
    }
}

__device__ inline void add_key_bias(f32x16 &s, const float *bias, int g) {
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
        const f32x4 bv = *(const f32x4 *)(bias + 8 * q4 + 4 * g);
#pragma unroll
        for (int e = 0; e < 4; ++e) s[4 * q4 + e] += bv[e];
    }
}

// One tile of 32 keys.  ktile/vtile point at row 0 of the tile (K rows laid out with
// tile_off_row, V rows with tile_off_tr; both offsets take tile-relative rows, so tiles must
// start at a multiple of 8 rows).  bias, if non-null, holds 0 / -inf per key of the tile.
template <int NT>
__device__ inline void attn_tile32(WaveState<NT> &w, const bf16x8 (&qreg)[NT][4],
                                   const unsigned char *ktile, const unsigned char *vtile,
                                   int krow0, const float *bias, float c, int lane) {
    const int g = lane >> 5, li = lane & 31;
    f32x16 s[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int v = 0; v < 16; ++v) s[nt][v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        const bf16x8 ka = as_bf16x8(*(const u32x4 *)(ktile + tile_off_row(krow0 + li, 2 * ks + g)));
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) s[nt] = mfma32(ka, qreg[nt][ks], s[nt]);
    }
    if (bias) {  // wave-uniform
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            const f32x4 bv = *(const f32x4 *)(bias + 8 * q4 + 4 * g);
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) s[nt][4 * q4 + e] += bv[e];
        }
    }
    unsigned pk[NT][8];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        update_reference<NT>(w, nt, s[nt], c);
        const float neg_m = -w.m[nt];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float p0 = __builtin_amdgcn_exp2f(fmaf(s[nt][2 * j], c, neg_m));
            const float p1 = __builtin_amdgcn_exp2f(fmaf(s[nt][2 * j + 1], c, neg_m));
            pk[nt][j] = pack_bf16x2(p0, p1);
            w.l[nt] = add_bf16x2(pk[nt][j], w.l[nt]);
        }
    }
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
#pragma unroll
        for (int mi = 0; mi < 2; ++mi) {
            const bf16x8 va = load_vt_operand(vtile, krow0 + 16 * kk, mi, lane);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                u32x4 pb = {pk[nt][4 * kk], pk[nt][4 * kk + 1], pk[nt][4 * kk + 2], pk[nt][4 * kk + 3]};
                w.acc[mi][nt] = mfma32(va, as_bf16x8(pb), w.acc[mi][nt]);
            }
        }
    }
}

// One tile of 32 keys for two query blocks, with the two blocks half a step apart so that each
// wavefront overlaps its own matrix and vector work: the scores of block 1 are formed while
// block 0 is exponentiated, and the products of block 0 are added while block 1 is
// exponentiated.  Scheduling fences pin that order.
__device__ inline void attn_tile32_skewed(WaveState<2> &w, const bf16x8 (&qreg)[2][4],
                                          const unsigned char *ktile, const unsigned char *vtile,
                                          int krow0, const float *bias, float c, int lane) {
    const int g = lane >> 5, li = lane & 31;
    bf16x8 ka[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
        ka[ks] = as_bf16x8(*(const u32x4 *)(ktile + tile_off_row(krow0 + li, 2 * ks + g)));
    f32x16 s0, s1;
#pragma unroll
    for (int v = 0; v < 16; ++v) { s0[v] = 0.f; s1[v] = 0.f; }
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) s0 = mfma32(ka[ks], qreg[0][ks], s0);
    if (bias) add_key_bias(s0, bias, g);  // wave-uniform
    update_reference<2>(w, 0, s0, c);

    unsigned pk0[8], pk1[8];
    {
        const float neg_m = -w.m[0];
        float l = w.l[0];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            s1 = mfma32(ka[ks], qreg[1][ks], s1);
#pragma unroll
            for (int j = 2 * ks; j < 2 * ks + 2; ++j) {
                const float p0 = __builtin_amdgcn_exp2f(fmaf(s0[2 * j], c, neg_m));
                const float p1 = __builtin_amdgcn_exp2f(fmaf(s0[2 * j + 1], c, neg_m));
                pk0[j] = pack_bf16x2(p0, p1);
                l = add_bf16x2(pk0[j], l);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        w.l[0] = l;
    }
    bf16x8 va[2][2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
        for (int mi = 0; mi < 2; ++mi) va[kk][mi] = load_vt_operand(vtile, krow0 + 16 * kk, mi, lane);
    if (bias) add_key_bias(s1, bias, g);
    update_reference<2>(w, 1, s1, c);
    {
        const float neg_m = -w.m[1];
        float l = w.l[1];
#pragma unroll
        for (int idx = 0; idx < 4; ++idx) {
            const int kk = idx >> 1, mi = idx & 1;
            u32x4 pb = {pk0[4 * kk], pk0[4 * kk + 1], pk0[4 * kk + 2], pk0[4 * kk + 3]};
            w.acc[mi][0] = mfma32(va[kk][mi], as_bf16x8(pb), w.acc[mi][0]);
#pragma unroll
            for (int j = 2 * idx; j < 2 * idx + 2; ++j) {
                const float p0 = __builtin_amdgcn_exp2f(fmaf(s1[2 * j], c, neg_m));
                const float p1 = __builtin_amdgcn_exp2f(fmaf(s1[2 * j + 1], c, neg_m));
                pk1[j] = pack_bf16x2(p0, p1);
                l = add_bf16x2(pk1[j], l);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        w.l[1] = l;
    }
#pragma unroll
    for (int idx = 0; idx < 4; ++idx) {
        const int kk = idx >> 1, mi = idx & 1;
        u32x4 pb = {pk1[4 * kk], pk1[4 * kk + 1], pk1[4 * kk + 2], pk1[4 * kk + 3]};
        w.acc[mi][1] = mfma32(va[kk][mi], as_bf16x8(pb), w.acc[mi][1]);
    }
}

template <int NT>
__device__ inline void attn_tile(WaveState<NT> &w, const bf16x8 (&qreg)[NT][4],
                                 const unsigned char *ktile, const unsigned char *vtile,
                                 int krow0, const float *bias, float c, int lane) {
#if JV_ATTN_SKEW
    if constexpr (NT == 2) {
        attn_tile32_skewed(w, qreg, ktile, vtile, krow0, bias, c, lane);
        return;
    }
#endif
    attn_tile32<NT>(w, qreg, ktile, vtile, krow0, bias, c, lane);
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
                if (tok >= 0) *(u32x4 *)(op + (long long)tok * a.o.sn + lchunk * 8) = val;
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

// Query operands (B of S^T = K Q^T): lane holds channels 16*ks + 8g .. +7 of query li.
template <int NT>
__device__ inline void load_queries(bf16x8 (&qreg)[NT][4], const AttnArgs &a, int wy, int wx,
                                    int q0, long long qbase, int lane) {
    const int g = lane >> 5, li = lane & 31;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int tok = slot_token(a, wy, wx, q0 + 32 * nt + li);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            u32x4 x = {0u, 0u, 0u, 0u};
            if (tok >= 0)
                x = *(const u32x4 *)((const __bf16 *)a.q.ptr + qbase + (long long)tok * a.q.sn +
                                     (2 * ks + g) * 8);
            qreg[nt][ks] = as_bf16x8(x);
        }
    }
}

// ---------------------------------------------------------------------------------------
// Streaming kernel: any window size, including the whole grid (full attention).
// A workgroup holds 128*NT consecutive query slots of one window (4 waves x 32*NT) and streams
// the window's keys through LDS in double-buffered stages of 64.
// grid (ceil(slots/(128*NT)), n_win, B*heads), 256 threads.
// ---------------------------------------------------------------------------------------
constexpr int kStage = 64;
constexpr int kStageBytes = 2 * kStage * 128;  // K rows then V rows

template <bool O_BF16, int NT>
__global__ void __launch_bounds__(256, JV_ATTN_MINW) attn_stream_bf16(AttnArgs a) {
    __shared__ __align__(16) unsigned char smem[2 * kStageBytes];
    __shared__ __align__(16) float bias[2][kStage];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int bh = blockIdx.z, b = bh / a.heads, h = bh % a.heads;
    const int win = blockIdx.y, wy = win / a.g.wins_x, wx = win % a.g.wins_x;
    const int q0 = blockIdx.x * (128 * NT) + wave * (32 * NT);
    const long long qbase = b * a.q.sb + h * a.q.sh, kbase = b * a.k.sb + h * a.k.sh;
    const long long vbase = b * a.v.sb + h * a.v.sh, obase = b * a.o.sb + h * a.o.sh;
    const bool wave_live = q0 < a.g.slots;

    bf16x8 qreg[NT][4];
    load_queries<NT>(qreg, a, wy, wx, q0, qbase, lane);
    WaveState<NT> w;
    wave_state_init<NT>(w);

    // Is any key slot of this window padding?  (Stages past the last slot are handled below.)
    const bool ragged = (wy + 1) * a.g.wh > a.g.H || (wx + 1) * a.g.ww > a.g.W;
    const int n_stage = (a.g.slots + kStage - 1) / kStage;
    const int lrow = tid >> 3, lchunk = tid & 7;
    // This thread moves rows lrow and lrow + 32 of every stage.  For windows that span whole
    // grid rows the token is "first token + slot", so the global pointers just advance by one
    // stage per step; otherwise the slot is mapped through the window geometry each time.
    const __bf16 *kptr = (const __bf16 *)a.k.ptr + kbase + lchunk * 8;
    const __bf16 *vptr = (const __bf16 *)a.v.ptr + vbase + lchunk * 8;
    const int tok_first = wy * a.g.wh * a.g.W, n_tok = a.g.H * a.g.W;
    const int tok_limit = min(a.g.slots, n_tok - tok_first);  // contiguous case: live slots
    u32x4 kreg[2], vreg[2];
    bool live[2];
    auto fetch = [&](int stage) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int slot = stage * kStage + lrow + 32 * i;
            int tok;
            if (a.contig) tok = slot < tok_limit ? tok_first + slot : -1;
            else tok = slot_token(a, wy, wx, slot);
            u32x4 zero = {0u, 0u, 0u, 0u};
            kreg[i] = zero;
            vreg[i] = zero;
            live[i] = tok >= 0;
            if (tok >= 0) {
                kreg[i] = *(const u32x4 *)(kptr + (long long)tok * a.k.sn);
                vreg[i] = *(const u32x4 *)(vptr + (long long)tok * a.v.sn);
            }
        }
    };
    auto stash = [&](int buf) {
        unsigned char *kt = smem + buf * kStageBytes, *vt = kt + kStage * 128;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int row = lrow + 32 * i;
            *(u32x4 *)(kt + tile_off_row(row, lchunk)) = kreg[i];
            *(u32x4 *)(vt + tile_off_tr(row, lchunk)) = vreg[i];
            if (lchunk == 0) bias[buf][row] = live[i] ? 0.f : -INFINITY;
        }
    };
    // One stage: prefetch the next one, run the two tiles of this one, publish the next one.
    // `buf` is a compile-time constant so that every LDS offset folds into the instruction.
    auto run_stage = [&](int st, auto buf_tag) {
        constexpr int buf = decltype(buf_tag)::value;
        const bool more = st + 1 < n_stage;
        if (more) fetch(st + 1);
        if (wave_live) {
            const unsigned char *kt = smem + buf * kStageBytes, *vt = kt + kStage * 128;
            const bool masked = ragged || (st + 1) * kStage > a.g.slots;
#pragma unroll
            for (int sub = 0; sub < 2; ++sub)
                attn_tile<NT>(w, qreg, kt, vt, 32 * sub, masked ? &bias[buf][32 * sub] : nullptr,
                              a.c, lane);
        }
        if (more) stash(buf ^ 1);
        __syncthreads();
    };

    fetch(0);
    stash(0);
    __syncthreads();
    for (int st = 0; st < n_stage; st += 2) {
        run_stage(st, std::integral_constant<int, 0>());
        if (st + 1 < n_stage) run_stage(st + 1, std::integral_constant<int, 1>());
    }
    if (wave_live) wave_store<O_BF16, NT>(w, a, wy, wx, q0, obase, smem + wave * 4096, lane);
}

// ---------------------------------------------------------------------------------------
// Window-resident kernel: windows of at most 64*WPW slots (WPW = wavefronts per window).
// All keys and values of a window are brought into LDS once, then every wavefront runs its 64
// query slots over the resident tiles with no further synchronisation.  WPW = 4: one
// workgroup per window (e.g. 16x16 windows); WPW = 1: one wavefront per window, four windows
// per workgroup (e.g. 8x8 windows).  Window attention moves 4 rows of 128 bytes per token and
// does little arithmetic on them, so the point of this kernel is to have many bytes in flight:
// 96 KB of loads per 256 query slots are issued up front.
// grid (ceil(n_win * WPW / 4), B*heads), 256 threads, kWindowLds bytes of dynamic LDS.
// ---------------------------------------------------------------------------------------
constexpr int kWindowLds = 4 * (2 * 64 * 128 + 64 * 4);

template <bool O_BF16, int WPW>
__global__ void __launch_bounds__(256, 2) attn_window_bf16(AttnArgs a) {
    extern __shared__ __align__(16) unsigned char wsm[];
    constexpr int R = 64 * WPW;  // LDS rows per window
    constexpr int T = 64 * WPW;  // threads that load one window
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int bh = blockIdx.y, b = bh / a.heads, h = bh % a.heads;
    const int win = WPW == 4 ? blockIdx.x : blockIdx.x * 4 + wave;
    const bool win_live = win < a.g.n_win;  // WPW == 1: the last workgroup may have idle waves
    const int wy = win_live ? win / a.g.wins_x : 0, wx = win_live ? win % a.g.wins_x : 0;
    unsigned char *ktile = wsm + (WPW == 4 ? 0 : wave * (2 * 64 * 128));
    unsigned char *vtile = ktile + R * 128;
    float *bias = (float *)(wsm + 4 * 2 * 64 * 128) + (WPW == 4 ? 0 : wave * 64);
    const int t = WPW == 4 ? tid : lane;
    const int q0 = WPW == 4 ? wave * 64 : 0;
    const long long qbase = b * a.q.sb + h * a.q.sh, kbase = b * a.k.sb + h * a.k.sh;
    const long long vbase = b * a.v.sb + h * a.v.sh, obase = b * a.o.sb + h * a.o.sh;
    const int n_tile = (a.g.slots + 31) >> 5;
    const bool wave_live = win_live && q0 < a.g.slots;

    bf16x8 qreg[2][4];
    if (wave_live) load_queries<2>(qreg, a, wy, wx, q0, qbase, lane);

    if (win_live) {
        const int lchunk = t & 7;
        const __bf16 *kptr = (const __bf16 *)a.k.ptr + kbase + lchunk * 8;
        const __bf16 *vptr = (const __bf16 *)a.v.ptr + vbase + lchunk * 8;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            u32x4 kreg[4], vreg[4];
            bool live[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = (4 * half + i) * (T / 8) + (t >> 3);
                const int tok = row < 32 * n_tile ? slot_token(a, wy, wx, row) : -1;
                u32x4 zero = {0u, 0u, 0u, 0u};
                kreg[i] = zero;
                vreg[i] = zero;
                live[i] = tok >= 0;
                if (tok >= 0) {
                    kreg[i] = *(const u32x4 *)(kptr + (long long)tok * a.k.sn);
                    vreg[i] = *(const u32x4 *)(vptr + (long long)tok * a.v.sn);
                }
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = (4 * half + i) * (T / 8) + (t >> 3);
                if (row < 32 * n_tile) {
                    *(u32x4 *)(ktile + tile_off_row(row, lchunk)) = kreg[i];
                    *(u32x4 *)(vtile + tile_off_tr(row, lchunk)) = vreg[i];
                    if (lchunk == 0) bias[row] = live[i] ? 0.f : -INFINITY;
                }
            }
        }
    }
    if (WPW == 4) __syncthreads();
    else __builtin_amdgcn_wave_barrier();

    WaveState<2> w;
    wave_state_init<2>(w);
    if (wave_live) {
        const bool ragged = (wy + 1) * a.g.wh > a.g.H || (wx + 1) * a.g.ww > a.g.W;
        for (int tile = 0; tile < n_tile; ++tile) {
            const bool masked = ragged || 32 * (tile + 1) > a.g.slots;
            attn_tile<2>(w, qreg, ktile, vtile, 32 * tile, masked ? bias + 32 * tile : nullptr, a.c,
                         lane);
        }
    }
    if (WPW == 4) __syncthreads();  // all waves are done with the tiles: reuse them as staging
    else __builtin_amdgcn_wave_barrier();
    if (wave_live)
        wave_store<O_BF16, 2>(w, a, wy, wx, q0, obase, ktile + (WPW == 4 ? wave * 4096 : 0), lane);
}

static jv_status set_lds_limit(const void *fn, int bytes) {
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e != hipSuccess) return fail(JV_ERR_HIP, "hipFuncSetAttribute: %s", hipGetErrorString(e));
    return JV_OK;
}

template <bool O_BF16, int WPW>
static jv_status launch_window(const AttnArgs &a, int BH, hipStream_t stream) {
    static bool attr_set = false;
    if (!attr_set) {
        jv_status st = set_lds_limit((const void *)attn_window_bf16<O_BF16, WPW>, kWindowLds);
        if (st != JV_OK) return st;
        attr_set = true;
    }
    dim3 grid((a.g.n_win * WPW + 3) / 4, BH);
    hipLaunchKernelGGL((attn_window_bf16<O_BF16, WPW>), grid, dim3(256), kWindowLds, stream, a);
    return launch_status("attn_window_bf16");
}

jv_status attn_bf16(const Problem &pr, const WindowGeom &g, float scale, hipStream_t stream) {
    AttnArgs a;
    a.q = pr.q; a.k = pr.k; a.v = pr.v; a.o = pr.o;
    a.g = g;
    a.heads = pr.heads;
    a.contig = g.ww == g.W ? 1 : 0;
    a.c = scale * kLog2e;
    if (g.n_win > 65535) return fail(JV_ERR_UNSUPPORTED, "more than 65535 windows");
    // Windows that fit in LDS whole take the window-resident kernel.
    if (g.slots <= 64)
        return pr.o_bf16 ? launch_window<true, 1>(a, pr.B * pr.heads, stream)
                         : launch_window<false, 1>(a, pr.B * pr.heads, stream);
    if (g.slots <= 256 && g.n_win > 1)
        return pr.o_bf16 ? launch_window<true, 4>(a, pr.B * pr.heads, stream)
                         : launch_window<false, 4>(a, pr.B * pr.heads, stream);
    constexpr int NT = JV_ATTN_NT;
    dim3 grid((g.slots + 128 * NT - 1) / (128 * NT), g.n_win, pr.B * pr.heads);
    if (pr.o_bf16)
        hipLaunchKernelGGL((attn_stream_bf16<true, NT>), grid, dim3(256), 0, stream, a);
    else
        hipLaunchKernelGGL((attn_stream_bf16<false, NT>), grid, dim3(256), 0, stream, a);
    return launch_status("attn_stream_bf16");
}

}  // namespace jv
