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

#include "jv_common.h"
#include "jv_mfma.h"

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

// Running softmax state of one wavefront: 64 query columns (2 blocks of 32), 64 channels.
struct WaveState {
    f32x16 acc[2][2];  // [channel block][query block]
    float m[2], l[2];  // per query block; l is this lane's half of the keys only
};

__device__ inline void wave_state_init(WaveState &w) {
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int v = 0; v < 16; ++v) w.acc[mi][nt][v] = 0.f;
    w.m[0] = w.m[1] = kMinusHuge;
    w.l[0] = w.l[1] = 0.f;
}

// One tile of 32 keys.  ktile/vtile point at row 0 of the tile (K rows laid out with
// tile_off_row, V rows with tile_off_tr; both offsets take tile-relative rows, so tiles must
// start at a multiple of 8 rows).  bias, if non-null, holds 0 / -inf per key of the tile.
__device__ inline void attn_tile32(WaveState &w, const bf16x8 (&qreg)[2][4],
                                   const unsigned char *ktile, const unsigned char *vtile,
                                   int krow0, const float *bias, float c, int lane) {
    const int g = lane >> 5, li = lane & 31;
    f32x16 s[2];
#pragma unroll
    for (int v = 0; v < 16; ++v) { s[0][v] = 0.f; s[1][v] = 0.f; }
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        const bf16x8 ka = as_bf16x8(*(const u32x4 *)(ktile + tile_off_row(krow0 + li, 2 * ks + g)));
        s[0] = mfma32(ka, qreg[0][ks], s[0]);
        s[1] = mfma32(ka, qreg[1][ks], s[1]);
    }
    if (bias) {  // wave-uniform
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            const f32x4 bv = *(const f32x4 *)(bias + 8 * q4 + 4 * g);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                s[0][4 * q4 + e] += bv[e];
                s[1][4 * q4 + e] += bv[e];
            }
        }
    }
    unsigned pk[2][8];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
        float tm = s[nt][0];
#pragma unroll
        for (int v = 1; v < 16; ++v) tm = fmaxf(tm, s[nt][v]);
        float a, b;
        pair_values(tm, &a, &b);
        const float tmy = fmaxf(a, b) * c;
        if (__builtin_amdgcn_ballot_w64(tmy > w.m[nt] + kLazyRescale) != 0) {
            const float m_new = fmaxf(w.m[nt], tmy);
            const float alpha = __builtin_amdgcn_exp2f(w.m[nt] - m_new);
            w.m[nt] = m_new;
            w.l[nt] *= alpha;
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                for (int v = 0; v < 16; ++v) w.acc[mi][nt][v] *= alpha;
        }
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
        u32x4 p0 = {pk[0][4 * kk], pk[0][4 * kk + 1], pk[0][4 * kk + 2], pk[0][4 * kk + 3]};
        u32x4 p1 = {pk[1][4 * kk], pk[1][4 * kk + 1], pk[1][4 * kk + 2], pk[1][4 * kk + 3]};
#pragma unroll
        for (int mi = 0; mi < 2; ++mi) {
            const bf16x8 va = load_vt_operand(vtile, krow0 + 16 * kk, mi, lane);
            w.acc[mi][0] = mfma32(va, as_bf16x8(p0), w.acc[mi][0]);
            w.acc[mi][1] = mfma32(va, as_bf16x8(p1), w.acc[mi][1]);
        }
    }
}

// Normalise and store the 64 query columns of a wavefront.  `stage` is 4 KB of wave-private
// LDS used to turn the channel-major accumulators into token rows for 16-byte stores.
template <bool O_BF16>
__device__ inline void wave_store(const WaveState &w, const AttnArgs &a, int wy, int wx,
                                  int q0, long long obase, unsigned char *stage, int lane) {
    const int g = lane >> 5, li = lane & 31, lrow = lane >> 3, lchunk = lane & 7;
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
__device__ inline void load_queries(bf16x8 (&qreg)[2][4], const AttnArgs &a, int wy, int wx,
                                    int q0, long long qbase, int lane) {
    const int g = lane >> 5, li = lane & 31;
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
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
// A workgroup holds 256 consecutive query slots of one window (4 waves x 64) and streams the
// window's keys through LDS in double-buffered stages of 64.
// grid (ceil(slots/256), n_win, B*heads), 256 threads.
// ---------------------------------------------------------------------------------------
constexpr int kStage = 64;
constexpr int kStageBytes = 2 * kStage * 128;  // K rows then V rows

template <bool O_BF16>
__global__ void __launch_bounds__(256, 2) attn_stream_bf16(AttnArgs a) {
    __shared__ __align__(16) unsigned char smem[2 * kStageBytes];
    __shared__ __align__(16) float bias[2][kStage];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int bh = blockIdx.z, b = bh / a.heads, h = bh % a.heads;
    const int win = blockIdx.y, wy = win / a.g.wins_x, wx = win % a.g.wins_x;
    const int q0 = blockIdx.x * 256 + wave * 64;
    const long long qbase = b * a.q.sb + h * a.q.sh, kbase = b * a.k.sb + h * a.k.sh;
    const long long vbase = b * a.v.sb + h * a.v.sh, obase = b * a.o.sb + h * a.o.sh;
    const bool wave_live = q0 < a.g.slots;

    bf16x8 qreg[2][4];
    load_queries(qreg, a, wy, wx, q0, qbase, lane);
    WaveState w;
    wave_state_init(w);

    // Is any key slot of this window padding?  (Stages past the last slot are handled below.)
    const bool ragged = (wy + 1) * a.g.wh > a.g.H || (wx + 1) * a.g.ww > a.g.W;
    const int n_stage = (a.g.slots + kStage - 1) / kStage;
    const int lrow = tid >> 3, lchunk = tid & 7;
    u32x4 kreg[2], vreg[2];
    bool live[2];
    auto fetch = [&](int stage) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int tok = slot_token(a, wy, wx, stage * kStage + lrow + 32 * i);
            u32x4 zero = {0u, 0u, 0u, 0u};
            kreg[i] = zero;
            vreg[i] = zero;
            live[i] = tok >= 0;
            if (tok >= 0) {
                kreg[i] = *(const u32x4 *)((const __bf16 *)a.k.ptr + kbase + (long long)tok * a.k.sn + lchunk * 8);
                vreg[i] = *(const u32x4 *)((const __bf16 *)a.v.ptr + vbase + (long long)tok * a.v.sn + lchunk * 8);
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

    fetch(0);
    stash(0);
    __syncthreads();
    for (int st = 0; st < n_stage; ++st) {
        const int buf = st & 1;
        const bool more = st + 1 < n_stage;
        if (more) fetch(st + 1);
        if (wave_live) {
            const unsigned char *kt = smem + buf * kStageBytes, *vt = kt + kStage * 128;
            const bool masked = ragged || (st + 1) * kStage > a.g.slots;
#pragma unroll
            for (int sub = 0; sub < 2; ++sub)
                attn_tile32(w, qreg, kt, vt, 32 * sub, masked ? &bias[buf][32 * sub] : nullptr,
                            a.c, lane);
        }
        if (more) stash(buf ^ 1);
        __syncthreads();
    }
    if (wave_live) wave_store<O_BF16>(w, a, wy, wx, q0, obase, smem + wave * 4096, lane);
}

jv_status attn_bf16(const Problem &pr, const WindowGeom &g, float scale, hipStream_t stream) {
    AttnArgs a;
    a.q = pr.q; a.k = pr.k; a.v = pr.v; a.o = pr.o;
    a.g = g;
    a.heads = pr.heads;
    a.contig = g.ww == g.W ? 1 : 0;
    a.c = scale * kLog2e;
    if (g.n_win > 65535) return fail(JV_ERR_UNSUPPORTED, "more than 65535 windows");
    dim3 grid((g.slots + 255) / 256, g.n_win, pr.B * pr.heads);
    if (pr.o_bf16)
        hipLaunchKernelGGL(attn_stream_bf16<true>, grid, dim3(256), 0, stream, a);
    else
        hipLaunchKernelGGL(attn_stream_bf16<false>, grid, dim3(256), 0, stream, a);
    return launch_status("attn_stream_bf16");
}

}  // namespace jv
