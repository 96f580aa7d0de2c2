// Linear attention (Eq. 2 of the paper, key-sum normaliser; phi = ReLU, or the focused map of
// Eq. 3 for the ablation variant) for bf16 tensors on the matrix cores, fp32 accumulation.
//
//   la_state_bf16   streams K and V once: every wavefront owns a 64 x 64 fp32 state in
//                   accumulators and adds relu(K_tile)^T V_tile per 64-token tile; the token
//                   axis is the contraction axis of both operands, so tiles go through LDS
//                   and come back with transposing reads.  z falls out of the same operands.
//   la_combine      sums the partial states when there are many chunks.
//   la_apply_bf16   sums the (few) partials, splits S and z into bf16 high and low parts held
//                   in registers, and streams Q -> O:  O^T = S^T relu(Q)^T on the matrix
//                   cores, the denominator relu(q).z as one more row block, fp32 divide.
//   la_state_wide_bf16, la_apply_wide_bf16   the same two passes for heads of 128 channels: the
//                   128 x 128 state as four 64 x 64 quadrants, one per wavefront of a workgroup.
#include <type_traits>

#include "jv_linear.h"
#include "jv_mfma.h"

namespace jv {

// Focused feature map (Eq. 3 of the paper, one of the block variants its Table 1 measures):
//   phi_p(x) = |r| / |r^p| * r^p,   r = relu(x), powers element-wise, norms over the 64 channels
// of the token's head; p is an integer >= 2 here (p = 1 is ReLU itself).  A token row is spread
// over the 8 consecutive lanes lane/8*8 .. +7, 8 channels each.  The row is divided by its
// largest entry before the power so that nothing overflows; fp32 arithmetic, result rounded to
// bf16 (the operand type of the matrix instructions).
__device__ inline float row8_combine(float x, bool take_max) {
    // lanes ^1 and ^2 through quad permutes, then the other quad of the 8-lane group through
    // the half-row mirror
    auto with = [&](float a, float b) { return take_max ? fmaxf(a, b) : a + b; };
    auto dpp = [](float v, auto ctrl_tag) {
        constexpr int ctrl = decltype(ctrl_tag)::value;
        return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), ctrl, 0xf, 0xf, true));
    };
    x = with(x, dpp(x, std::integral_constant<int, 0xB1>()));   // quad_perm [1, 0, 3, 2]
    x = with(x, dpp(x, std::integral_constant<int, 0x4E>()));   // quad_perm [2, 3, 0, 1]
    x = with(x, dpp(x, std::integral_constant<int, 0x141>()));  // row_half_mirror
    return x;
}

__device__ inline u32x4 focus_bf16x8(u32x4 x, int p) {
    float r[8] = {bf16_lo(x[0]), bf16_hi(x[0]), bf16_lo(x[1]), bf16_hi(x[1]),
                  bf16_lo(x[2]), bf16_hi(x[2]), bf16_lo(x[3]), bf16_hi(x[3])};
    float top = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        r[e] = fmaxf(r[e], 0.f);
        top = fmaxf(top, r[e]);
    }
    top = row8_combine(top, true);
    const float inv_top = top > 0.f ? __builtin_amdgcn_rcpf(top) : 0.f;
    float y[8], ss = 0.f, sy = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        r[e] *= inv_top;
        y[e] = r[e];
    }
    for (int i = 1; i < p; ++i) {  // uniform trip count
#pragma unroll
        for (int e = 0; e < 8; ++e) y[e] *= r[e];
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        ss = fmaf(r[e], r[e], ss);
        sy = fmaf(y[e], y[e], sy);
    }
    ss = row8_combine(ss, false);
    sy = row8_combine(sy, false);
    // |r| = top * sqrt(ss); sy >= 1 whenever top > 0 (the largest entry contributes 1)
    const float scale = top > 0.f ? top * __builtin_amdgcn_sqrtf(ss) * __builtin_amdgcn_rsqf(sy) : 0.f;
    u32x4 out = {pack_bf16x2(y[0] * scale, y[1] * scale), pack_bf16x2(y[2] * scale, y[3] * scale),
                 pack_bf16x2(y[4] * scale, y[5] * scale), pack_bf16x2(y[6] * scale, y[7] * scale)};
    return out;
}
__device__ inline u32x4 feature_map_bf16x8(u32x4 x, int focus_p) {
    return focus_p > 1 ? focus_bf16x8(x, focus_p) : relu_bf16x8(x);  // uniform
}

constexpr int kWaveLds = 64 * 68 * 4;  // per-wave LDS: K and V tiles (16 KB) or a padded state
constexpr int kStateLds = 4 * kWaveLds + 2 * 8 * kHeadDim * 4;

// grid (8 * ceil(n_split * B*heads / 8)), 256 threads, kStateLds bytes of dynamic LDS.
// VSUM: also write the chunk's token sum of V (the input of the dynamic-filter generator of
// the block's convolution branch) to vsum[part][bh][64]; it falls out of the V operands.
// KEEP_V: the apply pass reads V again (convolution branch), so V is loaded with the default
// cache policy; K, and V otherwise, are read once and loaded as a stream.
template <bool VSUM, bool KEEP_V>
__global__ void __launch_bounds__(256, 2)
la_state_bf16(TensorArg kt, TensorArg vt, float *__restrict__ ws, float *__restrict__ vsum,
              int heads, int N, int chunk, int focus_p, int n_split, int BH) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 5;
    // Items are the (batch * head, chunk) pairs, chunk fastest.  The hardware deals consecutive
    // workgroups to the eight XCDs in turn; workgroup w takes item (w % 8) * ceil(items / 8) + w / 8,
    // so that an XCD walks a contiguous range of heads -- the same heads whose partial states
    // la_combine sums on that XCD and whose token chunks the apply pass gives it: the states stay
    // in one L2 from pass to pass (8 x 4096 tokens x 16 heads: 58.2 -> 56.1 us for the layer; 2 x
    // 16 384 tokens: 61 -> 59 us).
    const int items = n_split * BH, per_xcd = (items + 7) >> 3;
    const int item = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (item >= items) return;  // whole workgroup
    const int bh = item / n_split, b = bh / heads, h = bh % heads, part = item % n_split;
    const __bf16 *kp = (const __bf16 *)kt.ptr + b * kt.sb + h * kt.sh;
    const __bf16 *vp = (const __bf16 *)vt.ptr + b * vt.sb + h * vt.sh;
    unsigned char *ktile = smem + wave * kWaveLds;
    unsigned char *vtile = ktile + 8192;
    const int n0 = part * chunk, n1 = min(N, n0 + chunk);
    const int lrow = lane >> 3, lchunk = lane & 7;

    f32x16 acc[2][2];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;
    float zacc[2] = {0.f, 0.f}, vacc[2] = {0.f, 0.f};

    u32x4 kreg[8], vreg[8];
    auto fetch = [&](int t0) {
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int n = t0 + r * 8 + lrow;
            u32x4 zero = {0u, 0u, 0u, 0u};
            kreg[r] = zero;
            vreg[r] = zero;
            if (n < n1) {
                kreg[r] = ld_stream((const u32x4 *)(kp + (long long)n * kt.sn + lchunk * 8));
                const u32x4 *vsrc = (const u32x4 *)(vp + (long long)n * vt.sn + lchunk * 8);
                vreg[r] = KEEP_V ? *vsrc : ld_stream(vsrc);
            }
        }
    };

    int t = n0 + wave * 64;
    if (t < n1) fetch(t);
    for (; t < n1; t += 256) {
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const unsigned off = tile_off_tr(r * 8 + lrow, lchunk);
            *(u32x4 *)(ktile + off) = feature_map_bf16x8(kreg[r], focus_p);
            *(u32x4 *)(vtile + off) = vreg[r];
        }
        if (t + 256 < n1) fetch(t + 256);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            bf16x8 a[2], bv[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                a[i] = load_tr_operand(ktile, 16 * ks, i, lane);
                bv[i] = load_tr_operand(vtile, 16 * ks, i, lane);
            }
#pragma unroll
            for (int mi = 0; mi < 2; ++mi) {
                u32x4 au = as_u32x4(a[mi]);
#pragma unroll
                for (int w = 0; w < 4; ++w) zacc[mi] = add_bf16x2(au[w], zacc[mi]);
#pragma unroll
                for (int ni = 0; ni < 2; ++ni) acc[mi][ni] = mfma32(a[mi], bv[ni], acc[mi][ni]);
            }
            if (VSUM) {
#pragma unroll
                for (int ni = 0; ni < 2; ++ni) {
                    u32x4 bu = as_u32x4(bv[ni]);
#pragma unroll
                    for (int w = 0; w < 4; ++w) vacc[ni] = add_bf16x2(bu[w], vacc[ni]);
                }
            }
        }
    }

    // Cross-wave sum through LDS, in a fixed order.
    __syncthreads();
    float *mine = (float *)(smem + wave * kWaveLds);
    float *zbuf = (float *)(smem + 4 * kWaveLds);
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int c2 = 32 * ni + (lane & 31), c1 = 32 * mi + 8 * q4 + 4 * g;
                f32x4 val = {acc[mi][ni][4 * q4], acc[mi][ni][4 * q4 + 1], acc[mi][ni][4 * q4 + 2],
                             acc[mi][ni][4 * q4 + 3]};
                *(f32x4 *)(mine + c2 * 68 + c1) = val;
            }
#pragma unroll
    for (int mi = 0; mi < 2; ++mi) {
        zbuf[(wave * 2 + g) * kHeadDim + 32 * mi + (lane & 31)] = zacc[mi];
        if (VSUM) zbuf[(8 + wave * 2 + g) * kHeadDim + 32 * mi + (lane & 31)] = vacc[mi];
    }
    __syncthreads();
    float *out = ws + ((size_t)part * BH + bh) * kStateFloats;
#pragma unroll
    for (int i = 0; i < kHeadDim * kHeadDim / 4 / 256; ++i) {  // 16-byte pieces, 4 per thread
        const int e4 = tid + 256 * i, at = (e4 >> 4) * 68 + (e4 & 15) * 4;
        f32x4 s = *(const f32x4 *)((const float *)smem + at);
#pragma unroll
        for (int w = 1; w < 4; ++w) s += *(const f32x4 *)((const float *)(smem + w * kWaveLds) + at);
        *(f32x4 *)(out + 4 * e4) = s;
    }
    if (tid < kHeadDim) {
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < 8; ++w) s += zbuf[w * kHeadDim + tid];
        out[kHeadDim * kHeadDim + tid] = s;
    } else if (VSUM && tid < 2 * kHeadDim) {
        float s = 0.f;
#pragma unroll
        for (int w = 8; w < 16; ++w) s += zbuf[w * kHeadDim + tid - kHeadDim];
        vsum[((size_t)part * BH + bh) * kHeadDim + tid - kHeadDim] = s;
    }
}

// grid (B*heads, or 8 * ceil(B*heads / 8) with xcd_ranges; ceil((kStateFloats + 64) / 1024)), 256
// threads: dst[bh] = sum_p ws[p][bh], one
// 16-byte piece per thread, the loads of eight partials in flight at a time.  With vsum (the
// partial token sums of V, [n_split][B*heads][64]) the sixteen threads after the state's last
// piece sum those too, into partial 0 (each element is read and written by one thread).
__global__ void __launch_bounds__(256)
la_combine(const float *__restrict__ ws, float *__restrict__ dst, float *vsum, int n_split, int BH, int xcd_ranges) {
    // xcd_ranges: states in contiguous ranges per XCD, as la_state_bf16 and la_apply_bf16 take them
    const int bh = xcd_ranges ? (blockIdx.x & 7) * ((BH + 7) >> 3) + (blockIdx.x >> 3) : blockIdx.x;
    if (bh >= BH) return;  // whole workgroup
    const int e4 = blockIdx.y * 256 + threadIdx.x;
    constexpr int kStateVec = kStateFloats / 4, kSumVec = kHeadDim / 4;
    if (e4 >= kStateVec + kSumVec || (e4 >= kStateVec && !vsum)) return;
    const bool state = e4 < kStateVec;
    const f32x4 *src = state ? (const f32x4 *)ws + (size_t)bh * kStateVec + e4
                             : (const f32x4 *)vsum + (size_t)bh * kSumVec + (e4 - kStateVec);
    const size_t stride4 = (size_t)BH * (state ? kStateVec : kSumVec);
    f32x4 sum = {0.f, 0.f, 0.f, 0.f};
    for (int p0 = 0; p0 < n_split; p0 += 8) {
        f32x4 part[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            f32x4 zero = {0.f, 0.f, 0.f, 0.f};
            part[i] = p0 + i < n_split ? src[(size_t)(p0 + i) * stride4] : zero;
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) sum += part[i];
    }
    if (state) ((f32x4 *)dst)[(size_t)bh * kStateVec + e4] = sum;
    else ((f32x4 *)vsum)[(size_t)bh * kSumVec + (e4 - kStateVec)] = sum;
}

// grid (8 * ceil(n_chunks * B*heads / 8)), 256 threads.  Workgroups are dealt to the eight XCDs
// in turn; the index is remapped so that the workgroups one XCD receives walk (batch, head)
// pairs chunk by chunk: the token chunks of a pair then share that XCD's L2 copy of the state.
// `states` holds n_part partial states per (batch, head), part_stride floats apart.
// KS = 0: linear attention alone.  KS = 3 or 5: the block's convolution branch is added before
// the store: the normalised tile is staged in LDS as fp32, and the lane that stores 8 channels
// of 4 consecutive tokens first adds sum_taps kappa[c][tap] * V[token + tap][c] for them (V rows
// of the neighbouring tokens come from the caches: every V row is used by KS*KS tokens).
template <bool O_BF16, int KS>
__global__ void __launch_bounds__(256, 2)
la_apply_bf16(TensorArg qt, TensorArg ot, const float *__restrict__ states, int n_part,
              long long part_stride, int heads, int N, int tokens_per_wg, int n_chunks, int n_wg,
              float eps, TensorArg vt, DwcArg cv, int focus_p) {
    // St[c2][c1] fp32 with the 8-float group index rotated by the row, then z; afterwards the
    // same bytes stage output tiles (4 KB of bf16 per wave, or 8 KB of fp32 with the
    // convolution).  Then one 8 KB query tile per wave, then the filters as [tap][channel].
    constexpr int kStageBytes = KS ? 4 * 8192 : kStateFloats * 4;
    __shared__ __align__(16) unsigned char smem[kStageBytes + 4 * 8192 + KS * KS * kHeadDim * 4];
    float *St = (float *)smem;
    float *zs = St + kHeadDim * kHeadDim;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 5, li = lane & 31;
    const int per_xcd = (n_wg + 7) / 8;
    const int wg = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (wg >= n_wg) return;  // whole workgroup
    const int bh = wg / n_chunks, b = bh / heads, h = bh % heads;
    const __bf16 *qp = (const __bf16 *)qt.ptr + b * qt.sb + h * qt.sh;
    const int n0 = (wg % n_chunks) * tokens_per_wg, n1 = min(N, n0 + tokens_per_wg);
    const int lrow = lane >> 3, lchunk = lane & 7;

    // Query tiles are fetched one step ahead; start the first fetch before the state prologue.
    u32x4 qreg[8];
    auto fetch = [&](int t0) {
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int n = t0 + r * 8 + lrow;
            u32x4 zero = {0u, 0u, 0u, 0u};
            qreg[r] = zero;
            if (n < n1) qreg[r] = ld_stream((const u32x4 *)(qp + (long long)n * qt.sn + lchunk * 8));
        }
    };
    int t = n0 + wave * 64;
    if (t < n1) fetch(t);

    float *kap = (float *)(smem + kStageBytes + 4 * 8192);
    if (KS) {
        const float *kbase = cv.kappa + b * cv.kappa_sb + (size_t)h * kHeadDim * KS * KS;
        for (int e = tid; e < kHeadDim * KS * KS; e += 256) kap[(e % (KS * KS)) * kHeadDim + e / (KS * KS)] = kbase[e];
    }

    // Sum the partial states: 16-byte loads, all of them issued before the first use.
    {
        const f32x4 *src = (const f32x4 *)(states + (size_t)bh * kStateFloats);
        const long long stride4 = part_stride / 4;
        constexpr int kVec = kStateFloats / 4, kIter = (kVec + 255) / 256;
        f32x4 part[kIter][4];
#pragma unroll
        for (int it = 0; it < kIter; ++it)
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const int e4 = it * 256 + tid;
                f32x4 zero = {0.f, 0.f, 0.f, 0.f};
                part[it][p] = (e4 < kVec && p < n_part) ? src[p * stride4 + e4] : zero;
            }
#pragma unroll
        for (int it = 0; it < kIter; ++it) {
            const int e4 = it * 256 + tid;
            if (e4 >= kVec) break;
            f32x4 sum = part[it][0];
            for (int p = 4; p < n_part; ++p) sum += src[p * stride4 + e4];  // more than 4: rare
#pragma unroll
            for (int p = 1; p < 4; ++p) sum += part[it][p];
            const int e = 4 * e4;
            if (e < kHeadDim * kHeadDim) {
                const int c2 = e >> 6, c1 = e & 63;  // 4 consecutive c1 stay inside one group
                *(f32x4 *)(St + c2 * 64 + ((((c1 >> 3) ^ (c2 & 7)) << 3) | (c1 & 7))) = sum;
            } else {
                *(f32x4 *)(zs + e - kHeadDim * kHeadDim) = sum;
            }
        }
    }
    __syncthreads();

    // A operands: S^T rows c2 = 32*mi + li, k-slots c1 = 16*ks + 8g + (0..7), as bf16 hi + lo.
    bf16x8 s_hi[2][4], s_lo[2][4], z_op[4];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const int c2 = 32 * mi + li, grp = 2 * ks + g;
            const float *row = St + c2 * 64 + ((grp ^ (c2 & 7)) << 3);
            f32x4 x0 = *(const f32x4 *)row, x1 = *(const f32x4 *)(row + 4);
            float x[8] = {x0[0], x0[1], x0[2], x0[3], x1[0], x1[1], x1[2], x1[3]};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                __bf16 hi = (__bf16)x[e];
                s_hi[mi][ks][e] = hi;
                s_lo[mi][ks][e] = (__bf16)(x[e] - (float)hi);
            }
        }
    // Denominator block: row 0 = z high part, row 1 = z low part, other rows zero.
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float zv = zs[16 * ks + 8 * g + e];
            const __bf16 hi = (__bf16)zv;
            const __bf16 lo = (__bf16)(zv - (float)hi);
            z_op[ks][e] = li == 0 ? hi : (li == 1 ? lo : (__bf16)0.f);
        }
    __syncthreads();  // the state bytes are reused as output staging from here on

    unsigned char *qtile = smem + kStageBytes + wave * 8192;
    unsigned char *otile = smem + wave * (KS ? 8192 : 4096);
    const __bf16 *vp = (const __bf16 *)vt.ptr + b * vt.sb + h * vt.sh;
    for (; t < n1; t += 256) {
#pragma unroll
        for (int r = 0; r < 8; ++r)
            *(u32x4 *)(qtile + tile_off_row(r * 8 + lrow, lchunk)) = feature_map_bf16x8(qreg[r], focus_p);
        if (t + 256 < n1) fetch(t + 256);
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            if (t + 32 * nt >= n1) break;  // wave-uniform
            const int row = 32 * nt + li;
            f32x16 acc[2], accz;
#pragma unroll
            for (int v = 0; v < 16; ++v) { acc[0][v] = 0.f; acc[1][v] = 0.f; accz[v] = 0.f; }
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const bf16x8 qb = as_bf16x8(*(const u32x4 *)(qtile + tile_off_row(row, 2 * ks + g)));
                accz = mfma32(z_op[ks], qb, accz);
#pragma unroll
                for (int mi = 0; mi < 2; ++mi) {
                    acc[mi] = mfma32(s_lo[mi][ks], qb, acc[mi]);
                    acc[mi] = mfma32(s_hi[mi][ks], qb, acc[mi]);
                }
            }
            // den lives in rows 0 and 1 of the denominator block: registers 0, 1 of lanes g = 0.
            float den_lo, den_hi;
            pair_values(accz[0] + accz[1], &den_lo, &den_hi);
            const float inv = __builtin_amdgcn_rcpf(den_lo + eps);
            const int n = t + row;
            if (KS) {
                // fp32 staging: 256-byte token rows, 16-byte chunk index rotated by the row
#pragma unroll
                for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4) {
                        f32x4 val = {acc[mi][4 * q4] * inv, acc[mi][4 * q4 + 1] * inv,
                                     acc[mi][4 * q4 + 2] * inv, acc[mi][4 * q4 + 3] * inv};
                        *(f32x4 *)(otile + li * 256 + (((8 * mi + 2 * q4 + g) ^ (li & 15)) << 4)) = val;
                    }
                // A lane finishes 4 consecutive tokens x 8 channels: the taps of neighbouring
                // tokens overlap, so one tap row needs 4 + KS - 1 loads instead of 4 * KS.
                // Out-of-grid taps (and slots past the end of the range) read a valid row with
                // weight zero, so the loads of a tap row are all in flight at once.
                constexpr int kPad = KS / 2, kSpan = 4 + KS - 1;
                const int tok0 = t + 32 * nt + 4 * lrow;            // first of this lane's tokens
                const int last = n1 - 1;
                float sum[4][8];
                int gr[4], gc[4];
                bool on_grid[4];  // prefix tokens (grid index below zero) get no convolution term
                {
                    const int g0 = min(tok0, last) - cv.P;  // grid index of the lane's first token
                    const int base = max(g0, 0);
                    int r0 = base / cv.W, c0 = base - r0 * cv.W;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int orow = 4 * lrow + r;
                        const f32x4 o0 = *(const f32x4 *)(otile + orow * 256 + (((2 * lchunk) ^ (orow & 15)) << 4));
                        const f32x4 o1 = *(const f32x4 *)(otile + orow * 256 + (((2 * lchunk + 1) ^ (orow & 15)) << 4));
                        sum[r][0] = o0[0]; sum[r][1] = o0[1]; sum[r][2] = o0[2]; sum[r][3] = o0[3];
                        sum[r][4] = o1[0]; sum[r][5] = o1[1]; sum[r][6] = o1[2]; sum[r][7] = o1[3];
                        gr[r] = r0;
                        gc[r] = c0;
                        on_grid[r] = g0 + r >= 0;
                        if (on_grid[r] && ++c0 == cv.W) { c0 = 0; ++r0; }
                    }
                }
#pragma unroll 1
                for (int di = -kPad; di <= kPad; ++di) {
                    u32x4 vv[kSpan];
#pragma unroll
                    for (int j = 0; j < kSpan; ++j) {
                        const int src = tok0 + j - kPad + di * cv.W;  // token of column j in this tap row
                        const int safe = min(max(src, 0), N - 1);
                        vv[j] = *(const u32x4 *)(vp + (long long)safe * vt.sn + lchunk * 8);
                    }
                    const float *krow = kap + (di + kPad) * KS * kHeadDim + 8 * lchunk;
#pragma unroll
                    for (int dj = -kPad; dj <= kPad; ++dj) {
                        const f32x4 k0 = *(const f32x4 *)(krow + (dj + kPad) * kHeadDim);
                        const f32x4 k1 = *(const f32x4 *)(krow + (dj + kPad) * kHeadDim + 4);
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const bool ok = tok0 + r <= last && on_grid[r] && (unsigned)(gr[r] + di) < (unsigned)cv.H &&
                                            (unsigned)(gc[r] + dj) < (unsigned)cv.W;
                            const float m = ok ? 1.0f : 0.0f;
                            const u32x4 x = vv[r + dj + kPad];
                            sum[r][0] = fmaf(k0[0] * m, bf16_lo(x[0]), sum[r][0]);
                            sum[r][1] = fmaf(k0[1] * m, bf16_hi(x[0]), sum[r][1]);
                            sum[r][2] = fmaf(k0[2] * m, bf16_lo(x[1]), sum[r][2]);
                            sum[r][3] = fmaf(k0[3] * m, bf16_hi(x[1]), sum[r][3]);
                            sum[r][4] = fmaf(k1[0] * m, bf16_lo(x[2]), sum[r][4]);
                            sum[r][5] = fmaf(k1[1] * m, bf16_hi(x[2]), sum[r][5]);
                            sum[r][6] = fmaf(k1[2] * m, bf16_lo(x[3]), sum[r][6]);
                            sum[r][7] = fmaf(k1[3] * m, bf16_hi(x[3]), sum[r][7]);
                        }
                    }
                }
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int on = tok0 + r;
                    if (on <= last) {
                        if (O_BF16) {
                            __bf16 *op = (__bf16 *)ot.ptr + b * ot.sb + h * ot.sh;
                            u32x4 pk = {pack_bf16x2(sum[r][0], sum[r][1]), pack_bf16x2(sum[r][2], sum[r][3]),
                                        pack_bf16x2(sum[r][4], sum[r][5]), pack_bf16x2(sum[r][6], sum[r][7])};
                            st_stream((u32x4 *)(op + (long long)on * ot.sn + lchunk * 8), pk);
                        } else {
                            float *op = (float *)ot.ptr + b * ot.sb + h * ot.sh + (long long)on * ot.sn + lchunk * 8;
                            f32x4 s0 = {sum[r][0], sum[r][1], sum[r][2], sum[r][3]};
                            f32x4 s1 = {sum[r][4], sum[r][5], sum[r][6], sum[r][7]};
                            *(f32x4 *)op = s0;
                            *(f32x4 *)(op + 4) = s1;
                        }
                    }
                }
            } else if (O_BF16) {
#pragma unroll
                for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4) {
                        u32x2 pk = {pack_bf16x2(acc[mi][4 * q4] * inv, acc[mi][4 * q4 + 1] * inv),
                                    pack_bf16x2(acc[mi][4 * q4 + 2] * inv, acc[mi][4 * q4 + 3] * inv)};
                        *(u32x2 *)(otile + tile_off_row(li, 4 * mi + q4) + 8 * g) = pk;
                    }
                __bf16 *op = (__bf16 *)ot.ptr + b * ot.sb + h * ot.sh;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int orow = r * 8 + lrow, on = t + 32 * nt + orow;
                    const u32x4 val = *(const u32x4 *)(otile + tile_off_row(orow, lchunk));
                    if (on < n1) st_stream((u32x4 *)(op + (long long)on * ot.sn + lchunk * 8), val);
                }
            } else {
                float *op = (float *)ot.ptr + b * ot.sb + h * ot.sh;
                if (n < n1) {
#pragma unroll
                    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                        for (int q4 = 0; q4 < 4; ++q4) {
                            f32x4 val = {acc[mi][4 * q4] * inv, acc[mi][4 * q4 + 1] * inv,
                                         acc[mi][4 * q4 + 2] * inv, acc[mi][4 * q4 + 3] * inv};
                            *(f32x4 *)(op + (long long)n * ot.sn + 32 * mi + 8 * q4 + 4 * g) = val;
                        }
                }
            }
        }
    }
}

template <bool O_BF16, int KS>
static void launch_apply(hipStream_t stream, const Problem &pr, const float *states, int n_part,
                         long long part_stride, int apply_tokens, float eps, const DwcArg &cv,
                         int focus_p) {
    const int n_chunks = (pr.N + apply_tokens - 1) / apply_tokens, n_wg = n_chunks * pr.B * pr.heads;
    hipLaunchKernelGGL((la_apply_bf16<O_BF16, KS>), dim3(8 * ((n_wg + 7) / 8)), dim3(256), 0, stream,
                       pr.q, pr.o, states, n_part, part_stride, pr.heads, pr.N, apply_tokens, n_chunks,
                       n_wg, eps, pr.v, cv, focus_p);
}

jv_status linear_bf16(const Problem &pr, const LinearPlan &plan, float eps, float *ws,
                      const DwcPlan &dwc, int focus_p, hipStream_t stream) {
    static LdsLimit lds_limit[3];
    jv_status st = ensure_lds_limit(lds_limit[0], (const void *)la_state_bf16<false, false>, kStateLds);
    if (st == JV_OK) st = ensure_lds_limit(lds_limit[1], (const void *)la_state_bf16<false, true>, kStateLds);
    if (st == JV_OK) st = ensure_lds_limit(lds_limit[2], (const void *)la_state_bf16<true, true>, kStateLds);
    if (st != JV_OK) return st;
    const int BH = pr.B * pr.heads;
    const bool dynamic = dwc.mode == JV_DWC_SQUEEZE_DYNAMIC;
    if (dynamic)
        hipLaunchKernelGGL((la_state_bf16<true, true>), dim3(8 * ((plan.n_split * BH + 7) / 8)), dim3(256), kStateLds, stream,
                           pr.k, pr.v, ws, ws + dwc.vsum_off, pr.heads, pr.N, plan.chunk, focus_p, plan.n_split, BH);
    else if (dwc.mode != JV_DWC_NONE)
        hipLaunchKernelGGL((la_state_bf16<false, true>), dim3(8 * ((plan.n_split * BH + 7) / 8)), dim3(256), kStateLds, stream,
                           pr.k, pr.v, ws, (float *)nullptr, pr.heads, pr.N, plan.chunk, focus_p, plan.n_split, BH);
    else
        hipLaunchKernelGGL((la_state_bf16<false, false>), dim3(8 * ((plan.n_split * BH + 7) / 8)), dim3(256), kStateLds, stream,
                           pr.k, pr.v, ws, (float *)nullptr, pr.heads, pr.N, plan.chunk, focus_p, plan.n_split, BH);
    if ((st = launch_status("la_state_bf16")) != JV_OK) return st;
    const float *states = ws;
    int n_part = plan.n_split;
    long long part_stride = (long long)BH * kStateFloats;
    if (plan.combine) {
        float *dst = ws + (size_t)plan.n_split * BH * kStateFloats;
        hipLaunchKernelGGL(la_combine, dim3(8 * ((BH + 7) / 8), ((kStateFloats + kHeadDim) / 4 + 255) / 256), dim3(256), 0,
                           stream, ws, dst, dynamic ? ws + dwc.vsum_off : (float *)nullptr, plan.n_split, BH, 1);
        if ((st = launch_status("la_combine")) != JV_OK) return st;
        states = dst;
        n_part = 1;
    }
    DwcArg cv = {dwc.static_kernel, 0, pr.H, pr.W, pr.P};
    if (dynamic) {
        if ((st = squeeze_generate(dwc, ws, n_part, pr.B, pr.heads, pr.N, stream)) != JV_OK) return st;
        cv.kappa = ws + dwc.kappa_off;
        cv.kappa_sb = (long long)pr.heads * kHeadDim * dwc.ksize * dwc.ksize;
    }
    const int ks = dwc.mode == JV_DWC_NONE ? 0 : dwc.ksize;
    if (pr.o_bf16) {
        if (ks == 0) launch_apply<true, 0>(stream, pr, states, n_part, part_stride, plan.apply_tokens, eps, cv, focus_p);
        else if (ks == 3) launch_apply<true, 3>(stream, pr, states, n_part, part_stride, plan.apply_tokens, eps, cv, focus_p);
        else launch_apply<true, 5>(stream, pr, states, n_part, part_stride, plan.apply_tokens, eps, cv, focus_p);
    } else {
        if (ks == 0) launch_apply<false, 0>(stream, pr, states, n_part, part_stride, plan.apply_tokens, eps, cv, focus_p);
        else if (ks == 3) launch_apply<false, 3>(stream, pr, states, n_part, part_stride, plan.apply_tokens, eps, cv, focus_p);
        else launch_apply<false, 5>(stream, pr, states, n_part, part_stride, plan.apply_tokens, eps, cv, focus_p);
    }
    return launch_status("la_apply_bf16");
}

// ---------------------------------------------------------------------------------------
// The apply pass folded into the output projection that follows a linear-attention block
// (Sec. 3.2.3: the block keeps the projection W_O it inherits).  With o_h = relu(q_h) S_h / den_h,
// den_h = relu(q_h) . z_h + eps, the projected output of a token is
//     sum_h o_h W_O[:, h]^T = sum_h (relu(q_h) / den_h) (W_O[:, h] S_h^T)^T,
// i.e. one product of the scaled queries A'[t, 64 h + i] = relu(q_h[t, i]) / den_h[t] with a
// weight matrix of the image, W'_b[n, 64 h + i] = sum_c W_O[n, 64 h + c] St_bh[c][i]  (St is the
// state as la_state_bf16 stores it, St[c][i] = sum_t relu(k[t, i]) v[t, c]).  Both operands are
// rounded to bf16 once; the product runs on the GEMM with one weight matrix per image.
// ---------------------------------------------------------------------------------------

// grid (C / 64, B*heads), 256 threads: 64 output features n x the 64 columns of head h of W'_b;
// a thread forms a 4 x 4 block of them (two 16-byte LDS reads per 16 multiply-adds), in fp32.
__global__ void __launch_bounds__(256)
la_fold_projection(const float *__restrict__ states, const __bf16 *__restrict__ w_o,
                   __bf16 *__restrict__ w_fold, int heads, int C) {
    __shared__ __align__(16) float St[kHeadDim][kHeadDim + 4];   // [c][i]
    __shared__ __align__(16) float Wt[kHeadDim][kHeadDim + 4];   // [c][n - n0]
    const int tid = threadIdx.x, bh = blockIdx.y, b = bh / heads, h = bh % heads, n0 = blockIdx.x * 64;
    const float *sp = states + (size_t)bh * kStateFloats;
    for (int e = tid; e < kHeadDim * kHeadDim; e += 256) St[e >> 6][e & 63] = sp[e];
    for (int e = tid; e < kHeadDim * kHeadDim; e += 256)
        Wt[e & 63][e >> 6] = (float)w_o[(size_t)(n0 + (e >> 6)) * C + h * kHeadDim + (e & 63)];
    __syncthreads();
    const int nb = (tid >> 4) * 4, ib = (tid & 15) * 4;
    float acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[a][i] = 0.f;
#pragma unroll 8
    for (int c = 0; c < kHeadDim; ++c) {
        const f32x4 w4 = *(const f32x4 *)&Wt[c][nb], s4 = *(const f32x4 *)&St[c][ib];
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[a][i] = fmaf(w4[a], s4[i], acc[a][i]);
    }
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        u32x2 pk = {pack_bf16x2(acc[a][0], acc[a][1]), pack_bf16x2(acc[a][2], acc[a][3])};
        *(u32x2 *)(w_fold + ((size_t)b * C + n0 + nb + a) * C + h * kHeadDim + ib) = pk;
    }
}

// grid (ceil(B * N * heads / 32)), 256 threads: 8 lanes per (token, head) row of 64 channels, rows in
// the order (batch, token, head), so that a workgroup writes 4 KB of consecutive bytes of a_out.
__global__ void __launch_bounds__(256)
la_scale_queries(TensorArg qt, const float *__restrict__ states, __bf16 *__restrict__ a_out, int heads,
                 int N, long long rows, float eps) {
    const long long row = (long long)blockIdx.x * 32 + (threadIdx.x >> 3);
    if (row >= rows) return;  // all eight lanes of a row together
    const int l8 = threadIdx.x & 7;
    const int h = (int)(row % heads);
    const long long tn = row / heads;
    const int n = (int)(tn % N), b = (int)(tn / N);
    const u32x4 q = relu_bf16x8(ld_stream((const u32x4 *)((const __bf16 *)qt.ptr + b * qt.sb + h * qt.sh + (long long)n * qt.sn + l8 * 8)));
    const float *zp = states + ((size_t)b * heads + h) * kStateFloats + kHeadDim * kHeadDim + l8 * 8;
    const f32x4 z0 = *(const f32x4 *)zp, z1 = *(const f32x4 *)(zp + 4);
    float r[8] = {bf16_lo(q[0]), bf16_hi(q[0]), bf16_lo(q[1]), bf16_hi(q[1]),
                  bf16_lo(q[2]), bf16_hi(q[2]), bf16_lo(q[3]), bf16_hi(q[3])};
    float den = r[0] * z0[0] + r[1] * z0[1] + r[2] * z0[2] + r[3] * z0[3] +
                r[4] * z1[0] + r[5] * z1[1] + r[6] * z1[2] + r[7] * z1[3];
    den += __shfl_xor(den, 1, 64);
    den += __shfl_xor(den, 2, 64);
    den += __shfl_xor(den, 4, 64);
    const float inv = 1.0f / (den + eps);
    u32x4 out = {pack_bf16x2(r[0] * inv, r[1] * inv), pack_bf16x2(r[2] * inv, r[3] * inv),
                 pack_bf16x2(r[4] * inv, r[5] * inv), pack_bf16x2(r[6] * inv, r[7] * inv)};
    st_stream((u32x4 *)(a_out + ((size_t)tn * heads + h) * kHeadDim + l8 * 8), out);
}

// State pass, sum of the partial states into `states` ([B*heads][kStateFloats], one per head),
// then the two operands of the fused projection: w_fold [B][C][C] and a_out [B*N][C], C = 64 heads.
// ws: the linear-attention workspace (the partial states).  64-channel heads, ReLU map, no
// convolution branch (the caller checks).
jv_status linear_fused_projection_operands(const Problem &pr, float eps, float *ws, float *states,
                                           const void *w_o, void *w_fold, void *a_out, hipStream_t stream) {
    static LdsLimit lds_limit;
    jv_status st = ensure_lds_limit(lds_limit, (const void *)la_state_bf16<false, false>, kStateLds);
    if (st != JV_OK) return st;
    const LinearPlan plan = plan_linear(pr.B, pr.heads, pr.N);
    const int BH = pr.B * pr.heads, C = pr.heads * kHeadDim;
    hipLaunchKernelGGL((la_state_bf16<false, false>), dim3(8 * ((plan.n_split * BH + 7) / 8)), dim3(256), kStateLds, stream,
                       pr.k, pr.v, ws, (float *)nullptr, pr.heads, pr.N, plan.chunk, 1, plan.n_split, BH);
    if ((st = launch_status("la_state_bf16")) != JV_OK) return st;
    hipLaunchKernelGGL(la_combine, dim3(8 * ((BH + 7) / 8), ((kStateFloats + kHeadDim) / 4 + 255) / 256), dim3(256), 0,
                       stream, ws, states, (float *)nullptr, plan.n_split, BH, 1);
    if ((st = launch_status("la_combine")) != JV_OK) return st;
    hipLaunchKernelGGL(la_fold_projection, dim3(C / 64, BH), dim3(256), 0, stream, states, (const __bf16 *)w_o,
                       (__bf16 *)w_fold, pr.heads, C);
    if ((st = launch_status("la_fold_projection")) != JV_OK) return st;
    const long long rows = (long long)pr.B * pr.N * pr.heads;
    hipLaunchKernelGGL(la_scale_queries, dim3((unsigned)((rows + 31) / 32)), dim3(256), 0, stream, pr.q, states,
                       (__bf16 *)a_out, pr.heads, pr.N, rows, eps);
    return launch_status("la_scale_queries");
}

// ---------------------------------------------------------------------------------------
// head_dim 128.  la_state_wide_bf16 (below) leaves four 64 x 64 quadrant states per head,
// la_combine sums the partial ones; this is the apply pass:
//   o[c2] = sum_i relu(q_i) S_ij[:, c2] / (sum_i relu(q_i) . z_i + eps),   j = c2 / 64,
// q_i the two 64-channel halves of a query row.  A workgroup streams one token chunk of one
// (batch, head); its four wavefronts own the four 32-channel quarters of the output, each with
// the matching rows of S_0j^T and S_1j^T as bf16 high + low operands in registers (what a
// wavefront of the 64-channel kernel holds for its 64 output channels), and all four run over
// the same 64-token query tile in LDS; the denominator is one more row block, as there.
// KS = 3 or 5: the block's convolution branch is added before the store, as in la_apply_bf16:
// the normalised tile is staged as fp32 (512-byte token rows, the 16-byte chunk index rotated
// by the row), and the thread that stores 8 channels of 4 consecutive tokens first adds
// sum_taps kappa[c][tap] * V[token + tap][c] for them; the sum is rounded once.
// grid (n_chunks * B*heads), 256 threads.
// ---------------------------------------------------------------------------------------
template <bool O_BF16, int KS>
__global__ void __launch_bounds__(256, 2)
la_apply_wide_bf16(TensorArg qt, TensorArg ot, const float *__restrict__ states, int heads, int N,
                   int tokens_per_wg, int n_chunks, float eps, TensorArg vt, DwcArg cv) {
    // query tile [64 tokens][256 B]; output tile (bf16 rows of 256 B, or fp32 rows of 512 B with
    // the convolution); the filters as [tap][channel]
    constexpr int kOutBytes = KS ? 32768 : 16384;
    __shared__ __align__(16) unsigned char smem[16384 + kOutBytes + KS * KS * kHeadDimWide * 4];
    unsigned char *qtile = smem, *otile = smem + 16384;
    float *kap = (float *)(smem + 16384 + kOutBytes);
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 5, li = lane & 31;
    const int bh = blockIdx.x / n_chunks, b = bh / heads, h = bh % heads;
    const __bf16 *qp = (const __bf16 *)qt.ptr + b * qt.sb + h * qt.sh;
    const int n0 = (blockIdx.x % n_chunks) * tokens_per_wg, n1 = min(N, n0 + tokens_per_wg);
    const int frow = tid >> 4, fchunk = tid & 15;  // this thread's 16 bytes of rows frow + 16 r of a tile

    u32x4 qreg[4];
    auto fetch = [&](int t0) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int n = t0 + 16 * r + frow;
            u32x4 zero = {0u, 0u, 0u, 0u};
            qreg[r] = zero;
            if (n < n1) qreg[r] = ld_stream((const u32x4 *)(qp + (long long)n * qt.sn + fchunk * 8));
        }
    };
    fetch(n0);
    if (KS) {  // (read after the first barrier of the token loop)
        const float *kbase = cv.kappa + b * cv.kappa_sb + (size_t)h * kHeadDimWide * KS * KS;
        for (int e = tid; e < kHeadDimWide * KS * KS; e += 256) kap[(e % (KS * KS)) * kHeadDimWide + e / (KS * KS)] = kbase[e];
    }

    // A operands: rows c2 of S_ij^T (this wavefront's quarter), k-slots c1 = 16 ks + 8 g + (0..7).
    const int j = wave >> 1, c2 = 32 * (wave & 1) + li;
    bf16x8 s_hi[2][4], s_lo[2][4], z_op[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const float *st = states + ((size_t)bh * 4 + 2 * i + j) * kStateFloats;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const float *row = st + c2 * kHeadDim + 16 * ks + 8 * g;
            const float *zrow = st + kHeadDim * kHeadDim + 16 * ks + 8 * g;
            const f32x4 x0 = *(const f32x4 *)row, x1 = *(const f32x4 *)(row + 4);
            const f32x4 z0 = *(const f32x4 *)zrow, z1 = *(const f32x4 *)(zrow + 4);
            const float x[8] = {x0[0], x0[1], x0[2], x0[3], x1[0], x1[1], x1[2], x1[3]};
            const float zv[8] = {z0[0], z0[1], z0[2], z0[3], z1[0], z1[1], z1[2], z1[3]};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const __bf16 hi = (__bf16)x[e];
                s_hi[i][ks][e] = hi;
                s_lo[i][ks][e] = (__bf16)(x[e] - (float)hi);
                // denominator block: row 0 = z high part, row 1 = z low part, other rows zero
                const __bf16 zh = (__bf16)zv[e];
                const __bf16 zl = (__bf16)(zv[e] - (float)zh);
                z_op[i][ks][e] = li == 0 ? zh : (li == 1 ? zl : (__bf16)0.f);
            }
        }
    }

    const __bf16 *vp = (const __bf16 *)vt.ptr + b * vt.sb + h * vt.sh;
    for (int t = n0; t < n1; t += 64) {
        __syncthreads();  // the previous tile has been read, and its output rows stored
#pragma unroll
        for (int r = 0; r < 4; ++r)
            *(u32x4 *)(qtile + wide_off_row(16 * r + frow, fchunk)) = relu_bf16x8(qreg[r]);
        if (t + 64 < n1) fetch(t + 64);
        __syncthreads();
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            if (t + 32 * nt >= n1) break;  // the same for every wavefront of the workgroup
            f32x16 acc, accz;
#pragma unroll
            for (int v = 0; v < 16; ++v) { acc[v] = 0.f; accz[v] = 0.f; }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    const bf16x8 qb = as_bf16x8(*(const u32x4 *)(qtile + wide_off_row(32 * nt + li, 2 * (4 * i + ks) + g)));
                    accz = mfma32(z_op[i][ks], qb, accz);
                    acc = mfma32(s_lo[i][ks], qb, acc);
                    acc = mfma32(s_hi[i][ks], qb, acc);
                }
            // den lives in rows 0 and 1 of the denominator block: registers 0, 1 of lanes g = 0.
            float den_lo, den_hi;
            pair_values(accz[0] + accz[1], &den_lo, &den_hi);
            const float inv = __builtin_amdgcn_rcpf(den_lo + eps);
            if (KS) {
                const int row = 32 * nt + li;
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    f32x4 val = {acc[4 * q4] * inv, acc[4 * q4 + 1] * inv, acc[4 * q4 + 2] * inv, acc[4 * q4 + 3] * inv};
                    *(f32x4 *)(otile + row * 512 + (((8 * wave + 2 * q4 + g) ^ (row & 15)) << 4)) = val;
                }
            } else if (O_BF16) {
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    u32x2 pk = {pack_bf16x2(acc[4 * q4] * inv, acc[4 * q4 + 1] * inv),
                                pack_bf16x2(acc[4 * q4 + 2] * inv, acc[4 * q4 + 3] * inv)};
                    *(u32x2 *)(otile + wide_off_row(32 * nt + li, 4 * wave + q4) + 8 * g) = pk;
                }
            } else {
                const int n = t + 32 * nt + li;
                float *op = (float *)ot.ptr + b * ot.sb + h * ot.sh;
                if (n < n1) {
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4) {
                        f32x4 val = {acc[4 * q4] * inv, acc[4 * q4 + 1] * inv, acc[4 * q4 + 2] * inv, acc[4 * q4 + 3] * inv};
                        *(f32x4 *)(op + (long long)n * ot.sn + 32 * wave + 8 * q4 + 4 * g) = val;
                    }
                }
            }
        }
        if (KS) {
            __syncthreads();  // the four quarters of every row are in the output tile
            // This thread finishes channels 8 fchunk .. + 7 of tokens tok0 .. tok0 + 3: the taps of
            // neighbouring tokens overlap, so one tap row needs 4 + KS - 1 loads instead of 4 * KS.
            // Out-of-grid taps (and tokens past the end of the range) read a valid row with
            // weight zero, so the loads of a tap row are all in flight at once.
            constexpr int kPad = KS / 2, kSpan = 4 + KS - 1;
            const int tok0 = t + 4 * frow, last = n1 - 1;
            float sum[4][8];
            int gr[4], gc[4];
            bool on_grid[4];  // prefix tokens (grid index below zero) get no convolution term
            {
                const int g0 = min(tok0, last) - cv.P;  // grid index of the thread's first token
                const int base = max(g0, 0);
                int r0 = base / cv.W, c0 = base - r0 * cv.W;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int orow = 4 * frow + r;
                    const f32x4 o0 = *(const f32x4 *)(otile + orow * 512 + (((2 * fchunk) ^ (orow & 15)) << 4));
                    const f32x4 o1 = *(const f32x4 *)(otile + orow * 512 + (((2 * fchunk + 1) ^ (orow & 15)) << 4));
                    sum[r][0] = o0[0]; sum[r][1] = o0[1]; sum[r][2] = o0[2]; sum[r][3] = o0[3];
                    sum[r][4] = o1[0]; sum[r][5] = o1[1]; sum[r][6] = o1[2]; sum[r][7] = o1[3];
                    gr[r] = r0;
                    gc[r] = c0;
                    on_grid[r] = g0 + r >= 0;
                    if (on_grid[r] && ++c0 == cv.W) { c0 = 0; ++r0; }
                }
            }
#pragma unroll 1
            for (int di = -kPad; di <= kPad; ++di) {
                u32x4 vv[kSpan];
#pragma unroll
                for (int jj = 0; jj < kSpan; ++jj) {
                    const int src = tok0 + jj - kPad + di * cv.W;  // token of column jj in this tap row
                    const int safe = min(max(src, 0), N - 1);
                    vv[jj] = *(const u32x4 *)(vp + (long long)safe * vt.sn + fchunk * 8);
                }
                const float *krow = kap + (di + kPad) * KS * kHeadDimWide + 8 * fchunk;
#pragma unroll
                for (int dj = -kPad; dj <= kPad; ++dj) {
                    const f32x4 k0 = *(const f32x4 *)(krow + (dj + kPad) * kHeadDimWide);
                    const f32x4 k1 = *(const f32x4 *)(krow + (dj + kPad) * kHeadDimWide + 4);
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const bool ok = tok0 + r <= last && on_grid[r] && (unsigned)(gr[r] + di) < (unsigned)cv.H &&
                                        (unsigned)(gc[r] + dj) < (unsigned)cv.W;
                        const float m = ok ? 1.0f : 0.0f;
                        const u32x4 x = vv[r + dj + kPad];
                        sum[r][0] = fmaf(k0[0] * m, bf16_lo(x[0]), sum[r][0]);
                        sum[r][1] = fmaf(k0[1] * m, bf16_hi(x[0]), sum[r][1]);
                        sum[r][2] = fmaf(k0[2] * m, bf16_lo(x[1]), sum[r][2]);
                        sum[r][3] = fmaf(k0[3] * m, bf16_hi(x[1]), sum[r][3]);
                        sum[r][4] = fmaf(k1[0] * m, bf16_lo(x[2]), sum[r][4]);
                        sum[r][5] = fmaf(k1[1] * m, bf16_hi(x[2]), sum[r][5]);
                        sum[r][6] = fmaf(k1[2] * m, bf16_lo(x[3]), sum[r][6]);
                        sum[r][7] = fmaf(k1[3] * m, bf16_hi(x[3]), sum[r][7]);
                    }
                }
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int on = tok0 + r;
                if (on <= last) {
                    if (O_BF16) {
                        __bf16 *op = (__bf16 *)ot.ptr + b * ot.sb + h * ot.sh;
                        u32x4 pk = {pack_bf16x2(sum[r][0], sum[r][1]), pack_bf16x2(sum[r][2], sum[r][3]),
                                    pack_bf16x2(sum[r][4], sum[r][5]), pack_bf16x2(sum[r][6], sum[r][7])};
                        st_stream((u32x4 *)(op + (long long)on * ot.sn + fchunk * 8), pk);
                    } else {
                        float *op = (float *)ot.ptr + b * ot.sb + h * ot.sh + (long long)on * ot.sn + fchunk * 8;
                        f32x4 s0 = {sum[r][0], sum[r][1], sum[r][2], sum[r][3]};
                        f32x4 s1 = {sum[r][4], sum[r][5], sum[r][6], sum[r][7]};
                        *(f32x4 *)op = s0;
                        *(f32x4 *)(op + 4) = s1;
                    }
                }
            }
        } else if (O_BF16) {
            __syncthreads();  // the four quarters of every row are in the output tile
            __bf16 *op = (__bf16 *)ot.ptr + b * ot.sb + h * ot.sh;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = 16 * r + frow, n = t + row;
                const u32x4 val = *(const u32x4 *)(otile + wide_off_row(row, fchunk));
                if (n < n1) st_stream((u32x4 *)(op + (long long)n * ot.sn + fchunk * 8), val);
            }
        }
    }
}

// State pass for heads of 128 channels: S = relu(K)^T V (128 x 128) and z = sum relu(K) of one
// token chunk, K and V read once.  The workgroup's four wavefronts share tiles of 64 tokens in
// LDS -- K (rectified) and V, each as two half tiles of 64 channels in the tile_off_tr layout --
// and wavefront 2i + j accumulates the quadrant S_ij = relu(K_i)^T V_j (channels 64i .. 64i+63
// of K against 64j .. 64j+63 of V) exactly as la_state_bf16 accumulates its one state, and z_i.
// Two tile buffers: the next tile is fetched into registers while this one is reduced, and
// stored after it; one barrier per tile.  The quadrants are written as four states of
// kStateFloats floats, quadrant 2i + j of (batch, head) bh at index 4 bh + 2i + j of `part`.
// VSUM: also write the chunk's token sum of V (the input of the dynamic-filter generator of the
// block's convolution branch) to vsum[part][bh][128]; it falls out of the V operands of the
// wavefronts with i = 0.
// grid (n_split, B*heads), 256 threads, kStateWideLds bytes of dynamic LDS.
constexpr int kStateWideLds = 2 * 4 * 8192;

template <bool VSUM>
__global__ void __launch_bounds__(256, 2)
la_state_wide_bf16(TensorArg kt, TensorArg vt, float *__restrict__ ws, float *__restrict__ vsum, int heads, int N,
                   int chunk) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int bh = blockIdx.y, b = bh / heads, h = bh % heads, part = blockIdx.x;
    const int BH = gridDim.y;
    const __bf16 *kp = (const __bf16 *)kt.ptr + b * kt.sb + h * kt.sh;
    const __bf16 *vp = (const __bf16 *)vt.ptr + b * vt.sb + h * vt.sh;
    const int n0 = part * chunk, n1 = min(N, n0 + chunk);
    // loads: 16 threads per token row (one 16-byte chunk each), 16 rows per pass, 4 passes per tile
    const int lrow = tid >> 4, lchunk = tid & 15;
    const int qi = wave >> 1, qj = wave & 1;

    f32x16 acc[2][2];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;
    float zacc[2] = {0.f, 0.f}, vacc[2] = {0.f, 0.f};

    u32x4 kreg[4], vreg[4];
    auto fetch = [&](int t0) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int n = t0 + r * 16 + lrow;
            u32x4 zero = {0u, 0u, 0u, 0u};
            kreg[r] = zero;
            vreg[r] = zero;
            if (n < n1) {
                kreg[r] = ld_stream((const u32x4 *)(kp + (long long)n * kt.sn + lchunk * 8));
                vreg[r] = ld_stream((const u32x4 *)(vp + (long long)n * vt.sn + lchunk * 8));
            }
        }
    };
    auto stash = [&](int buf) {
        unsigned char *kt0 = smem + buf * 32768 + (lchunk >> 3) * 8192, *vt0 = kt0 + 16384;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const unsigned off = tile_off_tr(r * 16 + lrow, lchunk & 7);
            *(u32x4 *)(kt0 + off) = relu_bf16x8(kreg[r]);
            *(u32x4 *)(vt0 + off) = vreg[r];
        }
    };

    int buf = 0;
    if (n0 < n1) fetch(n0);
    for (int t = n0; t < n1; t += 64) {
        stash(buf);
        __syncthreads();
        if (t + 64 < n1) fetch(t + 64);
        const unsigned char *ktile = smem + buf * 32768 + qi * 8192;
        const unsigned char *vtile = smem + buf * 32768 + 16384 + qj * 8192;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            bf16x8 a[2], bv[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                a[i] = load_tr_operand(ktile, 16 * ks, i, lane);
                bv[i] = load_tr_operand(vtile, 16 * ks, i, lane);
            }
#pragma unroll
            for (int mi = 0; mi < 2; ++mi) {
                u32x4 au = as_u32x4(a[mi]);
#pragma unroll
                for (int w = 0; w < 4; ++w) zacc[mi] = add_bf16x2(au[w], zacc[mi]);
#pragma unroll
                for (int ni = 0; ni < 2; ++ni) acc[mi][ni] = mfma32(a[mi], bv[ni], acc[mi][ni]);
            }
            if (VSUM && qi == 0) {  // wave-uniform
#pragma unroll
                for (int ni = 0; ni < 2; ++ni) {
                    u32x4 bu = as_u32x4(bv[ni]);
#pragma unroll
                    for (int w = 0; w < 4; ++w) vacc[ni] = add_bf16x2(bu[w], vacc[ni]);
                }
            }
        }
        buf ^= 1;
    }

    // St[c2][c1] (c2: channel of V_j, c1: channel of K_i), then z_i[c1]: straight from the registers
    // (16 KB per wavefront, once per chunk).
    float *out = ws + ((size_t)part * BH * 4 + (size_t)bh * 4 + wave) * kStateFloats;
    const int g = lane >> 5, li = lane & 31;
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int c2 = 32 * ni + li, c1 = 32 * mi + 8 * q4 + 4 * g;
                f32x4 val = {acc[mi][ni][4 * q4], acc[mi][ni][4 * q4 + 1], acc[mi][ni][4 * q4 + 2],
                             acc[mi][ni][4 * q4 + 3]};
                *(f32x4 *)(out + c2 * kHeadDim + c1) = val;
            }
#pragma unroll
    for (int mi = 0; mi < 2; ++mi) {
        float lo, hi;
        pair_values(zacc[mi], &lo, &hi);  // the two halves of the tokens
        if (g == 0) out[kHeadDim * kHeadDim + 32 * mi + li] = lo + hi;
    }
    if (VSUM && qi == 0) {
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
            float lo, hi;
            pair_values(vacc[ni], &lo, &hi);
            if (g == 0) vsum[((size_t)part * BH + bh) * kHeadDimWide + kHeadDim * qj + 32 * ni + li] = lo + hi;
        }
    }
}

LinearPlan plan_linear_wide(int B, int heads, int N) {
    LinearPlan p = plan_linear(B, heads, N);
    p.combine = p.n_split > 1;  // the apply pass reads one state per quadrant
    // (the token chunks of the apply pass follow from B * heads as in plan_linear; every workgroup
    // loads its head's state once, 64 KB)
    return p;
}
size_t linear_wide_workspace_floats(int B, int heads, int N) {
    return linear_workspace_floats(plan_linear_wide(B, heads, N), B, 4 * heads);
}

jv_status linear_wide_state(const Problem &pr, float *ws, float *vsum, hipStream_t stream) {
    if (4ll * pr.B * pr.heads > 65535) return fail(JV_ERR_UNSUPPORTED, "head_dim 128: batch * heads above 16383");
    static LdsLimit lds_limit[2];
    jv_status st = ensure_lds_limit(lds_limit[0], (const void *)la_state_wide_bf16<false>, kStateWideLds);
    if (st == JV_OK) st = ensure_lds_limit(lds_limit[1], (const void *)la_state_wide_bf16<true>, kStateWideLds);
    if (st != JV_OK) return st;
    const LinearPlan plan = plan_linear_wide(pr.B, pr.heads, pr.N);
    const dim3 grid(plan.n_split, (unsigned)(pr.B * pr.heads));
    if (vsum)
        hipLaunchKernelGGL(la_state_wide_bf16<true>, grid, dim3(256), kStateWideLds, stream, pr.k, pr.v, ws, vsum,
                           pr.heads, pr.N, plan.chunk);
    else
        hipLaunchKernelGGL(la_state_wide_bf16<false>, grid, dim3(256), kStateWideLds, stream, pr.k, pr.v, ws,
                           (float *)nullptr, pr.heads, pr.N, plan.chunk);
    return launch_status("la_state_wide_bf16");
}

jv_status linear_wide_apply(const Problem &pr, float eps, float *ws, hipStream_t stream, int ksize, const DwcArg *cv) {
    jv_status st;
    const LinearPlan plan = plan_linear_wide(pr.B, pr.heads, pr.N);
    const long long BHv = 4ll * pr.B * pr.heads;  // quadrant states
    const float *states = ws;
    if (plan.combine) {
        float *dst = ws + (size_t)plan.n_split * BHv * kStateFloats;
        hipLaunchKernelGGL(la_combine, dim3((unsigned)BHv, ((kStateFloats + kHeadDim) / 4 + 255) / 256), dim3(256), 0,
                           stream, ws, dst, (float *)nullptr, plan.n_split, (int)BHv, 0);
        if ((st = launch_status("la_combine")) != JV_OK) return st;
        states = dst;
    }
    const int n_chunks = (pr.N + plan.apply_tokens - 1) / plan.apply_tokens;
    const long long n_wg = (long long)n_chunks * pr.B * pr.heads;
    if (n_wg >= (1ll << 31)) return fail(JV_ERR_UNSUPPORTED, "head_dim 128: too many token chunks");
    const DwcArg none = {nullptr, 0, pr.H, pr.W, pr.P};
    auto launch = [&](auto bf_tag, auto ks_tag) {
        constexpr bool O_BF16 = decltype(bf_tag)::value;
        constexpr int KS = decltype(ks_tag)::value;
        hipLaunchKernelGGL((la_apply_wide_bf16<O_BF16, KS>), dim3((unsigned)n_wg), dim3(256), 0, stream, pr.q, pr.o, states,
                           pr.heads, pr.N, plan.apply_tokens, n_chunks, eps, pr.v, KS ? *cv : none);
    };
    const int ks = cv ? ksize : 0;
    if (pr.o_bf16) {
        if (ks == 0) launch(std::true_type(), std::integral_constant<int, 0>());
        else if (ks == 3) launch(std::true_type(), std::integral_constant<int, 3>());
        else launch(std::true_type(), std::integral_constant<int, 5>());
    } else {
        if (ks == 0) launch(std::false_type(), std::integral_constant<int, 0>());
        else if (ks == 3) launch(std::false_type(), std::integral_constant<int, 3>());
        else launch(std::false_type(), std::integral_constant<int, 5>());
    }
    return launch_status("la_apply_wide_bf16");
}

jv_status linear_wide_bf16(const Problem &pr, float eps, float *ws, hipStream_t stream) {
    jv_status st = linear_wide_state(pr, ws, nullptr, stream);
    return st == JV_OK ? linear_wide_apply(pr, eps, ws, stream, 0, nullptr) : st;
}

}  // namespace jv
