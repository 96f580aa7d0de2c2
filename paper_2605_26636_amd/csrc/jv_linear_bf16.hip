// ReLU linear attention (Eq. 2 of the paper, phi = ReLU, key-sum normaliser) for bf16 tensors
// on the matrix cores, fp32 accumulation.
//
//   la_state_bf16   streams K and V once: every wavefront owns a 64 x 64 fp32 state in
//                   accumulators and adds relu(K_tile)^T V_tile per 64-token tile; the token
//                   axis is the contraction axis of both operands, so tiles go through LDS
//                   and come back with transposing reads.  z falls out of the same operands.
//   la_combine      sums the partial states when there are many chunks.
//   la_apply_bf16   sums the (few) partials, splits S and z into bf16 high and low parts held
//                   in registers, and streams Q -> O:  O^T = S^T relu(Q)^T on the matrix
//                   cores, the denominator relu(q).z as one more row block, fp32 divide.
#include "jv_linear.h"
#include "jv_mfma.h"

namespace jv {

constexpr int kWaveLds = 64 * 68 * 4;  // per-wave LDS: K and V tiles (16 KB) or a padded state
constexpr int kStateLds = 4 * kWaveLds + 8 * kHeadDim * 4;

// grid (n_split, B*heads), 256 threads, kStateLds bytes of dynamic LDS.
__global__ void __launch_bounds__(256, 2)
la_state_bf16(TensorArg kt, TensorArg vt, float *__restrict__ ws, int heads, int N, int chunk) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 5;
    const int bh = blockIdx.y, b = bh / heads, h = bh % heads, part = blockIdx.x;
    const int BH = gridDim.y;
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
    float zacc[2] = {0.f, 0.f};

    u32x4 kreg[8], vreg[8];
    auto fetch = [&](int t0) {
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int n = t0 + r * 8 + lrow;
            u32x4 zero = {0u, 0u, 0u, 0u};
            kreg[r] = zero;
            vreg[r] = zero;
            if (n < n1) {
                kreg[r] = *(const u32x4 *)(kp + (long long)n * kt.sn + lchunk * 8);
                vreg[r] = *(const u32x4 *)(vp + (long long)n * vt.sn + lchunk * 8);
            }
        }
    };

    int t = n0 + wave * 64;
    if (t < n1) fetch(t);
    for (; t < n1; t += 256) {
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const unsigned off = tile_off_tr(r * 8 + lrow, lchunk);
            *(u32x4 *)(ktile + off) = relu_bf16x8(kreg[r]);
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
    for (int mi = 0; mi < 2; ++mi) zbuf[(wave * 2 + g) * kHeadDim + 32 * mi + (lane & 31)] = zacc[mi];
    __syncthreads();
    float *out = ws + ((size_t)part * BH + bh) * kStateFloats;
    for (int e = tid; e < kHeadDim * kHeadDim; e += 256) {
        const int at = (e >> 6) * 68 + (e & 63);
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) s += ((const float *)(smem + w * kWaveLds))[at];
        out[e] = s;
    }
    if (tid < kHeadDim) {
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < 8; ++w) s += zbuf[w * kHeadDim + tid];
        out[kHeadDim * kHeadDim + tid] = s;
    }
}

// grid (B*heads, ceil(kStateFloats / 1024)), 256 threads: dst[bh] = sum_p ws[p][bh], one
// 16-byte piece per thread, the loads of eight partials in flight at a time.
__global__ void __launch_bounds__(256)
la_combine(const float *__restrict__ ws, float *__restrict__ dst, int n_split) {
    const int bh = blockIdx.x, BH = gridDim.x;
    const int e4 = blockIdx.y * 256 + threadIdx.x;
    if (e4 >= kStateFloats / 4) return;
    const f32x4 *src = (const f32x4 *)ws + (size_t)bh * (kStateFloats / 4) + e4;
    const size_t stride4 = (size_t)BH * (kStateFloats / 4);
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
    ((f32x4 *)dst)[(size_t)bh * (kStateFloats / 4) + e4] = sum;
}

// grid (ceil(N / tokens_per_wg), B*heads), 256 threads.
// `states` holds n_part partial states per (batch, head), part_stride floats apart.
template <bool O_BF16>
__global__ void __launch_bounds__(256, 2)
la_apply_bf16(TensorArg qt, TensorArg ot, const float *__restrict__ states, int n_part,
              long long part_stride, int heads, int N, int tokens_per_wg, float eps) {
    // St[c2][c1] fp32 with the 8-float group index rotated by the row, then z; afterwards the
    // same bytes stage output tiles.  Then one 8 KB query tile per wave.
    __shared__ __align__(16) unsigned char smem[kStateFloats * 4 + 4 * 8192];
    float *St = (float *)smem;
    float *zs = St + kHeadDim * kHeadDim;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 5, li = lane & 31;
    const int bh = blockIdx.y, b = bh / heads, h = bh % heads;
    const __bf16 *qp = (const __bf16 *)qt.ptr + b * qt.sb + h * qt.sh;
    const int n0 = blockIdx.x * tokens_per_wg, n1 = min(N, n0 + tokens_per_wg);
    const int lrow = lane >> 3, lchunk = lane & 7;

    // Query tiles are fetched one step ahead; start the first fetch before the state prologue.
    u32x4 qreg[8];
    auto fetch = [&](int t0) {
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int n = t0 + r * 8 + lrow;
            u32x4 zero = {0u, 0u, 0u, 0u};
            qreg[r] = zero;
            if (n < n1) qreg[r] = *(const u32x4 *)(qp + (long long)n * qt.sn + lchunk * 8);
        }
    };
    int t = n0 + wave * 64;
    if (t < n1) fetch(t);

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

    unsigned char *qtile = smem + kStateFloats * 4 + wave * 8192;
    unsigned char *otile = smem + wave * 4096;
    for (; t < n1; t += 256) {
#pragma unroll
        for (int r = 0; r < 8; ++r)
            *(u32x4 *)(qtile + tile_off_row(r * 8 + lrow, lchunk)) = relu_bf16x8(qreg[r]);
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
            if (O_BF16) {
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
                    if (on < n1) *(u32x4 *)(op + (long long)on * ot.sn + lchunk * 8) = val;
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

jv_status linear_bf16(const Problem &pr, const LinearPlan &plan, float eps, float *ws,
                      hipStream_t stream) {
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)la_state_bf16,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kStateLds);
        if (e != hipSuccess) return fail(JV_ERR_HIP, "hipFuncSetAttribute: %s", hipGetErrorString(e));
        attr_set = true;
    }
    const int BH = pr.B * pr.heads;
    jv_status st;
    hipLaunchKernelGGL(la_state_bf16, dim3(plan.n_split, BH), dim3(256), kStateLds, stream, pr.k,
                       pr.v, ws, pr.heads, pr.N, plan.chunk);
    if ((st = launch_status("la_state_bf16")) != JV_OK) return st;
    const float *states = ws;
    int n_part = plan.n_split;
    long long part_stride = (long long)BH * kStateFloats;
    if (plan.combine) {
        float *dst = ws + (size_t)plan.n_split * BH * kStateFloats;
        hipLaunchKernelGGL(la_combine, dim3(BH, (kStateFloats / 4 + 255) / 256), dim3(256), 0, stream, ws, dst,
                           plan.n_split);
        if ((st = launch_status("la_combine")) != JV_OK) return st;
        states = dst;
        n_part = 1;
    }
    dim3 grid((pr.N + plan.apply_tokens - 1) / plan.apply_tokens, BH);
    if (pr.o_bf16)
        hipLaunchKernelGGL(la_apply_bf16<true>, grid, dim3(256), 0, stream, pr.q, pr.o, states,
                           n_part, part_stride, pr.heads, pr.N, plan.apply_tokens, eps);
    else
        hipLaunchKernelGGL(la_apply_bf16<false>, grid, dim3(256), 0, stream, pr.q, pr.o, states,
                           n_part, part_stride, pr.heads, pr.N, plan.apply_tokens, eps);
    return launch_status("la_apply_bf16");
}

}  // namespace jv
