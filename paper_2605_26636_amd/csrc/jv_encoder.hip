// Encoder pieces around the token mixers (the pre-LN transformer block the paper's hybrid
// encoder inherits from the pretrained ViT): LayerNorm, the bf16 matrix-core GEMM with fused
// bias / GELU / residual epilogues, and the host loop that runs the blocks.
#include <math.h>
#include <new>

#include "jv_common.h"
#include "jv_linear.h"
#include "jv_mfma.h"

namespace jv {

// ---------------------------------------------------------------------------------------
// LayerNorm: one wavefront per row, the row held in registers (16-byte pieces, lane-strided),
// mean and variance in two register passes, fp32 statistics.
// grid (8 * ceil(ceil(rows / 4) / 8)), 256 threads.  NV = 16-byte pieces per lane (cols <= 256 * NV).
// ---------------------------------------------------------------------------------------
template <bool IN_BF16, bool OUT_BF16, int NV>
__global__ void __launch_bounds__(256)
layernorm_kernel(const void *__restrict__ xin, const float *__restrict__ gamma,
                 const float *__restrict__ beta, void *__restrict__ yout, long long rows, int cols,
                 float eps) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    // workgroups in contiguous ranges per XCD (workgroup w of the launch takes range w % 8): an
    // XCD then normalises the rows whose tiles it wrote in the product before and reads in the
    // product after (their tiles are dealt the same way), which keeps part of them in its L2
    const long long n_wg = (rows + 3) / 4, per_xcd = (n_wg + 7) / 8;
    const long long wg = (long long)(blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    const long long row = wg * 4 + wave;
    if (wg >= n_wg || row >= rows) return;
    // piece p of a lane covers columns 4 * (lane + 64 p) .. + 3
    f32x4 v[NV];
    float sum = 0.f;
#pragma unroll
    for (int p = 0; p < NV; ++p) {
        const int c = 4 * (lane + 64 * p);
        f32x4 x = {0.f, 0.f, 0.f, 0.f};
        if (c < cols) {
            if (IN_BF16) {
                const u32x2 raw = *(const u32x2 *)((const __bf16 *)xin + row * cols + c);
                x[0] = bf16_lo(raw[0]); x[1] = bf16_hi(raw[0]);
                x[2] = bf16_lo(raw[1]); x[3] = bf16_hi(raw[1]);
            } else {
                x = *(const f32x4 *)((const float *)xin + row * cols + c);
            }
        }
        v[p] = x;
        sum += (x[0] + x[1]) + (x[2] + x[3]);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, 64);
    const float mean = sum / (float)cols;
    float sq = 0.f;
#pragma unroll
    for (int p = 0; p < NV; ++p) {
        const int c = 4 * (lane + 64 * p);
        if (c < cols) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float dlt = v[p][e] - mean;
                sq = fmaf(dlt, dlt, sq);
            }
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) sq += __shfl_xor(sq, off, 64);
    const float inv = 1.0f / sqrtf(sq / (float)cols + eps);
#pragma unroll
    for (int p = 0; p < NV; ++p) {
        const int c = 4 * (lane + 64 * p);
        if (c < cols) {
            const f32x4 gm = *(const f32x4 *)(gamma + c), bt = *(const f32x4 *)(beta + c);
            f32x4 y;
#pragma unroll
            for (int e = 0; e < 4; ++e) y[e] = (v[p][e] - mean) * inv * gm[e] + bt[e];
            if (OUT_BF16) {
                u32x2 pk = {pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3])};
                *(u32x2 *)((__bf16 *)yout + row * cols + c) = pk;
            } else {
                *(f32x4 *)((float *)yout + row * cols + c) = y;
            }
        }
    }
}

template <bool IN_BF16, bool OUT_BF16>
static void launch_layernorm(const void *x, const float *gamma, const float *beta, void *y,
                             long long rows, int cols, float eps, hipStream_t stream) {
    dim3 grid((unsigned)(8 * (((rows + 3) / 4 + 7) / 8)));
    const int nv = (cols + 255) / 256;
    if (nv <= 1)
        hipLaunchKernelGGL((layernorm_kernel<IN_BF16, OUT_BF16, 1>), grid, dim3(256), 0, stream, x, gamma, beta, y, rows, cols, eps);
    else if (nv <= 2)
        hipLaunchKernelGGL((layernorm_kernel<IN_BF16, OUT_BF16, 2>), grid, dim3(256), 0, stream, x, gamma, beta, y, rows, cols, eps);
    else if (nv <= 4)
        hipLaunchKernelGGL((layernorm_kernel<IN_BF16, OUT_BF16, 4>), grid, dim3(256), 0, stream, x, gamma, beta, y, rows, cols, eps);
    else if (nv <= 8)
        hipLaunchKernelGGL((layernorm_kernel<IN_BF16, OUT_BF16, 8>), grid, dim3(256), 0, stream, x, gamma, beta, y, rows, cols, eps);
    else
        hipLaunchKernelGGL((layernorm_kernel<IN_BF16, OUT_BF16, 32>), grid, dim3(256), 0, stream, x, gamma, beta, y, rows, cols, eps);
}

static jv_status layernorm_forward(const void *x, const float *gamma, const float *beta, void *y,
                                   long long rows, int cols, float eps, bool in_bf16,
                                   bool out_bf16, hipStream_t stream) {
    if (in_bf16 && out_bf16) launch_layernorm<true, true>(x, gamma, beta, y, rows, cols, eps, stream);
    else if (in_bf16) launch_layernorm<true, false>(x, gamma, beta, y, rows, cols, eps, stream);
    else if (out_bf16) launch_layernorm<false, true>(x, gamma, beta, y, rows, cols, eps, stream);
    else launch_layernorm<false, false>(x, gamma, beta, y, rows, cols, eps, stream);
    return launch_status("layernorm_kernel");
}

// ---------------------------------------------------------------------------------------
// GEMM  y = epilogue(a w^T + bias):  a [M, K], w [N, K], both bf16 with K contiguous, so both
// matrix-instruction operands are 16-byte row pieces.  One workgroup (8 wavefronts, two per
// SIMD, half the register file each) owns a 256 x 256 tile of y; a wavefront owns 128 tokens x
// 64 features of it (4 x 2 blocks of 32 x 32, 128 accumulator registers).  Two wavefronts per
// SIMD: while one waits (barrier, operands), the other keeps the matrix pipeline busy.
// K is walked in blocks of 64, i.e. whole 128-byte lines of every row: the 256 x 64 parts of a
// and of w go from global memory straight into LDS (no register staging) through a ring of
// five 32 KB slots filled in the order a0 w0 a1 w1 a2 ...  While block p is multiplied, the
// parts of block p+1 are in flight or landed and the a part of block p+2 is being issued, a
// load or two per step, into the slot the block before p has left; the w part of p+2 follows
// into block p's a slot as soon as its last operands have been read.  The wait before a block
// is therefore a counted one (the youngest part may still be outstanding), written by hand
// next to the barrier.
// A block is four steps of 16 in K; the LDS reads of a step are issued among the matrix
// instructions of the step before it, and the workgroup barrier sits before the last step:
// when a wavefront leaves it, the operands of that step are already in registers, so the
// matrix pipeline restarts at once, and the reads of the next block's first step overlap it.
// Rows are 128 bytes in LDS; the 16-byte chunk index is rotated by the row pair, which
// spreads the sixteen rows that one pass of a row-per-lane read touches over all 64 banks.
// The product is formed transposed (features x tokens): a lane then holds 4 consecutive output
// features of one token (bias pieces are 16-byte loads); the epilogue regroups the blocks into
// token rows through LDS before it touches global memory.
// Tiles are assigned so that the workgroups an XCD receives (every eighth) walk a contiguous
// range of tiles, feature-tile fastest: they share the a row-tile and keep w in that L2.
// grid (8 * ceil(tiles / 8)), 512 threads, kGemmLds bytes of dynamic LDS.
// ---------------------------------------------------------------------------------------
constexpr int kBM = 256, kBN = 256, kBK = 64;
constexpr int kGemmPart = kBM * kBK * 2;               // one operand part: 32 KB
constexpr int kGemmSlots = 5;
constexpr int kGemmLds = kGemmSlots * kGemmPart;       // 160 KB

typedef __attribute__((address_space(1))) const void global_cvoid;
typedef __attribute__((address_space(3))) void lds_void;

// gelu(x) = x Phi(x), Phi the standard normal distribution function.  The GEMM epilogue reads
// Phi from a table in LDS (kPhiSteps intervals on [-6, 6], linear interpolation: absolute error
// below 5e-6; outside the range Phi is 0 or 1 to 1e-9) that every workgroup builds for itself
// from  Phi(x) = 1 - erfc(x / sqrt 2) / 2,  erfc(z) = (a1 t + ... + a5 t^5) exp(-z^2),
// t = 1 / (1 + p z), z >= 0  (Abramowitz-Stegun 7.1.26, absolute error 1.5e-7).
constexpr int kPhiSteps = 1024;
constexpr float kPhiLo = -6.0f, kPhiStep = 12.0f / kPhiSteps;
__device__ inline float normal_cdf(float x) {
    const float z = fabsf(x) * 0.70710678118654752f;
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, z, 1.0f));
    const float poly = t * fmaf(t, fmaf(t, fmaf(t, fmaf(t, 1.061405429f, -1.453152027f), 1.421413741f),
                                        -0.284496736f), 0.254829592f);
    const float half_erfc = 0.5f * poly * __builtin_amdgcn_exp2f(-1.4426950408889634f * z * z);
    return x < 0.f ? half_erfc : 1.0f - half_erfc;
}
// table[2 i] = Phi(x_i), table[2 i + 1] = Phi(x_i+1) - Phi(x_i), x_i = kPhiLo + i kPhiStep.
__device__ inline float gelu_from_table(float x, const float *table) {
    const float t = __builtin_amdgcn_fmed3f(fmaf(x, 1.0f / kPhiStep, -kPhiLo / kPhiStep), 0.0f,
                                            (float)kPhiSteps - 0.004f);
    const unsigned i = (unsigned)t;
    const float2 pd = *(const float2 *)(table + 2 * i);
    return x * fmaf(t - (float)i, pd.y, pd.x);
}

// Byte offset of 16-byte chunk `chunk` (0..7) of row `row` in a [rows][64] bf16 LDS part.
__device__ inline unsigned gemm_part_off(int row, int chunk) {
    return (unsigned)(row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4));
}

// Wait until at most `pending` of this wavefront's vector-memory loads are outstanding, then
// the workgroup barrier.  "memory" keeps the compiler from moving LDS traffic across it.
__device__ inline void wait_loads_and_barrier(int pending) {
    // the count is an immediate: take the largest supported value not above `pending`
    if (pending >= 12) asm volatile("s_waitcnt vmcnt(12) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    else if (pending >= 8) asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    else if (pending >= 4) asm volatile("s_waitcnt vmcnt(4) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// LayerNorm folded into the matrix product that consumes it (the block's two LayerNorms sit
// between a residual GEMM and a GEMM):
//   sum_k w[n][k] LN(x)[k] = rstd (sum_k (w gamma)[n][k] x[k] - mean c1[n]) + c2[n],
//   c1[n] = sum_k (w gamma)[n][k],  c2[n] = sum_k w[n][k] beta[k] + bias[n].
// kLnProduce (residual epilogue): besides y it writes the stream rounded to bf16 (the A operand
// of the next product; omitted when y is bf16 itself) and, per row and group of 64 features, the
// group's mean and its sum of squared deviations.  kLnConsume (plain and GELU epilogues): A is
// that bf16 stream, w is (w gamma) rounded to bf16, `bias` is c2; every workgroup first merges
// the group statistics of its 256 rows into mean and 1/sigma (pairwise update of mean and
// squared deviations), and the epilogue applies the formula above.
enum { kLnNone = 0, kLnConsume = 1, kLnProduce = 2, kGemmExtras = 3 };  // kGemmExtras: w_rows / k_split below are read
struct GemmLn {
    const float *c1;        // consume: [N]
    const float *stats_in;  // consume: [groups][M][2] (mean, sum of squared deviations) of 64 features each
    float *stats_out;       // produce: [N / 64][M][2]
    void *xb_out;           // produce: [M][N] bf16 copy of y, or null
    int groups;             // consume: K / 64
    float eps;              // consume
    // One weight matrix per group of rows (the fused projection of a linear-attention block:
    // one matrix per image): rows m use w + (m / w_rows) * w_stride; w_rows = 0: one matrix.
    // w_rows is a multiple of the tile height, so a tile never straddles two matrices.
    int w_rows;
    long long w_stride;     // elements
    // K split over k_split workgroups per tile (0 or 1: none): workgroup (part, tile) multiplies
    // columns part * K / k_split .. of a and w and writes its tile of partial part, y_split
    // elements after the one before (plain epilogue, fp32 output; gemm_split_combine adds them up).
    int k_split;
    long long y_split;      // elements
};

// Sum over the 16 lanes of a DPP row (the lanes that hold one token row of the fp32 tile).
__device__ inline float row16_sum(float x) {
    auto dpp = [](float v, auto ctrl_tag) {
        constexpr int ctrl = decltype(ctrl_tag)::value;
        return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), ctrl, 0xf, 0xf, true));
    };
    x += dpp(x, std::integral_constant<int, 0xB1>());   // quad_perm [1, 0, 3, 2]
    x += dpp(x, std::integral_constant<int, 0x4E>());   // quad_perm [2, 3, 0, 1]
    x += dpp(x, std::integral_constant<int, 0x141>());  // row_half_mirror
    x += dpp(x, std::integral_constant<int, 0x140>());  // row_mirror
    return x;
}

template <int EPI, bool OUT_BF16, int LN>
__global__ void __launch_bounds__(512, 1)
gemm_bf16_kernel(const __bf16 *__restrict__ A, const __bf16 *__restrict__ W,
                 const float *__restrict__ bias, const void *residual, void *Y, int M, int N,
                 int K, int lda, int tiles_n, int n_tiles, GemmLn ln) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 5, li = lane & 31;
    // (the per-image weights and the K split exist only in the kGemmExtras instances: the
    // other instances pay nothing for them)
    const int k_split = (LN == kGemmExtras && ln.k_split > 1) ? ln.k_split : 1;
    const int per_xcd = (n_tiles * k_split + 7) / 8;
    int tile = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (tile >= n_tiles * k_split) return;  // whole workgroup
    int k_part = 0, k_len = K;          // which part of K, and the columns this workgroup multiplies
    if (LN == kGemmExtras) {
        k_part = tile / n_tiles;
        tile -= k_part * n_tiles;
        k_len = K / k_split;
        Y = (void *)((char *)Y + (size_t)k_part * (size_t)ln.y_split * (OUT_BF16 ? 2 : 4));
    }
    const int m0 = (tile / tiles_n) * kBM, n0 = (tile % tiles_n) * kBN;
    const int wm = wave >> 2, wn = wave & 3;  // 128-token half, 64-feature quarter
    constexpr int kPartLoads = 4;             // load instructions per part and wavefront

    // Global -> LDS: a wavefront moves rows 32*wave .. +31 of a part, 8 rows (1 KB) per
    // instruction; lane = 8 * (row in group) + LDS chunk slot, and it fetches the global chunk
    // that belongs in that slot under the row rotation.  Four loads per wavefront and part.
    const int lrow = lane >> 3;
    // The tile's first rows are 64-bit bases (the same in every lane); the offsets inside the
    // tile, 255 rows at most, fit 32 bits (the launcher bounds lda and K).
    const char *a_tile = (const char *)(A + (size_t)m0 * lda + (size_t)k_part * k_len);
    const char *w_tile = (const char *)(W + (size_t)n0 * K + (size_t)k_part * k_len +
                                        ((LN == kGemmExtras && ln.w_rows) ? (size_t)(m0 / ln.w_rows) * (size_t)ln.w_stride : (size_t)0));
    unsigned a_off[kPartLoads], w_off[kPartLoads];  // byte offsets of this lane's 16 bytes, k = 0
#pragma unroll
    for (int j = 0; j < kPartLoads; ++j) {
        const int r = wave * 32 + j * 8 + lrow;
        const int gchunk = (lane & 7) ^ ((r >> 1) & 7);
        const int ar = min(r, M - 1 - m0), wr = min(r, N - 1 - n0);  // edge tiles re-read the last row
        a_off[j] = 2u * ((unsigned)ar * (unsigned)lda + gchunk * 8);  // rows of a are lda elements apart
        w_off[j] = 2u * ((unsigned)wr * (unsigned)K + gchunk * 8);
    }
    const int n_b = k_len / kBK, n_parts = 2 * n_b;
    // part = 2 * block + (0: a, 1: w); it lives in slot part % 5.  Loads j0 .. j1-1 of a part:
    auto issue_loads = [&](int part, int slot, int j0, int j1) __attribute__((always_inline)) {
        unsigned char *base = smem + slot * kGemmPart + wave * 32 * 128;
        const unsigned kbytes = 2u * (unsigned)(part >> 1) * kBK;
        if (part & 1) {
#pragma unroll
            for (int j = j0; j < j1; ++j)
                __builtin_amdgcn_global_load_lds((global_cvoid *)(w_tile + (w_off[j] + kbytes)),
                                                 (lds_void *)(base + j * 1024), 16, 0, 0);
        } else {
#pragma unroll
            for (int j = j0; j < j1; ++j)
                __builtin_amdgcn_global_load_lds((global_cvoid *)(a_tile + (a_off[j] + kbytes)),
                                                 (lds_void *)(base + j * 1024), 16, 0, 0);
        }
    };
    auto issue_part = [&](int part, int slot) __attribute__((always_inline)) { issue_loads(part, slot, 0, kPartLoads); };

    f32x16 acc[2][4];  // [feature block][token block]
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[nt][mt][v] = 0.f;

    // Operand registers, two sets used in turn by the steps.
    bf16x8 aop[2][4], wop[2][2];
    auto load_ops = [&](int a_slot, int w_slot, int step, int set) {
        const unsigned char *at = smem + a_slot * kGemmPart, *wt = smem + w_slot * kGemmPart;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            aop[set][i] = as_bf16x8(*(const u32x4 *)(at + gemm_part_off(wm * 128 + i * 32 + li, 2 * step + g)));
#pragma unroll
        for (int i = 0; i < 2; ++i)
            wop[set][i] = as_bf16x8(*(const u32x4 *)(wt + gemm_part_off(wn * 64 + i * 32 + li, 2 * step + g)));
    };
    auto products = [&](int set) {
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) acc[nt][mt] = mfma32(wop[set][nt], aop[set][mt], acc[nt][mt]);
    };
    auto next_slot = [](int s, int by) { s += by; return s >= kGemmSlots ? s - kGemmSlots : s; };
    // One step (8 matrix instructions) interleaved with the 6 LDS reads of the next one and with
    // `n_loads` global->LDS loads (written before the reads in the source: the compiler keeps
    // LDS reads and loads that write LDS in program order).
    auto step_with_reads = [&](int set, int n_loads) __attribute__((always_inline)) {
        products(set);
        if (n_loads >= 2) {
            __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);
        } else {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (n_loads == 1) __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);
        }
#pragma unroll
        for (int i = 0; i < 6; ++i) {  // the reads early, so that they have landed by the end
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    };
    // One block of 64 in K.  a_slot/w_slot hold it; the set-0 operands of its first step are in
    // registers.  The refill loads are spread over the block instead of issued in one burst:
    // all eight wavefronts pass the barrier together, and 64 loads issued at once queue in the
    // address path while the matrix instructions behind them in program order wait (the loop
    // ran 9 % faster with them spread).  `refill`: parts 2p+4 and 2p+5 exist.  Part 2p+4 goes
    // into the slot of part 2p-1 (free since the previous barrier) during the first three
    // steps, part 2p+5 into this block's a slot after the barrier; at the barrier block p+1
    // (parts 2p+2, 2p+3) must have landed and only part 2p+4 may be pending.  `next`: there is
    // a block p+1.
    auto block = [&](int p, int a_slot, int w_slot, bool refill, bool next) __attribute__((always_inline)) {
        const int slot4 = next_slot(w_slot, 3);
        if (refill) issue_loads(2 * p + 4, slot4, 0, 2);
        load_ops(a_slot, w_slot, 1, 1);
        step_with_reads(0, refill ? 2 : 0);
        if (refill) issue_loads(2 * p + 4, slot4, 2, 3);
        load_ops(a_slot, w_slot, 2, 0);
        step_with_reads(1, refill ? 1 : 0);
        if (refill) issue_loads(2 * p + 4, slot4, 3, 4);
        load_ops(a_slot, w_slot, 3, 1);
        step_with_reads(0, refill ? 1 : 0);
        // every wavefront is done reading this block once it arrives here
        if (next) wait_loads_and_barrier(refill ? kPartLoads : 0);
        if (next) load_ops(next_slot(a_slot, 2), next_slot(w_slot, 2), 0, 0);
        if (refill) issue_part(2 * p + 5, a_slot);
        products(1);
        if (refill) {
            // after the barrier: the six LDS reads of the next block's first step, then the
            // four loads of part 2p+5 among the last matrix instructions
#pragma unroll
            for (int i = 0; i < 6; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x010, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x010, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        }
    };
    static_assert(kPartLoads == 4, "the block spreads four loads per part over its steps");
    // Folded LayerNorm: thread t < 256 turns the group statistics of row m0 + t into the row's mean
    // and 1/sigma.  The groups all hold 64 features, so the mean is the plain average of the group
    // means and the squared deviations add up as sum_g (m2_g + 64 (mean_g - mean)^2): two short
    // passes over values in registers, no chain of dependent updates.  The statistics are stored
    // group-major ([group][row]), so that the 64 rows of a wavefront are one contiguous 512-byte
    // piece per group; they are fetched before the first operand parts are issued and combined
    // while those are in flight, so that the epilogue finds the two values in registers.
    constexpr int kStatChunk = 16;  // groups held in registers at a time (width 1024: all of them)
    float2 stat_part[kStatChunk];
    const float2 *gs = (const float2 *)ln.stats_in + min(m0 + tid, M - 1);
    auto fetch_stats = [&](int g0) {
#pragma unroll
        for (int i = 0; i < kStatChunk; ++i) stat_part[i] = gs[(size_t)min(g0 + i, ln.groups - 1) * M];
    };
    if (LN == kLnConsume && tid < kBM) fetch_stats(0);
    const int n_first = min(n_parts, kGemmSlots - 1);  // parts 0..3 go out at once, part 4 with block 0
    for (int part = 0; part < n_first; ++part) issue_part(part, part);
    float row_mean = 0.f, row_rstd = 1.f;
    if (LN == kLnConsume && tid < kBM) {
        float sum = 0.f;
        for (int g0 = 0; g0 < ln.groups; g0 += kStatChunk) {
            if (g0 > 0) fetch_stats(g0);  // more than sixteen groups (width above 1024)
#pragma unroll
            for (int i = 0; i < kStatChunk; ++i) sum += g0 + i < ln.groups ? stat_part[i].x : 0.f;
        }
        const float mean = sum / (float)ln.groups;
        float m2 = 0.f;
        for (int g0 = 0; g0 < ln.groups; g0 += kStatChunk) {
            if (ln.groups > kStatChunk) fetch_stats(g0);
#pragma unroll
            for (int i = 0; i < kStatChunk; ++i) {
                const float d = stat_part[i].x - mean;
                m2 += g0 + i < ln.groups ? fmaf(64.f * d, d, stat_part[i].y) : 0.f;
            }
        }
        row_mean = mean;
        row_rstd = 1.0f / sqrtf(m2 / (64.f * (float)ln.groups) + ln.eps);
    }
    wait_loads_and_barrier(kPartLoads * (n_first - 2));  // block 0 has landed
    load_ops(0, 1, 0, 0);
    int p = 0, a_slot = 0, w_slot = 1;
    for (; 2 * p + 5 < n_parts; ++p) {  // steady state
        block(p, a_slot, w_slot, true, true);
        a_slot = next_slot(a_slot, 2);
        w_slot = next_slot(w_slot, 2);
    }
    for (; p < n_b; ++p) {  // the last two blocks: everything has been issued
        block(p, a_slot, w_slot, false, p + 1 < n_b);
        a_slot = next_slot(a_slot, 2);
        w_slot = next_slot(w_slot, 2);
    }

    // Epilogue: accumulator register v of block (nt, mt) is output feature
    // n0 + 64 wn + 32 nt + 8 (v/4) + 4 g + v%4 of token m0 + 128 wm + 32 mt + li: a lane holds
    // 4 consecutive features of one token.  Stored from there, an instruction would touch 32
    // token rows with 16 or 32 bytes each, and every 128-byte line of y would be written by 4 to
    // 8 different instructions.  Instead each wavefront turns its 32 x 64 blocks into token rows
    // in 8 KB of LDS of its own and stores whole rows (128 or 256 contiguous bytes per token);
    // the residual is read in the same row layout.  The LDS comes from the operand ring: the
    // last block occupies two of the five slots, and every wavefront has passed the barrier
    // after which nobody reads the other three (a_slot points at the first of them here).
    unsigned char *stage = smem + next_slot(a_slot, 1 + (wave >> 2)) * kGemmPart + (wave & 3) * 8192;
    // GELU reads the normal distribution function from a table in the third free slot, built
    // here by all threads (two or three entries each; see gelu_from_table).
    float *phi_table = (float *)(smem + a_slot * kGemmPart);
    // Folded LayerNorm: the rows' mean and 1/sigma (merged under the first operand loads, above)
    // go to the lanes that hold the rows' tokens through LDS.
    float2 *row_stats = (float2 *)(smem + a_slot * kGemmPart + 16384);  // behind the table, [256]
    if (LN == kLnConsume && tid < kBM) row_stats[tid] = float2{row_mean, row_rstd};
    if (EPI == JV_EPI_GELU) {
        for (int i = tid; i <= kPhiSteps; i += 512) {
            const float p0 = normal_cdf(kPhiLo + (float)i * kPhiStep);
            phi_table[2 * i] = p0;
            phi_table[2 * i + 1] = normal_cdf(kPhiLo + (float)(i + 1) * kPhiStep) - p0;
        }
    }
    if (EPI == JV_EPI_GELU || LN == kLnConsume) asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    f32x4 c1_reg[2][4];
    if (LN == kLnConsume) {
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int col = n0 + wn * 64 + nt * 32 + 8 * q4 + 4 * g;
                f32x4 zero = {0.f, 0.f, 0.f, 0.f};
                c1_reg[nt][q4] = col < N ? *(const f32x4 *)(ln.c1 + col) : zero;
            }
    }
    f32x4 bias_reg[2][4];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            const int col = n0 + wn * 64 + nt * 32 + 8 * q4 + 4 * g;
            f32x4 zero = {0.f, 0.f, 0.f, 0.f};
            bias_reg[nt][q4] = (bias && col < N) ? *(const f32x4 *)(bias + col) : zero;
        }
    // The residual has y's element type and is added in the row layout; with bf16 tensors the
    // blocks are staged in fp32 all the same, so that the sum is rounded once.
    constexpr bool kResidual = EPI == JV_EPI_RESIDUAL;
    constexpr bool kStageF32 = !OUT_BF16 || kResidual;
    // Row layout of the fp32 tile: 16 lanes per token row (256 bytes), 4 rows per instruction.
    const int frow = lane >> 4, fchunk = lane & 15;
    const int fcol = n0 + wn * 64 + 4 * fchunk;
    // The residual rows of token block mt+1 are fetched before block mt is stored (different
    // rows, so this is safe although the residual may be y itself): one round trip is exposed
    // instead of four.
    f32x4 res_reg[2][8];
    u32x2 res16_reg[2][8];
    auto load_residual = [&](int mt, int set) {
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int row = m0 + wm * 128 + mt * 32 + 4 * r + frow;
            const bool inside = row < M && fcol < N;
            if (OUT_BF16) {
                u32x2 zero = {0u, 0u};
                res16_reg[set][r] = inside ? *(const u32x2 *)((const __bf16 *)residual + (size_t)row * N + fcol) : zero;
            } else {
                f32x4 zero = {0.f, 0.f, 0.f, 0.f};
                res_reg[set][r] = inside ? *(const f32x4 *)((const float *)residual + (size_t)row * N + fcol) : zero;
            }
        }
    };
    if (kResidual) load_residual(0, 0);
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) {
        if (kResidual && mt + 1 < 4) load_residual(mt + 1, (mt + 1) & 1);
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                f32x4 val = {acc[nt][mt][4 * q4], acc[nt][mt][4 * q4 + 1], acc[nt][mt][4 * q4 + 2],
                             acc[nt][mt][4 * q4 + 3]};
                if (LN == kLnConsume) {  // rstd (acc - mean c1) + c2 for this lane's token
                    const float2 st = row_stats[wm * 128 + mt * 32 + li];
                    const float rm = -st.x * st.y;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        val[e] = fmaf(val[e], st.y, fmaf(rm, c1_reg[nt][q4][e], bias_reg[nt][q4][e]));
                } else {
                    val += bias_reg[nt][q4];
                }
                if (EPI == JV_EPI_GELU) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) val[e] = gelu_from_table(val[e], phi_table);
                }
                if (EPI == JV_EPI_SILU) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) val[e] = val[e] * __builtin_amdgcn_rcpf(1.0f + __expf(-val[e]));
                }
                if (kStageF32) {
                    *(f32x4 *)(stage + li * 256 + (((8 * nt + 2 * q4 + g) ^ (li & 15)) << 4)) = val;
                } else {
                    u32x2 pk = {pack_bf16x2(val[0], val[1]), pack_bf16x2(val[2], val[3])};
                    *(u32x2 *)(stage + tile_off_row(li, 4 * nt + q4) + 8 * g) = pk;
                }
            }
        if (!kStageF32) {  // 8 lanes per token row (128 bytes), 8 rows per instruction
            const int col = n0 + wn * 64 + 8 * (lane & 7);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int orow = 8 * r + lrow, row = m0 + wm * 128 + mt * 32 + orow;
                const u32x4 out = *(const u32x4 *)(stage + tile_off_row(orow, lane & 7));
                // N % 8 == 0: the eight features of a piece are in or out together
                if (row < M && col < N) *(u32x4 *)((__bf16 *)Y + (size_t)row * N + col) = out;
            }
        } else {
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                const int orow = 4 * r + frow, row = m0 + wm * 128 + mt * 32 + orow;
                f32x4 out = *(const f32x4 *)(stage + orow * 256 + ((fchunk ^ (orow & 15)) << 4));
                if (OUT_BF16) {  // bf16 tensors with a residual: 16 lanes x 8 bytes = one 128-byte row
                    const u32x2 rr = res16_reg[mt & 1][r];
                    out[0] += bf16_lo(rr[0]); out[1] += bf16_hi(rr[0]);
                    out[2] += bf16_lo(rr[1]); out[3] += bf16_hi(rr[1]);
                    u32x2 pk = {pack_bf16x2(out[0], out[1]), pack_bf16x2(out[2], out[3])};
                    if (row < M && fcol < N) *(u32x2 *)((__bf16 *)Y + (size_t)row * N + fcol) = pk;
                    if (LN == kLnProduce) {  // the statistics describe the stream as stored
                        out[0] = bf16_lo(pk[0]); out[1] = bf16_hi(pk[0]);
                        out[2] = bf16_lo(pk[1]); out[3] = bf16_hi(pk[1]);
                    }
                } else {
                    if (kResidual) out += res_reg[mt & 1][r];
                    if (row < M && fcol < N) *(f32x4 *)((float *)Y + (size_t)row * N + fcol) = out;
                    if (LN == kLnProduce && ln.xb_out) {
                        u32x2 pk = {pack_bf16x2(out[0], out[1]), pack_bf16x2(out[2], out[3])};
                        if (row < M && fcol < N) *(u32x2 *)((__bf16 *)ln.xb_out + (size_t)row * N + fcol) = pk;
                        // (the next product multiplies these rounded values)
                        out[0] = bf16_lo(pk[0]); out[1] = bf16_hi(pk[0]);
                        out[2] = bf16_lo(pk[1]); out[3] = bf16_hi(pk[1]);
                    }
                }
                if (LN == kLnProduce) {
                    // mean and squared deviations of this wavefront's 64 features of the row
                    // (16 lanes x 4); N % 64 == 0 here, so a group is inside y or outside whole
                    const float mean = row16_sum((out[0] + out[1]) + (out[2] + out[3])) * (1.0f / 64.0f);
                    const float d0 = out[0] - mean, d1 = out[1] - mean, d2 = out[2] - mean, d3 = out[3] - mean;
                    const float m2 = row16_sum(fmaf(d0, d0, d1 * d1) + fmaf(d2, d2, d3 * d3));
                    if (fchunk == 0 && row < M && fcol < N)
                        *(float2 *)(ln.stats_out + ((size_t)((n0 + wn * 64) >> 6) * M + row) * 2) = float2{mean, m2};
                }
            }
        }
    }
}

template <int EPI, bool OUT_BF16, int LN = kLnNone>
static jv_status launch_gemm(const void *a, const void *w, const float *bias, const void *residual,
                             void *y, long long M, int N, int K, int lda, hipStream_t stream,
                             const GemmLn &ln = GemmLn{}) {
    static LdsLimit lds_limit;
    jv_status st = ensure_lds_limit(lds_limit, (const void *)gemm_bf16_kernel<EPI, OUT_BF16, LN>, kGemmLds);
    if (st != JV_OK) return st;
    const int tiles_m = (int)((M + kBM - 1) / kBM), tiles_n = (N + kBN - 1) / kBN;
    const int n_tiles = tiles_m * tiles_n;
    dim3 grid(8 * ((n_tiles * ((LN == kGemmExtras && ln.k_split > 1) ? ln.k_split : 1) + 7) / 8));
    hipLaunchKernelGGL((gemm_bf16_kernel<EPI, OUT_BF16, LN>), grid, dim3(512), kGemmLds, stream,
                       (const __bf16 *)a, (const __bf16 *)w, bias, residual, y, (int)M, N, K, lda,
                       tiles_n, n_tiles, ln);
    return launch_status("gemm_bf16_kernel");
}

// Residual product with K split over several workgroups per tile, for launches that would leave
// most compute units without a tile (fc2 of a ViT-L block on 8 192 tokens: 128 tiles of
// 256 x 256 for 256 units, each with a K loop of 4096): k_split workgroups per tile multiply a
// part of K each and write fp32 partial tiles; gemm_split_combine then forms
//     y = sum of the partials + bias + residual
// in a fixed order (no atomics: the same bits on every run).
constexpr int kComputeUnits = 256;  // MI355X
// k_split for a residual product of M x N x K, or 1: as many parts as fill the chip, at most 4,
// each a multiple of the K block and at least 1024 long.
static int gemm_k_split(long long M, int N, int K) {
    const long long tiles = ((M + kBM - 1) / kBM) * ((N + kBN - 1) / kBN);
    int split = 1;
    while (split < 4 && tiles * split * 2 <= kComputeUnits && K % (2 * split * kBK) == 0 && K / (2 * split) >= 1024) split *= 2;
    return split;
}
// grid (ceil(M * N / 4 / 256)), 256 threads; N % 4 == 0; y may be the residual itself.
template <bool OUT_BF16>
__global__ void __launch_bounds__(256)
gemm_split_combine(const float *__restrict__ parts, long long part_stride, int n_parts,
                   const float *__restrict__ bias, const void *residual, void *y, long long total4, int N) {
    const long long i4 = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i4 >= total4) return;
    const int col = (int)((i4 * 4) % N);
    f32x4 sum = *(const f32x4 *)(parts + i4 * 4);
    for (int p = 1; p < n_parts; ++p) sum += *(const f32x4 *)(parts + (size_t)p * part_stride + i4 * 4);
    if (bias) sum += *(const f32x4 *)(bias + col);
    if (OUT_BF16) {
        const u32x2 rr = *(const u32x2 *)((const __bf16 *)residual + i4 * 4);
        sum[0] += bf16_lo(rr[0]); sum[1] += bf16_hi(rr[0]);
        sum[2] += bf16_lo(rr[1]); sum[3] += bf16_hi(rr[1]);
        u32x2 pk = {pack_bf16x2(sum[0], sum[1]), pack_bf16x2(sum[2], sum[3])};
        *(u32x2 *)((__bf16 *)y + i4 * 4) = pk;
    } else {
        sum += *(const f32x4 *)((const float *)residual + i4 * 4);
        *(f32x4 *)((float *)y + i4 * 4) = sum;
    }
}
// y = a w^T + bias + residual with K split k_split ways; parts: k_split * M * N floats of scratch.
static jv_status gemm_residual_split(const void *a, const void *w, const float *bias, const void *residual,
                                     void *y, long long M, int N, int K, bool out_bf16, int k_split,
                                     float *parts, hipStream_t stream) {
    GemmLn ex{};
    ex.k_split = k_split;
    ex.y_split = M * N;
    jv_status st = launch_gemm<JV_EPI_NONE, false, kGemmExtras>(a, w, nullptr, nullptr, parts, M, N, K, K, stream, ex);
    if (st != JV_OK) return st;
    const long long total4 = M * N / 4;
    const dim3 grid((unsigned)((total4 + 255) / 256));
    if (out_bf16)
        hipLaunchKernelGGL(gemm_split_combine<true>, grid, dim3(256), 0, stream, parts, M * N, k_split, bias, residual, y, total4, N);
    else
        hipLaunchKernelGGL(gemm_split_combine<false>, grid, dim3(256), 0, stream, parts, M * N, k_split, bias, residual, y, total4, N);
    return launch_status("gemm_split_combine");
}

// Shape limits of the GEMM (no pointers): what jv_gemm_bias_act documents.  The kernel addresses
// a tile's rows with 32-bit byte offsets from the tile's first row (256 rows of at most 2^21
// elements) and counts tiles and rows in 32-bit integers.
jv_status gemm_check_shape(long long M, int N, int K, long long lda_arg) {
    if (M <= 0 || N <= 0 || K <= 0) return fail(JV_ERR_INVALID_ARG, "M, N, K must be positive");
    const long long lda = lda_arg > 0 ? lda_arg : K;
    if (lda < K || lda % 8) return fail(JV_ERR_INVALID_ARG, "row stride of a below K or not a multiple of 8");
    if (K % 64) return fail(JV_ERR_UNSUPPORTED, "K must be a multiple of 64");
    if (N % 8) return fail(JV_ERR_UNSUPPORTED, "N must be a multiple of 8");
    if (lda > (1 << 21)) return fail(JV_ERR_UNSUPPORTED, "rows of a above 2^21 elements");
    if (M > (1ll << 30) || N > (1 << 30)) return fail(JV_ERR_UNSUPPORTED, "M or N above 2^30");
    const long long tiles = ((M + kBM - 1) / kBM) * ((N + kBN - 1) / kBN);
    if (tiles > (1ll << 30)) return fail(JV_ERR_UNSUPPORTED, "more than 2^30 output tiles");
    return JV_OK;
}

jv_status gemm_forward(const void *a, const void *w, const float *bias, const void *residual,
                       void *y, long long M, int N, int K, int epi, bool out_bf16,
                       hipStream_t stream, long long lda_arg) {
    jv_status shape = gemm_check_shape(M, N, K, lda_arg);
    if (shape != JV_OK) return shape;
    const int lda = (int)(lda_arg > 0 ? lda_arg : K);
    if (!a || !w || !y) return fail(JV_ERR_INVALID_ARG, "a, w, y must be non-null");
    if (((uintptr_t)a | (uintptr_t)w | (uintptr_t)y | (uintptr_t)bias | (uintptr_t)residual) & 15)
        return fail(JV_ERR_INVALID_ARG, "pointers must be 16-byte aligned");
    if (epi == JV_EPI_RESIDUAL && !residual)
        return fail(JV_ERR_INVALID_ARG, "residual epilogue needs a residual tensor");
    switch (epi) {
        case JV_EPI_NONE:
            return out_bf16 ? launch_gemm<JV_EPI_NONE, true>(a, w, bias, residual, y, M, N, K, lda, stream)
                            : launch_gemm<JV_EPI_NONE, false>(a, w, bias, residual, y, M, N, K, lda, stream);
        case JV_EPI_GELU:
            return out_bf16 ? launch_gemm<JV_EPI_GELU, true>(a, w, bias, residual, y, M, N, K, lda, stream)
                            : launch_gemm<JV_EPI_GELU, false>(a, w, bias, residual, y, M, N, K, lda, stream);
        case JV_EPI_RESIDUAL:
            return out_bf16 ? launch_gemm<JV_EPI_RESIDUAL, true>(a, w, bias, residual, y, M, N, K, lda, stream)
                            : launch_gemm<JV_EPI_RESIDUAL, false>(a, w, bias, residual, y, M, N, K, lda, stream);
        case JV_EPI_SILU:
            return out_bf16 ? launch_gemm<JV_EPI_SILU, true>(a, w, bias, residual, y, M, N, K, lda, stream)
                            : launch_gemm<JV_EPI_SILU, false>(a, w, bias, residual, y, M, N, K, lda, stream);
    }
    return fail(JV_ERR_INVALID_ARG, "unknown epilogue");
}

// The two GEMM forms of the folded LayerNorm (encoder only; shapes checked by the caller).
// Residual product that also leaves what the next LayerNorm needs: y = a w^T + bias + residual
// (fp32 or bf16), xb = bf16(y) when y is fp32, stats [M][N / 64][2].
static jv_status gemm_ln_produce(const void *a, const void *w, const float *bias, const void *residual,
                                 void *y, long long M, int N, int K, bool out_bf16, void *xb,
                                 float *stats, hipStream_t stream) {
    GemmLn ln{};
    ln.stats_out = stats;
    ln.xb_out = out_bf16 ? nullptr : xb;
    return out_bf16 ? launch_gemm<JV_EPI_RESIDUAL, true, kLnProduce>(a, w, bias, residual, y, M, N, K, K, stream, ln)
                    : launch_gemm<JV_EPI_RESIDUAL, false, kLnProduce>(a, w, bias, residual, y, M, N, K, K, stream, ln);
}
// Product that consumes a LayerNorm: y = epilogue(rstd (xb wg^T - mean c1) + c2), bf16 output.
static jv_status gemm_ln_consume(const void *xb, const void *wg, const float *c1, const float *c2,
                                 const float *stats, float eps, void *y, long long M, int N, int K,
                                 bool gelu, hipStream_t stream) {
    GemmLn ln{};
    ln.c1 = c1;
    ln.stats_in = stats;
    ln.groups = K / 64;
    ln.eps = eps;
    return gelu ? launch_gemm<JV_EPI_GELU, true, kLnConsume>(xb, wg, c2, nullptr, y, M, N, K, K, stream, ln)
                : launch_gemm<JV_EPI_NONE, true, kLnConsume>(xb, wg, c2, nullptr, y, M, N, K, K, stream, ln);
}

// Folding a LayerNorm's scale and shift into the weights of the product behind it, one
// wavefront per output feature n:  wg[n][k] = bf16(w[n][k] gamma[k]),  c1[n] = sum_k wg[n][k]
// (of the rounded values, which are what the matrix cores multiply),  c2[n] = bias[n] +
// sum_k w[n][k] beta[k].  grid (ceil(N / 4)), 256 threads; K % 8 == 0.
__global__ void __launch_bounds__(256)
fold_layernorm_kernel(const __bf16 *__restrict__ w, const float *__restrict__ bias,
                      const float *__restrict__ gamma, const float *__restrict__ beta,
                      __bf16 *__restrict__ wg, float *__restrict__ c1, float *__restrict__ c2, int N, int K) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int n = blockIdx.x * 4 + wave;
    if (n >= N) return;
    float s1 = 0.f, s2 = 0.f;
    for (int k = 8 * lane; k < K; k += 512) {
        const u32x4 raw = *(const u32x4 *)(w + (size_t)n * K + k);
        const f32x4 g0 = *(const f32x4 *)(gamma + k), g1 = *(const f32x4 *)(gamma + k + 4);
        const f32x4 b0 = *(const f32x4 *)(beta + k), b1 = *(const f32x4 *)(beta + k + 4);
        const float x[8] = {bf16_lo(raw[0]), bf16_hi(raw[0]), bf16_lo(raw[1]), bf16_hi(raw[1]),
                            bf16_lo(raw[2]), bf16_hi(raw[2]), bf16_lo(raw[3]), bf16_hi(raw[3])};
        const float gm[8] = {g0[0], g0[1], g0[2], g0[3], g1[0], g1[1], g1[2], g1[3]};
        const float bt[8] = {b0[0], b0[1], b0[2], b0[3], b1[0], b1[1], b1[2], b1[3]};
        u32x4 out;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            out[e] = pack_bf16x2(x[2 * e] * gm[2 * e], x[2 * e + 1] * gm[2 * e + 1]);
            s1 += bf16_lo(out[e]) + bf16_hi(out[e]);
            s2 = fmaf(x[2 * e], bt[2 * e], fmaf(x[2 * e + 1], bt[2 * e + 1], s2));
        }
        *(u32x4 *)(wg + (size_t)n * K + k) = out;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        s1 += __shfl_xor(s1, off, 64);
        s2 += __shfl_xor(s2, off, 64);
    }
    if (lane == 0) {
        c1[n] = s1;
        c2[n] = s2 + (bias ? bias[n] : 0.f);
    }
}

static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

}  // namespace jv

struct jv_encoder;
namespace jv {
static size_t encoder_linear_workspace(const jv_encoder *enc, int batch, int N);
}

// The encoder object: configuration and weight pointers, host memory only.
struct jv_encoder {
    jv_encoder_config cfg;
    uint8_t *pattern;
    jv_block_weights *blocks;
    jv_dwc_params *dwc;  // per block, a copy of the caller's parameters (mode none if absent)
    unsigned char *folded;  // caller's buffer with the LayerNorm-folded weights, or null (jv_encoder_fold_layernorm)
    bool fuse_la;           // jv_encoder_fuse_linear_projection
};

namespace jv {
// Largest linear-attention workspace any block needs (the blocks with a convolution branch
// also keep their generated filters there).
static int encoder_head_dim(const jv_encoder_config &c) { return c.width / c.heads; }  // 64 or 128 (jv_encoder_create)
static size_t encoder_linear_workspace(const jv_encoder *enc, int batch, int N) {
    if (encoder_head_dim(enc->cfg) == kHeadDimWide) {
        const size_t base = linear_wide_workspace_floats(batch, enc->cfg.heads, N);
        size_t need = base;
        for (int l = 0; l < enc->cfg.n_blocks; ++l) {
            DwcPlan plan;
            if (plan_dwc_wide(&enc->dwc[l], base, batch, enc->cfg.heads, N, &plan) == JV_OK)
                need = plan.total_floats > need ? plan.total_floats : need;
        }
        return need * sizeof(float);
    }
    const LinearPlan lp = plan_linear(batch, enc->cfg.heads, N);
    size_t need = linear_workspace_bytes(batch, enc->cfg.heads, N);
    for (int l = 0; l < enc->cfg.n_blocks; ++l) {
        DwcPlan plan;
        if (plan_dwc(&enc->dwc[l], lp, batch, enc->cfg.heads, N, &plan) == JV_OK) {
            const size_t bytes = plan.total_floats * sizeof(float);
            need = bytes > need ? bytes : need;
        }
    }
    return need;
}
// The linear-attention blocks that run with the apply pass folded into the output projection
// when jv_encoder_fuse_linear_projection is on: 64-channel heads, ReLU map, no convolution
// branch, separate LayerNorm passes, and images of a multiple of 256 tokens (a GEMM tile then
// lies inside one image).  The other blocks run the two passes and the plain projection.
static bool encoder_block_fuses(const jv_encoder *enc, int l, int N) {
    return enc->fuse_la && !enc->folded && enc->pattern[l] == 0 && encoder_head_dim(enc->cfg) == kHeadDim &&
           enc->cfg.la_focus_p <= 1 && enc->dwc[l].mode == JV_DWC_NONE && N % kBM == 0;
}
static bool encoder_any_block_fuses(const jv_encoder *enc, int N) {
    for (int l = 0; l < enc->cfg.n_blocks; ++l)
        if (encoder_block_fuses(enc, l, N)) return true;
    return false;
}
// Everything a forward pass over (batch, grid) would be refused for after its first launch,
// checked on the host: the four GEMM shapes, the window partition, the token-count limits of
// the mixers.
static jv_status encoder_check_shapes(const jv_encoder *enc, int batch, int grid_h, int grid_w) {
    const jv_encoder_config &c = enc->cfg;
    if (batch <= 0 || grid_h <= 0 || grid_w <= 0)
        return fail(JV_ERR_INVALID_ARG, "batch and grid must be positive");
    if ((long long)grid_h * grid_w > (1 << 24)) return fail(JV_ERR_UNSUPPORTED, "more than 2^24 tokens per image");
    if ((long long)batch * c.heads > 65535) return fail(JV_ERR_UNSUPPORTED, "batch * heads above 65535");
    if (encoder_head_dim(c) == kHeadDimWide && (long long)batch * c.heads > 16383)
        for (int l = 0; l < c.n_blocks; ++l)
            if (enc->pattern[l] == 0) return fail(JV_ERR_UNSUPPORTED, "head_dim 128: batch * heads above 16383");
    const long long N = c.n_prefix + (long long)grid_h * grid_w, T = batch * N;
    const int C = c.width;
    jv_status st;
    if ((st = gemm_check_shape(T, 3 * C, C)) != JV_OK) return st;
    if ((st = gemm_check_shape(T, C, C)) != JV_OK) return st;
    if ((st = gemm_check_shape(T, c.mlp_hidden, C)) != JV_OK) return st;
    if ((st = gemm_check_shape(T, C, c.mlp_hidden)) != JV_OK) return st;
    if (T > (1ll << 31)) return fail(JV_ERR_UNSUPPORTED, "more than 2^31 tokens");
    Problem pr;
    pr.B = batch; pr.heads = c.heads; pr.H = grid_h; pr.W = grid_w; pr.N = (int)N; pr.P = c.n_prefix;
    pr.D = encoder_head_dim(c);
    for (int l = 0; l < c.n_blocks; ++l)
        if (enc->pattern[l] == 1) return window_check(pr, c.win_h, c.win_w);
    return JV_OK;
}

}  // namespace jv

extern "C" {

jv_status jv_layernorm_fwd(const void *x, const float *gamma, const float *beta, void *y,
                           int64_t rows, int32_t cols, float eps, jv_dtype x_dtype,
                           jv_dtype y_dtype, void *hip_stream) {
    jv::clear_error();
    if (!x || !gamma || !beta || !y) return jv::fail(JV_ERR_INVALID_ARG, "null pointer");
    if (rows <= 0 || cols <= 0) return jv::fail(JV_ERR_INVALID_ARG, "rows and cols must be positive");
    if (cols % 8) return jv::fail(JV_ERR_UNSUPPORTED, "cols must be a multiple of 8");
    if (cols > 8192) return jv::fail(JV_ERR_UNSUPPORTED, "cols above 8192");
    if (rows > (1ll << 31)) return jv::fail(JV_ERR_UNSUPPORTED, "rows above 2^31");
    if (!(eps >= 0.f)) return jv::fail(JV_ERR_INVALID_ARG, "eps must be >= 0");
    if ((x_dtype != JV_F32 && x_dtype != JV_BF16) || (y_dtype != JV_F32 && y_dtype != JV_BF16))
        return jv::fail(JV_ERR_INVALID_ARG, "unknown dtype");
    if (((uintptr_t)x | (uintptr_t)y | (uintptr_t)gamma | (uintptr_t)beta) & 15)
        return jv::fail(JV_ERR_INVALID_ARG, "pointers must be 16-byte aligned");
    return jv::layernorm_forward(x, gamma, beta, y, rows, cols, eps, x_dtype == JV_BF16,
                                 y_dtype == JV_BF16, (hipStream_t)hip_stream);
}

jv_status jv_gemm_bias_act(const void *a, const void *w, const float *bias, const void *residual,
                           void *y, int64_t M, int32_t N, int32_t K, jv_epilogue epilogue,
                           jv_dtype y_dtype, void *hip_stream) {
    jv::clear_error();
    if (y_dtype != JV_F32 && y_dtype != JV_BF16) return jv::fail(JV_ERR_INVALID_ARG, "unknown dtype");
    return jv::gemm_forward(a, w, bias, residual, y, M, N, K, (int)epilogue, y_dtype == JV_BF16,
                            (hipStream_t)hip_stream);
}

jv_status jv_encoder_create(const jv_encoder_config *config, const jv_block_weights *blocks,
                            jv_encoder **out) {
    jv::clear_error();
    if (!config || !blocks || !out || !config->pattern)
        return jv::fail(JV_ERR_INVALID_ARG, "null argument");
    const jv_encoder_config &c = *config;
    if (c.n_blocks <= 0 || c.n_blocks > 4096) return jv::fail(JV_ERR_INVALID_ARG, "bad n_blocks");
    if (c.heads <= 0 || (c.width != c.heads * jv::kHeadDim && c.width != c.heads * jv::kHeadDimWide))
        return jv::fail(JV_ERR_UNSUPPORTED, "width must be heads * 64 or heads * 128");
    const bool wide = c.width == c.heads * jv::kHeadDimWide;
    if (wide && c.la_focus_p > 1)
        return jv::fail(JV_ERR_UNSUPPORTED, "head_dim 128: the focused map is built for 64-channel heads");
    if (c.mlp_hidden <= 0 || c.mlp_hidden % 64)
        return jv::fail(JV_ERR_UNSUPPORTED, "mlp_hidden must be a positive multiple of 64");
    if (c.win_h <= 0 || c.win_w <= 0) return jv::fail(JV_ERR_INVALID_ARG, "window must be positive");
    if (!(c.ln_eps >= 0.f) || !(c.la_eps >= 0.f)) return jv::fail(JV_ERR_INVALID_ARG, "bad epsilon");
    if (c.la_focus_p < 0 || c.la_focus_p > 16) return jv::fail(JV_ERR_INVALID_ARG, "la_focus_p must be 0 .. 16");
    if (c.n_prefix < 0 || c.n_prefix > 64) return jv::fail(JV_ERR_INVALID_ARG, "n_prefix must be 0 .. 64");
    if (c.stream_dtype != JV_F32 && c.stream_dtype != JV_BF16) return jv::fail(JV_ERR_INVALID_ARG, "bad stream_dtype");
    for (int l = 0; l < c.n_blocks; ++l) {
        if (c.pattern[l] > 2) return jv::fail(JV_ERR_INVALID_ARG, "pattern[%d] is not 0, 1 or 2", l);
        const jv_block_weights &b = blocks[l];
        const void *ptrs[] = {b.ln1_g, b.ln1_b, b.w_qkv, b.b_qkv, b.w_o, b.b_o,
                              b.ln2_g, b.ln2_b, b.w_fc1, b.b_fc1, b.w_fc2, b.b_fc2};
        for (const void *p : ptrs)
            if (!p || ((uintptr_t)p & 15))
                return jv::fail(JV_ERR_INVALID_ARG, "block %d: null or misaligned weight pointer", l);
        if (c.pattern[l] == 0 && b.dwc) {  // validate the convolution parameters now
            jv::DwcPlan plan;
            jv_status st = wide ? jv::plan_dwc_wide(b.dwc, 0, 1, c.heads, 256, &plan)
                                : jv::plan_dwc(b.dwc, jv::plan_linear(1, c.heads, 256), 1, c.heads, 256, &plan);
            if (st != JV_OK) return st;
        }
    }
    jv_encoder *e = new (std::nothrow) jv_encoder;
    if (!e) return jv::fail(JV_ERR_INVALID_ARG, "out of host memory");
    e->cfg = c;
    e->pattern = new (std::nothrow) uint8_t[c.n_blocks];
    e->blocks = new (std::nothrow) jv_block_weights[c.n_blocks];
    e->dwc = new (std::nothrow) jv_dwc_params[c.n_blocks];
    if (!e->pattern || !e->blocks || !e->dwc) {
        delete[] e->pattern;
        delete[] e->blocks;
        delete[] e->dwc;
        delete e;
        return jv::fail(JV_ERR_INVALID_ARG, "out of host memory");
    }
    for (int l = 0; l < c.n_blocks; ++l) {
        e->pattern[l] = c.pattern[l];
        e->blocks[l] = blocks[l];
        jv_dwc_params none = {JV_DWC_NONE, 3, 0, nullptr, nullptr, nullptr, nullptr, nullptr};
        e->dwc[l] = (c.pattern[l] == 0 && blocks[l].dwc) ? *blocks[l].dwc : none;
        e->blocks[l].dwc = &e->dwc[l];
    }
    e->cfg.pattern = e->pattern;
    e->folded = nullptr;
    e->fuse_la = false;
    *out = e;
    return JV_OK;
}

void jv_encoder_destroy(jv_encoder *enc) {
    if (!enc) return;
    delete[] enc->pattern;
    delete[] enc->blocks;
    delete[] enc->dwc;
    delete enc;
}

// Folded LayerNorm weights in the caller's buffer, per block: (w_qkv gamma1) bf16 [3C][C], c1 and
// c2 fp32 [3C]; (w_fc1 gamma2) bf16 [hidden][C], c1 and c2 fp32 [hidden]; each 256-byte aligned.
namespace jv {
struct FoldLayout {
    size_t wqkv, c1qkv, c2qkv, wfc1, c1fc1, c2fc1, block_bytes;
};
static FoldLayout fold_layout(const jv_encoder_config &c) {
    const size_t C = c.width, Hd = c.mlp_hidden;
    FoldLayout f;
    f.wqkv = 0;
    f.c1qkv = f.wqkv + align256(3 * C * C * 2);
    f.c2qkv = f.c1qkv + align256(3 * C * 4);
    f.wfc1 = f.c2qkv + align256(3 * C * 4);
    f.c1fc1 = f.wfc1 + align256(Hd * C * 2);
    f.c2fc1 = f.c1fc1 + align256(Hd * 4);
    f.block_bytes = f.c2fc1 + align256(Hd * 4);
    return f;
}
}  // namespace jv

jv_status jv_encoder_fuse_linear_projection(jv_encoder *enc, int32_t enable) {
    jv::clear_error();
    if (!enc) return jv::fail(JV_ERR_INVALID_ARG, "null encoder");
    enc->fuse_la = enable != 0;
    return JV_OK;
}

size_t jv_encoder_fold_bytes(const jv_encoder *enc) {
    jv::clear_error();
    if (!enc) return 0;
    return jv::fold_layout(enc->cfg).block_bytes * (size_t)enc->cfg.n_blocks;
}

jv_status jv_encoder_fold_layernorm(jv_encoder *enc, void *buffer, size_t buffer_bytes, void *hip_stream) {
    jv::clear_error();
    if (!enc) return jv::fail(JV_ERR_INVALID_ARG, "null encoder");
    if (!buffer) {  // back to separate LayerNorm passes
        enc->folded = nullptr;
        return JV_OK;
    }
    if ((uintptr_t)buffer & 255) return jv::fail(JV_ERR_INVALID_ARG, "buffer must be 256-byte aligned");
    const size_t need = jv_encoder_fold_bytes(enc);
    if (buffer_bytes < need)
        return jv::fail(JV_ERR_WORKSPACE_TOO_SMALL, "buffer has %zu bytes, %zu needed", buffer_bytes, need);
    const jv_encoder_config &c = enc->cfg;
    const jv::FoldLayout f = jv::fold_layout(c);
    hipStream_t stream = (hipStream_t)hip_stream;
    enc->folded = nullptr;
    for (int l = 0; l < c.n_blocks; ++l) {
        const jv_block_weights &b = enc->blocks[l];
        unsigned char *base = (unsigned char *)buffer + (size_t)l * f.block_bytes;
        hipLaunchKernelGGL(jv::fold_layernorm_kernel, dim3((3 * c.width + 3) / 4), dim3(256), 0, stream,
                           (const __bf16 *)b.w_qkv, b.b_qkv, b.ln1_g, b.ln1_b, (__bf16 *)(base + f.wqkv),
                           (float *)(base + f.c1qkv), (float *)(base + f.c2qkv), 3 * c.width, c.width);
        hipLaunchKernelGGL(jv::fold_layernorm_kernel, dim3((c.mlp_hidden + 3) / 4), dim3(256), 0, stream,
                           (const __bf16 *)b.w_fc1, b.b_fc1, b.ln2_g, b.ln2_b, (__bf16 *)(base + f.wfc1),
                           (float *)(base + f.c1fc1), (float *)(base + f.c2fc1), c.mlp_hidden, c.width);
        jv_status st = jv::launch_status("fold_layernorm_kernel");
        if (st != JV_OK) return st;
    }
    enc->folded = (unsigned char *)buffer;
    return JV_OK;
}

// Workspace: [T, width] bf16 (LayerNorm output, later the mixer output), [T, max(3 width,
// mlp_hidden)] bf16 (QKV, later the MLP hidden layer), then the linear-attention states; with
// folded LayerNorms also a second [T, width] bf16 buffer and the row statistics
// [T, width / 64, 2] fp32; with fused linear-attention projections the summed states
// [batch * heads][64 * 64 + 64] fp32 and the per-image weights [batch][width][width] bf16; for
// small token counts (fc2 with fewer than 128 output tiles) the fp32 partial results of its
// K split, [parts][T, width].
size_t jv_encoder_workspace_bytes(const jv_encoder *enc, int32_t batch, int32_t grid_h,
                                  int32_t grid_w) {
    jv::clear_error();
    if (!enc || jv::encoder_check_shapes(enc, batch, grid_h, grid_w) != JV_OK) return 0;
    const size_t T = (size_t)batch * (enc->cfg.n_prefix + (size_t)grid_h * grid_w), C = enc->cfg.width;
    const size_t wide = 3 * C > (size_t)enc->cfg.mlp_hidden ? 3 * C : (size_t)enc->cfg.mlp_hidden;
    const size_t fold = enc->folded ? jv::align256(T * C * 2) + jv::align256(T * (C / 64) * 8) : 0;
    const int N = enc->cfg.n_prefix + grid_h * grid_w;
    const size_t fuse = jv::encoder_any_block_fuses(enc, N)
                            ? jv::align256((size_t)batch * enc->cfg.heads * jv::kStateFloats * 4) + jv::align256((size_t)batch * C * C * 2)
                            : 0;
    const int k_split = enc->folded ? 1 : jv::gemm_k_split((long long)T, (int)C, enc->cfg.mlp_hidden);
    const size_t split = k_split > 1 ? jv::align256((size_t)k_split * T * C * 4) : 0;
    return jv::align256(T * C * 2) + jv::align256(T * wide * 2) +
           jv::align256(jv::encoder_linear_workspace(enc, batch, N)) + fold + fuse + split;
}

jv_status jv_encoder_forward(const jv_encoder *enc, const void *x, void *y, int32_t batch,
                             int32_t grid_h, int32_t grid_w, void *workspace,
                             size_t workspace_bytes, void *hip_stream) {
    return jv_encoder_forward_taps(enc, x, y, batch, grid_h, grid_w, 0, nullptr, nullptr, workspace,
                                   workspace_bytes, hip_stream);
}

jv_status jv_encoder_forward_taps(const jv_encoder *enc, const void *x, void *y, int32_t batch,
                                  int32_t grid_h, int32_t grid_w, int32_t n_taps,
                                  const int32_t *tap_blocks, void *const *tap_out,
                                  void *workspace, size_t workspace_bytes, void *hip_stream) {
    jv::clear_error();
    if (!enc || !x || !y || !workspace) return jv::fail(JV_ERR_INVALID_ARG, "null argument");
    if (n_taps < 0 || (n_taps > 0 && (!tap_blocks || !tap_out)))
        return jv::fail(JV_ERR_INVALID_ARG, "taps: negative count or null arrays");
    for (int i = 0; i < n_taps; ++i) {
        if (tap_blocks[i] < 0 || tap_blocks[i] >= enc->cfg.n_blocks || (i > 0 && tap_blocks[i] <= tap_blocks[i - 1]))
            return jv::fail(JV_ERR_INVALID_ARG, "tap_blocks must be strictly increasing block indices");
        if (!tap_out[i] || ((uintptr_t)tap_out[i] & 15) || tap_out[i] == x || tap_out[i] == y)
            return jv::fail(JV_ERR_INVALID_ARG, "tap_out[%d] must be a 16-byte aligned buffer of its own", i);
        for (int j = 0; j < i; ++j)
            if (tap_out[j] == tap_out[i]) return jv::fail(JV_ERR_INVALID_ARG, "tap_out entries must be distinct");
    }
    jv_status shapes = jv::encoder_check_shapes(enc, batch, grid_h, grid_w);
    if (shapes != JV_OK) return shapes;
    if (((uintptr_t)x | (uintptr_t)y) & 15) return jv::fail(JV_ERR_INVALID_ARG, "x, y must be 16-byte aligned");
    if ((uintptr_t)workspace & 255) return jv::fail(JV_ERR_INVALID_ARG, "workspace must be 256-byte aligned");
    const size_t need = jv_encoder_workspace_bytes(enc, batch, grid_h, grid_w);
    if (workspace_bytes < need)
        return jv::fail(JV_ERR_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed",
                        workspace_bytes, need);
    const jv_encoder_config &c = enc->cfg;
    const int N = c.n_prefix + grid_h * grid_w, C = c.width;
    const long long T = (long long)batch * N;
    hipStream_t stream = (hipStream_t)hip_stream;
    const size_t wide = 3 * (size_t)C > (size_t)c.mlp_hidden ? 3 * (size_t)C : (size_t)c.mlp_hidden;
    unsigned char *ws = (unsigned char *)workspace;
    __bf16 *narrow = (__bf16 *)ws;                                  // [T, C]
    __bf16 *widebuf = (__bf16 *)(ws + jv::align256(T * C * 2));     // [T, 3C] or [T, hidden]
    void *la_ws = ws + jv::align256(T * C * 2) + jv::align256(T * wide * 2);
    const size_t la_ws_bytes = jv::align256(jv::encoder_linear_workspace(enc, batch, N));
    // Folded LayerNorms (jv_encoder_fold_layernorm): the residual products leave the stream as
    // bf16 rows (when it is fp32) and the row statistics, and the products behind a LayerNorm
    // read those; only block 0's first LayerNorm, whose input no product of this pass wrote,
    // runs as a pass of its own.
    const bool fold = enc->folded != nullptr;
    __bf16 *stream16 = (__bf16 *)((unsigned char *)la_ws + la_ws_bytes);  // [T, C], the stream before LayerNorm 2
    float *row_stats = (float *)((unsigned char *)stream16 + jv::align256(T * C * 2));
    const jv::FoldLayout fl = jv::fold_layout(c);
    // fused linear-attention projections (jv_encoder_fuse_linear_projection): behind the fold buffers
    unsigned char *fuse_base = (unsigned char *)la_ws + la_ws_bytes +
                               (fold ? jv::align256(T * C * 2) + jv::align256(T * (C / 64) * 8) : 0);
    float *la_states = (float *)fuse_base;
    __bf16 *w_fold = (__bf16 *)(fuse_base + jv::align256((size_t)batch * c.heads * jv::kStateFloats * 4));
    // K split of fc2 when its tiles would leave most compute units idle (gemm_residual_split)
    const int fc2_split = fold ? 1 : jv::gemm_k_split(T, C, c.mlp_hidden);
    float *fc2_parts = (float *)(fuse_base + (jv::encoder_any_block_fuses(enc, N)
                                                  ? jv::align256((size_t)batch * c.heads * jv::kStateFloats * 4) + jv::align256((size_t)batch * C * C * 2)
                                                  : 0));
    bool ln1_folded = false;  // the previous block's last product has left rows and statistics for LayerNorm 1

    // Q, K, V as strided views of the [B, N, 3, heads, 64] projection output; O as [B, N, heads, 64].
    jv::Problem pr;
    pr.B = batch; pr.heads = c.heads; pr.H = grid_h; pr.W = grid_w; pr.N = N; pr.P = c.n_prefix;
    pr.D = jv::encoder_head_dim(c);
    pr.bf16 = true; pr.o_bf16 = true;
    const long long sb = (long long)N * 3 * C, sn = 3LL * C;
    pr.q = {widebuf, sb, pr.D, sn};
    pr.k = {widebuf + C, sb, pr.D, sn};
    pr.v = {widebuf + 2 * C, sb, pr.D, sn};
    pr.o = {narrow, (long long)N * C, pr.D, C};

    jv_status st;
    const bool s16 = c.stream_dtype == JV_BF16;  // element type of the residual stream
    const void *resid = x;  // the first residual add reads the input and writes y
    int next_tap = 0;
    for (int l = 0; l < c.n_blocks; ++l) {
        const jv_block_weights &b = enc->blocks[l];
        const unsigned char *fw = fold ? enc->folded + (size_t)l * fl.block_bytes : nullptr;
        if (ln1_folded) {
            st = jv::gemm_ln_consume(s16 ? resid : (const void *)narrow, fw + fl.wqkv, (const float *)(fw + fl.c1qkv),
                                     (const float *)(fw + fl.c2qkv), row_stats, c.ln_eps, widebuf, T, 3 * C, C, false, stream);
            if (st != JV_OK) return st;
        } else {
            if ((st = jv::layernorm_forward(resid, b.ln1_g, b.ln1_b, narrow, T, C, c.ln_eps, s16, true, stream)) != JV_OK) return st;
            if ((st = jv::gemm_forward(narrow, b.w_qkv, b.b_qkv, nullptr, widebuf, T, 3 * C, C, JV_EPI_NONE, true, stream)) != JV_OK) return st;
        }
        const bool fused = jv::encoder_block_fuses(enc, l, N);
        switch (enc->pattern[l]) {
            case 0:
                if (fused)  // the scaled queries take the place of the mixer's output
                    st = jv::linear_fused_projection_operands(pr, c.la_eps, (float *)la_ws, la_states, b.w_o, w_fold, narrow, stream);
                else
                    st = jv::linear_block_forward(pr, c.la_eps, &enc->dwc[l], la_ws, la_ws_bytes, stream,
                                                  c.la_focus_p > 1 ? c.la_focus_p : 1);
                break;
            case 1: st = jv::window_forward(pr, c.win_h, c.win_w, 0.f, stream); break;
            default: st = jv::full_forward(pr, 0.f, stream); break;
        }
        if (st != JV_OK) return st;
        if (fold) {
            if ((st = jv::gemm_ln_produce(narrow, b.w_o, b.b_o, resid, y, T, C, C, s16, stream16, row_stats, stream)) != JV_OK) return st;
            st = jv::gemm_ln_consume(s16 ? (const void *)y : (const void *)stream16, fw + fl.wfc1, (const float *)(fw + fl.c1fc1),
                                     (const float *)(fw + fl.c2fc1), row_stats, c.ln_eps, widebuf, T, c.mlp_hidden, C, true, stream);
            if (st != JV_OK) return st;
        } else {
            if (fused) {
                jv::GemmLn per_image{};
                per_image.w_rows = N;
                per_image.w_stride = (long long)C * C;
                st = s16 ? jv::launch_gemm<JV_EPI_RESIDUAL, true, jv::kGemmExtras>(narrow, w_fold, b.b_o, resid, y, T, C, C, C, stream, per_image)
                         : jv::launch_gemm<JV_EPI_RESIDUAL, false, jv::kGemmExtras>(narrow, w_fold, b.b_o, resid, y, T, C, C, C, stream, per_image);
            } else {
                st = jv::gemm_forward(narrow, b.w_o, b.b_o, resid, y, T, C, C, JV_EPI_RESIDUAL, s16, stream);
            }
            if (st != JV_OK) return st;
            if ((st = jv::layernorm_forward(y, b.ln2_g, b.ln2_b, narrow, T, C, c.ln_eps, s16, true, stream)) != JV_OK) return st;
            if ((st = jv::gemm_forward(narrow, b.w_fc1, b.b_fc1, nullptr, widebuf, T, c.mlp_hidden, C, JV_EPI_GELU, true, stream)) != JV_OK) return st;
        }
        // A tapped block leaves its result in the tap buffer and the next block picks the stream
        // up from there; the last block's result has to be in y as well.
        const bool tapped = next_tap < n_taps && tap_blocks[next_tap] == l;
        void *out = tapped && l + 1 < c.n_blocks ? tap_out[next_tap] : y;
        ln1_folded = fold && l + 1 < c.n_blocks;
        if (ln1_folded) {  // (the bf16 rows go where the next block's LayerNorm 1 would have written)
            if ((st = jv::gemm_ln_produce(widebuf, b.w_fc2, b.b_fc2, y, out, T, C, c.mlp_hidden, s16, narrow, row_stats, stream)) != JV_OK) return st;
        } else if (fc2_split > 1) {
            if ((st = jv::gemm_residual_split(widebuf, b.w_fc2, b.b_fc2, y, out, T, C, c.mlp_hidden, s16, fc2_split, fc2_parts, stream)) != JV_OK) return st;
        } else {
            if ((st = jv::gemm_forward(widebuf, b.w_fc2, b.b_fc2, y, out, T, C, c.mlp_hidden, JV_EPI_RESIDUAL, s16, stream)) != JV_OK) return st;
        }
        if (tapped && out == y) {
            hipError_t e = hipMemcpyAsync(tap_out[next_tap], y, (size_t)T * C * (s16 ? 2 : 4), hipMemcpyDeviceToDevice, stream);
            if (e != hipSuccess) return jv::fail(JV_ERR_HIP, "hipMemcpyAsync: %s", hipGetErrorString(e));
        }
        if (tapped) ++next_tap;
        resid = out;
    }
    return JV_OK;
}

}  // extern "C"
