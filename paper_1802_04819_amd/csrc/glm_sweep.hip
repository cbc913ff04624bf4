// Hyper-parameter sweep kernels for gfx950: up to 64 models at a time (the entry point loops over
// groups of 64; a group of at most 32 runs kernels that carry one 32-model tile instead of two)
// share one X, so the margins and the
// gradients are dense fp32 matrix products, computed on the matrix cores with
// v_mfma_f32_32x32x2_f32 (fp32 inputs, fp32 accumulate: the same roundings class as an fma chain).
//
//   forward  : Z = X . W^T   [N, 64], then per element loss and residual; R [N, 64] is written,
//              per-tile per-model loss sums go to lossP.  Tile = 128 rows x 64 models per block,
//              K-loop over D in chunks of 32 staged through LDS (coalesced float4 global loads,
//              128-bit LDS reads along k).
//   backward : G = R^T . X   [64, D], contraction over the N rows, split across blocks; a block
//              owns a 256-column slab and every S-th 32-row chunk, and writes its partial
//              [64, 256] to Gpart[s]; nothing is added atomically.
//   finalize : per model, sums the S partials in order (fp64), applies 1/N, lambda_m, step_m,
//              writes G, the loss-history row and the new W.
//
// Lane layout of the 32x32x2 instruction (lane l of 64): A[i][k] from lane i + 32 k,
// B[k][j] from lane j + 32 k, D[i][j] in lane j + 32 ((i / 4) % 2), register (i % 4) + 4 (i / 8).
#include <algorithm>

#include "glm_internal.h"
#include "glm_loss.h"

namespace slaqglm {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float f4 __attribute__((ext_vector_type(4)));   // first-class vector: stays in registers

constexpr int kFwdRows = kSweepFwdRows;    // rows per forward block (4 waves x 32)
constexpr int kFwdK = 32;        // k-chunk staged per step
constexpr int kFwdLd = 36;       // LDS row stride in floats (16-byte aligned, staggers banks)

__device__ __forceinline__ floatx16 mfma32(float a, float b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

// Address arithmetic of the K loops: every global load is "uniform base + a 32-bit byte offset that
// the thread keeps for the whole kernel"; the base moves from chunk to chunk on the scalar unit.
// Vector instructions issued between matrix instructions cost matrix-core time (the kernel with
// 58 of them per 32 matrix instructions in the loop ran 5 % slower than with 6), so the masks for
// the ragged cases (last chunk of a D that is no multiple of 32, fewer models than the tile holds)
// exist only in the kernel variant for those cases (PLAIN = false); both variants add the same
// numbers in the same order.
__device__ __forceinline__ f4 load_nt_at(const f4 *__restrict__ base, unsigned byte_off) {
    return __builtin_nontemporal_load(reinterpret_cast<const f4 *>(reinterpret_cast<const char *>(base) + byte_off));
}
__device__ __forceinline__ f4 load_at(const f4 *__restrict__ base, unsigned byte_off) {
    return *reinterpret_cast<const f4 *>(reinterpret_cast<const char *>(base) + byte_off);
}

template <bool HALF, bool PLAIN>
__global__ __launch_bounds__(256) void sweep_forward_kernel(
    const float *__restrict__ X, const float *__restrict__ y, const float *__restrict__ W,
    long long N, int D, int M, int loss, float *__restrict__ R, float *__restrict__ lossP, int T) {
    __shared__ f4 Xs4[kFwdRows * kFwdLd / 4];
    __shared__ f4 Ws4[kSweepM * kFwdLd / 4];
    __shared__ float lsm[4][kSweepM];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 31, lh = lane >> 5;
    const int tile = blockIdx.x;
    const long long r0 = (long long)tile * kFwdRows;
    const int D4 = D >> 2;
    const f4 *__restrict__ Xb = reinterpret_cast<const f4 *>(X) + r0 * D4;     // the tile's first row
    const f4 *__restrict__ Wb = reinterpret_cast<const f4 *>(W);

    // staging assignments: X chunk = 128 rows x 8 f4, W chunk = 64 rows x 8 f4
    constexpr int WQ = HALF ? 1 : 2;          // W rows staged per thread: 32 or 64 models
    constexpr int RS = HALF ? 32 : kSweepM;   // row stride of R
    constexpr int MT = HALF ? 32 : kSweepM;   // models of a full tile
    unsigned xo[4], xrow_o[4]; int xc4[4];   // byte offsets from Xb: of the thread's slot, of its row
    f4 *xdst[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int idx = tid + 256 * q;
        const long long r = r0 + (idx >> 3);
        const unsigned rel = (unsigned)((r < N ? r : N - 1) - r0);     // rows past N read the last row
        xc4[q] = idx & 7;
        xrow_o[q] = rel * (unsigned)D4 * 16u;
        xo[q] = xrow_o[q] + (unsigned)xc4[q] * 16u;
        xdst[q] = Xs4 + (idx >> 3) * (kFwdLd / 4) + (idx & 7);
    }
    unsigned wo[WQ], wrow_o[WQ]; int wc4[WQ]; float wmask[WQ];   // models past M read row 0 and are multiplied by 0
    f4 *wdst[WQ];
#pragma unroll
    for (int q = 0; q < WQ; ++q) {
        const int idx = tid + 256 * q;
        const int m = idx >> 3;
        wmask[q] = m < M ? 1.0f : 0.0f;
        wc4[q] = idx & 7;
        wrow_o[q] = (unsigned)(m < M ? m : 0) * (unsigned)D4 * 16u;
        wo[q] = wrow_o[q] + (unsigned)wc4[q] * 16u;
        wdst[q] = Ws4 + (idx >> 3) * (kFwdLd / 4) + (idx & 7);
    }
    const int nchunk = (D + kFwdK - 1) / kFwdK;
    // PLAIN: D is a multiple of 32 and the tile is full of models (the launch checks it)
    const int ragged = PLAIN ? -1 : ((D % kFwdK) != 0 ? nchunk - 1 : -1);   // the chunk with slots past the row length
    (void)MT;

    floatx16 acc0 = {0}, acc1 = {0};
    // A chunk is 8 float4 slots of k.  Slots past the row length (last chunk of a D that is not a
    // multiple of 32) read a clamped slot and are multiplied by 0 on both operands; every other
    // chunk is staged as it is (also its infinities and NaNs).
#define SLAQ_FWD_FETCH(KC)                                                                   \
    {                                                                                        \
        const int kc_ = (KC);                                                                \
        if (PLAIN || kc_ != ragged) {                                                        \
            const f4 *__restrict__ xc_ = Xb + kc_ * (kFwdK / 4);                             \
            const f4 *__restrict__ wc_ = Wb + kc_ * (kFwdK / 4);                             \
            _Pragma("unroll") for (int q = 0; q < 4; ++q) xr[q] = load_nt_at(xc_, xo[q]);    \
            _Pragma("unroll") for (int q = 0; q < WQ; ++q) wr[q] = load_at(wc_, wo[q]);      \
        } else {                                                                             \
            _Pragma("unroll") for (int q = 0; q < 4; ++q) {                                  \
                const int c_ = kc_ * (kFwdK / 4) + xc4[q];                                   \
                xr[q] = load_nt_at(Xb, xrow_o[q] + (unsigned)(c_ < D4 ? c_ : D4 - 1) * 16u); \
            }                                                                                \
            _Pragma("unroll") for (int q = 0; q < WQ; ++q) {                                 \
                const int c_ = kc_ * (kFwdK / 4) + wc4[q];                                   \
                wr[q] = load_at(Wb, wrow_o[q] + (unsigned)(c_ < D4 ? c_ : D4 - 1) * 16u);    \
            }                                                                                \
        }                                                                                    \
    }
#define SLAQ_FWD_STASH(KC)                                                                   \
    {                                                                                        \
        const int kc_ = (KC);                                                                \
        if (PLAIN) {                                                                         \
            _Pragma("unroll") for (int q = 0; q < 4; ++q) *xdst[q] = xr[q];                  \
            _Pragma("unroll") for (int q = 0; q < WQ; ++q) *wdst[q] = wr[q];                 \
        } else if (kc_ != ragged) {                                                          \
            _Pragma("unroll") for (int q = 0; q < 4; ++q) *xdst[q] = xr[q];                  \
            _Pragma("unroll") for (int q = 0; q < WQ; ++q) *wdst[q] = wr[q] * wmask[q];      \
        } else {                                                                             \
            _Pragma("unroll") for (int q = 0; q < 4; ++q)                                    \
                *xdst[q] = xr[q] * (kc_ * (kFwdK / 4) + xc4[q] < D4 ? 1.0f : 0.0f);          \
            _Pragma("unroll") for (int q = 0; q < WQ; ++q)                                   \
                *wdst[q] = wr[q] * (kc_ * (kFwdK / 4) + wc4[q] < D4 ? wmask[q] : 0.0f);      \
        }                                                                                    \
    }

    {
        f4 xr[4], wr[WQ];
        SLAQ_FWD_FETCH(0)
        SLAQ_FWD_STASH(0)
    }
    __syncthreads();
    const f4 *arow = Xs4 + (wave * 32 + li) * (kFwdLd / 4) + lh;
    const f4 *b0row = Ws4 + li * (kFwdLd / 4) + lh;
    const f4 *b1row = Ws4 + (32 + li) * (kFwdLd / 4) + lh;
    for (int kc = 0; kc < nchunk; ++kc) {
        f4 xr[4], wr[WQ];
        const int kn = kc + 1 < nchunk ? kc + 1 : kc;   // last trip re-reads its own chunk (cache hit)
        SLAQ_FWD_FETCH(kn)
        __builtin_amdgcn_sched_barrier(0);              // keep the prefetch ahead of the matrix ops
#pragma unroll
        for (int kb = 0; kb < kFwdK / 8; ++kb) {        // 8 k values: lanes lh=0 take 0..3, lh=1 4..7
            const f4 a = arow[2 * kb];
            const f4 b0 = b0row[2 * kb];
            if constexpr (HALF) {
                acc0 = mfma32(a.x, b0.x, acc0);
                acc0 = mfma32(a.y, b0.y, acc0);
                acc0 = mfma32(a.z, b0.z, acc0);
                acc0 = mfma32(a.w, b0.w, acc0);
            } else {
                const f4 b1 = b1row[2 * kb];
                acc0 = mfma32(a.x, b0.x, acc0); acc1 = mfma32(a.x, b1.x, acc1);
                acc0 = mfma32(a.y, b0.y, acc0); acc1 = mfma32(a.y, b1.y, acc1);
                acc0 = mfma32(a.z, b0.z, acc0); acc1 = mfma32(a.z, b1.z, acc1);
                acc0 = mfma32(a.w, b0.w, acc0); acc1 = mfma32(a.w, b1.w, acc1);
            }
        }
        __syncthreads();
        SLAQ_FWD_STASH(kn)
        __syncthreads();
    }
#undef SLAQ_FWD_FETCH
#undef SLAQ_FWD_STASH

    // epilogue: lane holds models li (acc0) and 32 + li (acc1) for 16 rows of the wave's 32
    float ls0 = 0.0f, ls1 = 0.0f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const long long row = r0 + wave * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
        const bool valid = row < N;
        const float yy = y[valid ? row : N - 1];
        float l0, q0, l1 = 0.0f, q1 = 0.0f;
        loss_residual(loss, acc0[r], yy, l0, q0);
        if constexpr (!HALF) loss_residual(loss, acc1[r], yy, l1, q1);
        if (valid) {
            ls0 += l0; ls1 += l1;
            R[row * RS + li] = q0;                       // a half group keeps 32 residuals per row
            if constexpr (!HALF) R[row * RS + 32 + li] = q1;
        }
    }
    // add the two half-waves (fixed order), then the four waves in wave order
    ls0 = ls0 + __shfl_xor(ls0, 32, 64);
    ls1 = ls1 + __shfl_xor(ls1, 32, 64);
    if (lh == 0) { lsm[wave][li] = ls0; lsm[wave][32 + li] = ls1; }
    __syncthreads();
    if (tid < M) {
        const float s = ((lsm[0][tid] + lsm[1][tid]) + lsm[2][tid]) + lsm[3][tid];
        lossP[(size_t)tid * T + tile] = s;
    }
}

constexpr int kBwdRows = kSweepBwdRows;     // rows per staged chunk
constexpr int kBwdCols = kSweepBwdCols;     // columns per block slab (4 waves x 64)

template <bool HALF>
__global__ __launch_bounds__(256) void sweep_backward_kernel(
    const float *__restrict__ X, const float *__restrict__ R, long long N, int D, int S,
    float *__restrict__ Gpart) {
    __shared__ f4 Xs4[kBwdRows * kBwdCols / 4];
    __shared__ f4 Rs4[kBwdRows * kSweepM / 4];
    const float *Xs = reinterpret_cast<const float *>(Xs4);
    const float *Rs = reinterpret_cast<const float *>(Rs4);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 31, lh = lane >> 5;
    const int nslab = (D + kBwdCols - 1) / kBwdCols;
    const int slab = blockIdx.x % nslab;
    const int s = blockIdx.x / nslab;
    const int D4 = D >> 2;
    const f4 *__restrict__ X4 = reinterpret_cast<const f4 *>(X);
    const f4 *__restrict__ R4 = reinterpret_cast<const f4 *>(R);
    const long long nchunks = (N + kBwdRows - 1) / kBwdRows;

    constexpr int RS = HALF ? 32 : kSweepM;            // row stride of R (and of its copy in LDS)
    constexpr int RQ = HALF ? 1 : 2;                   // float4 of R staged per thread and chunk
    floatx16 acc[2][2] = {{{0}, {0}}, {{0}, {0}}};     // [model tile][column tile]
    // Byte offsets from the chunk's first row, kept for the whole kernel (see the forward kernel):
    // X slot (row = idx / 64, f4 column = idx % 64 of the slab; slab columns past D read a valid
    // slot, their sums are never stored); the R chunk is contiguous.
    unsigned xo[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        const int idx = tid + 256 * q;
        int c4 = slab * (kBwdCols / 4) + (idx & 63);
        c4 = c4 < D4 ? c4 : D4 - 1;
        xo[q] = ((unsigned)(idx >> 6) * (unsigned)D4 + (unsigned)c4) * 16u;
    }
#define SLAQ_BWD_FETCH(CH)                                                                   \
    {                                                                                        \
        const long long rbase = (CH) * kBwdRows;                                             \
        if (rbase + kBwdRows <= N) {                   /* every row of the chunk exists */   \
            const f4 *__restrict__ xc_ = X4 + rbase * D4;                                    \
            const f4 *__restrict__ rc_ = R4 + rbase * (RS / 4);                              \
            _Pragma("unroll") for (int q = 0; q < 8; ++q) xr[q] = load_nt_at(xc_, xo[q]);    \
            _Pragma("unroll") for (int q = 0; q < RQ; ++q)                                   \
                rr[q] = load_at(rc_, (unsigned)(tid + 256 * q) * 16u);                       \
        } else {                                                                             \
            _Pragma("unroll") for (int q = 0; q < 8; ++q) {                                  \
                const int idx = tid + 256 * q;                                               \
                long long row = rbase + (idx >> 6);                                          \
                row = row < N ? row : N - 1;                                                 \
                xr[q] = load_nt_at(X4 + row * D4, xo[q] - (unsigned)(idx >> 6) * (unsigned)D4 * 16u); \
            }                                                                                \
            _Pragma("unroll") for (int q = 0; q < RQ; ++q) {                                 \
                const int idx = tid + 256 * q;     /* row = idx / (RS/4), f4 model = idx % (RS/4) */ \
                const long long row = rbase + idx / (RS / 4);                                \
                const f4 v_ = R4[(row < N ? row : N - 1) * (RS / 4) + idx % (RS / 4)];       \
                rr[q] = v_ * (row < N ? 1.0f : 0.0f);      /* rows past N add nothing */      \
            }                                                                                \
        }                                                                                    \
    }
#define SLAQ_BWD_STASH()                                                                     \
    {                                                                                        \
        _Pragma("unroll") for (int q = 0; q < 8; ++q) Xs4[tid + 256 * q] = xr[q];            \
        _Pragma("unroll") for (int q = 0; q < RQ; ++q) Rs4[tid + 256 * q] = rr[q];           \
    }

    long long c = s;
    if (c < nchunks) {
        f4 xr[8], rr[RQ];
        SLAQ_BWD_FETCH(c)
        SLAQ_BWD_STASH()
    }
    __syncthreads();
    const float *xa = Xs + lh * kBwdCols + wave * 64 + li;
    const float *ra = Rs + lh * RS + li;
    for (; c < nchunks; c += S) {
        f4 xr[8], rr[RQ];
        SLAQ_BWD_FETCH(c + S < nchunks ? c + S : c)     // last trip re-reads its own chunk
        __builtin_amdgcn_sched_barrier(0);              // keep the prefetch ahead of the matrix ops
#pragma unroll
        for (int kp = 0; kp < kBwdRows / 2; ++kp) {       // contraction rows 2 kp + lh
            const float a0 = ra[2 * kp * RS];
            const float b0 = xa[2 * kp * kBwdCols];
            const float b1 = xa[2 * kp * kBwdCols + 32];
            acc[0][0] = mfma32(a0, b0, acc[0][0]);
            acc[0][1] = mfma32(a0, b1, acc[0][1]);
            if constexpr (!HALF) {
                const float a1 = ra[2 * kp * RS + 32];
                acc[1][0] = mfma32(a1, b0, acc[1][0]);
                acc[1][1] = mfma32(a1, b1, acc[1][1]);
            }
        }
        __syncthreads();
        SLAQ_BWD_STASH()
        __syncthreads();
    }
#undef SLAQ_BWD_FETCH
#undef SLAQ_BWD_STASH

    float *__restrict__ gp = Gpart + (size_t)s * kSweepM * D + slab * kBwdCols + wave * 64;
#pragma unroll
    for (int mt = 0; mt < (HALF ? 1 : 2); ++mt)
#pragma unroll
        for (int ct = 0; ct < 2; ++ct)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int model = 32 * mt + 8 * (r >> 2) + 4 * lh + (r & 3);
                if (slab * kBwdCols + wave * 64 + 32 * ct + li < D)
                    gp[(size_t)model * D + 32 * ct + li] = acc[mt][ct][r];
            }
}

// ------------------------------------------------------------------ one-pass kernel for a group of at most 16 models
//
// With 16 models the two products of an iteration are 64 flop per byte of X together: the iteration is
// bound by the memory, and reading X twice (forward, then backward) costs twice the time.  Here a
// block keeps a tile of 16 rows x D of X in LDS and uses it for both products, so X is read once and
// R never leaves the chip.  v_mfma_f32_16x16x4_f32; lane l = (l % 16, l / 16) = (c, g):
//   A[i][k] from lane (i, k), B[k][j] from lane (j, k), D[i][j] in lane (j, i / 4), register i % 4.
//   forward : Z[row][model] = sum_k X[row][k] W[model][k].  The wave takes the 16-wide k steps
//             4 u + wave; its slice of W stays in registers for the whole launch (lane (model, g)
//             holds W[model][16 s + 4 g .. + 3] of step s, matching the 128-bit LDS read of lane
//             (row, g) from the tile).  The four waves' partial Z meet in LDS and are added in wave
//             order; thread (model, row) forms loss and residual and keeps its loss sum.
//   backward: Gp[model][col] += sum_row R[row][model] X[row][col].  The wave takes the 64-column
//             groups 4 u + wave; lane (model, g) supplies R[4 g + q][model] in step q, lane (dd, g)
//             X[4 g + q][64 grp + 4 dd + t] for column tile t from one 128-bit read, so tile t
//             covers the columns 64 grp + 4 dd + t and the four tiles of a lane store as one float4.
// Blocks walk the row tiles with stride gridDim and write one partial [16, D] each; the grid is a
// function of N only, so the order of all additions is fixed by the shape.
constexpr int kFusedM = kSweepFusedM;
constexpr int kFusedRows = 16;
constexpr int kFusedZld = 20;         // LDS row stride of the 16 x 16 exchange tiles

typedef float floatx4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ floatx4 mfma16(float a, float b, floatx4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

// Waves per block: eight for the long rows, so that a wave's slice of W, its accumulators and its share
// of the next tile fit in 128 registers and two blocks (16 waves) share a compute unit.
constexpr int fused_waves(int dmax) { return dmax >= 1024 ? 16 : dmax >= 512 ? 8 : 4; }

size_t sweep_fused_lds_bytes(int D, int dmax) {
    return sizeof(float) * ((size_t)kFusedRows * (D + 4) + (size_t)fused_waves(dmax) * kFusedM * kFusedZld +
                            kFusedM * kFusedZld);
}

template <int DMAX>
__global__ __launch_bounds__(64 * fused_waves(DMAX), 4) void sweep_fused_kernel(      // four waves per SIMD
    const float *__restrict__ X, const float *__restrict__ y, const float *__restrict__ W,
    long long N, int D, int M, int loss, float *__restrict__ Gpart, float *__restrict__ lossP) {
    extern __shared__ f4 fused_smem[];
    constexpr int NW = fused_waves(DMAX);
    constexpr int NGW = DMAX / (64 * NW);   // column groups of 64 per wave
    constexpr int NQ = 4 * NGW;             // float4 slots of the tile per lane: 16 rows x 64 columns per group
    static_assert(NGW >= 1, "fewer column groups than waves");
    const int LD = D + 4;                   // row stride of the tile in LDS (floats)
    float *Xs = reinterpret_cast<float *>(fused_smem);
    float *zs = Xs + kFusedRows * LD;                   // [NW waves][16 models][kFusedZld]
    float *rs = zs + NW * kFusedM * kFusedZld;          // [16 models][kFusedZld]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lc = lane & 15, lg = lane >> 4;
    const int D4 = D >> 2;
    const long long ntiles = (N + kFusedRows - 1) / kFusedRows;
    const f4 *__restrict__ X4 = reinterpret_cast<const f4 *>(X);

    // The wave owns the column groups NW u + wave of the tile: it fetches them, puts them into LDS,
    // takes their 16-wide k steps in the forward product and their columns in the backward product.
    // Nobody else touches them, so the tile itself needs no barrier: the wave's own LDS operations
    // are carried out in program order.
    // its slice of W: zero for models past M and steps past D
    f4 wreg[NGW][4];
#pragma unroll
    for (int u = 0; u < NGW; ++u)
#pragma unroll
        for (int sidx = 0; sidx < 4; ++sidx) {
            const int st = 4 * (NW * u + wave) + sidx;
            const bool ok = lc < M && 16 * st < D;
            const f4 t = reinterpret_cast<const f4 *>(W)[(size_t)(lc < M ? lc : 0) * D4 + (16 * st < D ? 4 * st + lg : 0)];
            wreg[u][sidx] = ok ? t : f4{0.f, 0.f, 0.f, 0.f};
        }
    const int lj = (tid >> 4) & 15, li = tid & 15;      // loss phase: thread (model lj, row li) of the first 256

    floatx4 acc[NGW][4];
#pragma unroll
    for (int u = 0; u < NGW; ++u)
#pragma unroll
        for (int t = 0; t < 4; ++t) acc[u][t] = floatx4{0.f, 0.f, 0.f, 0.f};
    float lsum = 0.0f;

    // Slot (u, q) of the lane: row 4 lg + q, float4 column 16 (NW u + wave) + lc: a load instruction
    // takes 256 contiguous bytes of each of four rows.  Rows past N (last tile only) read row N - 1 and
    // get residual zero below; one form for both cases keeps the slots in one set of registers.
    f4 xr[NQ];
    float yr = 0.0f;
#define SLAQ_FUSED_LOAD(U, Q, TB, LIM)                                                                      \
    {                                                                                                       \
        const int c4_ = 16 * (NW * (U) + wave) + lc;                                                        \
        const int row_ = 4 * lg + (Q) < (LIM) ? 4 * lg + (Q) : (LIM);                                       \
        xr[4 * (U) + (Q)] = load_nt_at(TB, (unsigned)(row_ * D4 + (c4_ < D4 ? c4_ : 0)) * 16u);             \
    }
#define SLAQ_FUSED_STASH()                                                                                  \
    {                                                                                                       \
        _Pragma("unroll") for (int u = 0; u < NGW; ++u) {                                                   \
            const int c4_ = 16 * (NW * u + wave) + lc;                                                      \
            if (c4_ < D4) {                                                                                 \
                _Pragma("unroll") for (int q = 0; q < 4; ++q)                                               \
                    *reinterpret_cast<f4 *>(Xs + (4 * lg + q) * LD + 4 * c4_) = xr[4 * u + q];              \
            }                                                                                               \
        }                                                                                                   \
    }

    long long tile = blockIdx.x;
    float yc = 0.0f;
    if (tile < ntiles) {
        const long long r0 = tile * kFusedRows;
        const int lim = (int)(N - 1 - r0 < kFusedRows - 1 ? N - 1 - r0 : kFusedRows - 1);
        const f4 *__restrict__ tb = X4 + r0 * D4;
#pragma unroll
        for (int u = 0; u < NGW; ++u)
#pragma unroll
            for (int q = 0; q < 4; ++q) SLAQ_FUSED_LOAD(u, q, tb, lim)
        yr = y[r0 + li < N ? r0 + li : N - 1];
    }
    for (; tile < ntiles; tile += gridDim.x) {
        // the tile's columns into LDS, then the request for the next tile's
        SLAQ_FUSED_STASH()
        yc = yr;
        const long long nt = tile + gridDim.x;
        if (nt < ntiles) {
            const long long nr0 = nt * kFusedRows;
            const int nlim = (int)(N - 1 - nr0 < kFusedRows - 1 ? N - 1 - nr0 : kFusedRows - 1);
            const f4 *__restrict__ ntb = X4 + nr0 * D4;
#pragma unroll
            for (int u = 0; u < NGW; ++u)
#pragma unroll
                for (int q = 0; q < 4; ++q) SLAQ_FUSED_LOAD(u, q, ntb, nlim)
            yr = y[nr0 + li < N ? nr0 + li : N - 1];
        }
        __builtin_amdgcn_sched_barrier(0);

        // forward: the wave's share of Z
        floatx4 zacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < NGW; ++u)
#pragma unroll
            for (int sidx = 0; sidx < 4; ++sidx) {
                const int st = 4 * (NW * u + wave) + sidx;
                if (16 * st < D) {
                    const f4 xa = *reinterpret_cast<const f4 *>(Xs + lc * LD + 16 * st + 4 * lg);
                    zacc = mfma16(xa.x, wreg[u][sidx].x, zacc);
                    zacc = mfma16(xa.y, wreg[u][sidx].y, zacc);
                    zacc = mfma16(xa.z, wreg[u][sidx].z, zacc);
                    zacc = mfma16(xa.w, wreg[u][sidx].w, zacc);
                }
            }
        // lane (model lc, lg) holds Z[4 lg + r][lc]
        *reinterpret_cast<f4 *>(zs + (wave * kFusedM + lc) * kFusedZld + 4 * lg) = f4{zacc[0], zacc[1], zacc[2], zacc[3]};
        __syncthreads();

        // loss and residual: thread (model lj, row li); the waves' shares are added in wave order
        if (tid < kFusedM * kFusedRows) {
            const float *zp = zs + lj * kFusedZld + li;
            float z = zp[0];
#pragma unroll
            for (int w = 1; w < NW; ++w) z = z + zp[w * kFusedM * kFusedZld];
            float l, r;
            loss_residual(loss, z, yc, l, r);
            const bool valid = tile * kFusedRows + li < N;
            l = valid ? l : 0.0f;
            r = valid ? r : 0.0f;
            lsum = lsum + l;
            rs[lj * kFusedZld + li] = r;
        }
        __syncthreads();

        // backward: the wave's column groups
        {
            const f4 av = *reinterpret_cast<const f4 *>(rs + lc * kFusedZld + 4 * lg);
#pragma unroll
            for (int u = 0; u < NGW; ++u) {
                const int grp = NW * u + wave;
                if (64 * grp < D) {
                    // two rows of the group in flight at a time: all four at once cost the registers that
                    // the next tile's slots need
                    const float *xb = Xs + (4 * lg) * LD + 64 * grp + 4 * lc;
                    f4 b0 = *reinterpret_cast<const f4 *>(xb);
                    f4 b1 = *reinterpret_cast<const f4 *>(xb + LD);
                    __builtin_amdgcn_sched_barrier(0);
                    acc[u][0] = mfma16(av.x, b0.x, acc[u][0]); acc[u][1] = mfma16(av.x, b0.y, acc[u][1]);
                    acc[u][2] = mfma16(av.x, b0.z, acc[u][2]); acc[u][3] = mfma16(av.x, b0.w, acc[u][3]);
                    b0 = *reinterpret_cast<const f4 *>(xb + 2 * LD);
                    __builtin_amdgcn_sched_barrier(0);
                    acc[u][0] = mfma16(av.y, b1.x, acc[u][0]); acc[u][1] = mfma16(av.y, b1.y, acc[u][1]);
                    acc[u][2] = mfma16(av.y, b1.z, acc[u][2]); acc[u][3] = mfma16(av.y, b1.w, acc[u][3]);
                    b1 = *reinterpret_cast<const f4 *>(xb + 3 * LD);
                    __builtin_amdgcn_sched_barrier(0);
                    acc[u][0] = mfma16(av.z, b0.x, acc[u][0]); acc[u][1] = mfma16(av.z, b0.y, acc[u][1]);
                    acc[u][2] = mfma16(av.z, b0.z, acc[u][2]); acc[u][3] = mfma16(av.z, b0.w, acc[u][3]);
                    acc[u][0] = mfma16(av.w, b1.x, acc[u][0]); acc[u][1] = mfma16(av.w, b1.y, acc[u][1]);
                    acc[u][2] = mfma16(av.w, b1.z, acc[u][2]); acc[u][3] = mfma16(av.w, b1.w, acc[u][3]);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
    }
#undef SLAQ_FUSED_LOAD
#undef SLAQ_FUSED_STASH

    // the block's partial gradient: lane (dd = lc, lg) holds models 4 lg + r, columns 64 grp + 4 dd + t
    float *__restrict__ gp = Gpart + (size_t)blockIdx.x * kFusedM * D;
#pragma unroll
    for (int u = 0; u < NGW; ++u) {
        const int grp = NW * u + wave;
        const int col = 64 * grp + 4 * lc;
        if (col < D) {
#pragma unroll
            for (int r = 0; r < 4; ++r)
                *reinterpret_cast<f4 *>(gp + (size_t)(4 * lg + r) * D + col) =
                    f4{acc[u][0][r], acc[u][1][r], acc[u][2][r], acc[u][3][r]};
        }
    }
    // the block's loss sums: rows in order for every model
    __syncthreads();                                    // the last tile's partial Z has been read
    if (tid < kFusedM * kFusedRows) zs[lj * kFusedZld + li] = lsum;
    __syncthreads();
    if (tid < M) {
        float sacc = zs[tid * kFusedZld];
#pragma unroll
        for (int i = 1; i < kFusedRows; ++i) sacc = sacc + zs[tid * kFusedZld + i];
        lossP[(size_t)tid * gridDim.x + blockIdx.x] = sacc;
    }
}

// One block per model: column sums of the S partials, update, loss.
__global__ __launch_bounds__(1024) void sweep_finalize_kernel(
    const float *__restrict__ Gpart, const float *__restrict__ lossP, int S, int T, long long N,
    int D, int M, size_t gstride, const float *__restrict__ lambdas, const float *__restrict__ steps,
    float *__restrict__ W, float *__restrict__ G, float *__restrict__ loss_row) {
    __shared__ double red[1024];
    __shared__ double red2[32];
    const int m = blockIdx.x;
    const int tid = threadIdx.x;
    const double invN = 1.0 / (double)N;
    const double lam = (double)lambdas[m];
    const double eta = (double)steps[m];

    double ww = 0.0;
    for (int d = tid; d < D; d += 1024) {
        const float *__restrict__ gp = Gpart + (size_t)m * D + d;
        double tot = 0.0;
        int sidx = 0;
        for (; sidx + 16 <= S; sidx += 16) {
            float v[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) v[u] = gp[(size_t)(sidx + u) * gstride];
#pragma unroll
            for (int u = 0; u < 16; ++u) tot += (double)v[u];
        }
        for (; sidx < S; ++sidx) tot += (double)gp[(size_t)sidx * gstride];
        const float wj = W[(size_t)m * D + d];
        const double g = tot * invN + lam * (double)wj;
        ww += (double)wj * (double)wj;
        G[(size_t)m * D + d] = (float)g;
        if (eta != 0.0) W[(size_t)m * D + d] = (float)((double)wj - eta * g);
    }
    // loss: thread t adds a contiguous run of the model's tile partials
    double ls = 0.0;
    {
        const int t0 = (int)((long long)T * tid / 1024);
        const int t1 = (int)((long long)T * (tid + 1) / 1024);
        const float *__restrict__ lp = lossP + (size_t)m * T;
        for (int t = t0; t < t1; ++t) ls += (double)lp[t];
    }
    // two fixed-order block sums (|w|^2, then loss)
    double out[2];
    for (int which = 0; which < 2; ++which) {
        red[tid] = which == 0 ? ww : ls;
        __syncthreads();
        if (tid < 32) {
            double a = 0.0;
            for (int q = 0; q < 32; ++q) a += red[tid * 32 + q];
            red2[tid] = a;
        }
        __syncthreads();
        double a = 0.0;
        if (tid == 0) for (int q = 0; q < 32; ++q) a += red2[q];
        out[which] = a;
        __syncthreads();
    }
    if (tid == 0) loss_row[m] = (float)(out[1] * invN + 0.5 * lam * out[0]);
}

// A group of at most 16 models with a row length the one-pass kernel takes.
bool sweep_uses_fused(int D, int M) { return M <= kFusedM && D <= 1024 && (D % 16) == 0; }

// Blocks of the one-pass kernel = partial gradients and loss sums per model: a function of the shape
// only, so the order of all additions is fixed by the shape.  As many as the chip holds at once of the
// instantiation that takes the row length (one 16-wave block per compute unit for the longest rows,
// two 8-wave blocks, four 4-wave blocks), and no more than there are tiles.
int sweep_fused_blocks(long long N, int D) {
    const long long tiles = (N + kFusedRows - 1) / kFusedRows;
    const int cap = D > 512 ? kSweepFusedBlocksMax / 4 : D > 256 ? kSweepFusedBlocksMax / 2 : kSweepFusedBlocksMax;
    return (int)std::min<long long>(tiles, cap);
}

static hipError_t launch_sweep_fused(const SweepArgs &a, hipEvent_t *ev, hipStream_t st) {
    hipError_t e;
    const int G = sweep_fused_blocks(a.N, a.D);
    if (ev && (e = hipEventRecord(ev[0], st)) != hipSuccess) return e;
#define SLAQ_FUSED_LAUNCH(DMAX)                                                                              \
    {                                                                                                        \
        static bool attr_set[64];               /* per device: the kernel may use more than 64 KB of LDS */  \
        int dev = 0;                                                                                         \
        if ((e = hipGetDevice(&dev)) != hipSuccess) return e;                                                \
        if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;                                              \
        if (!attr_set[dev]) {                                                                                \
            if ((e = hipFuncSetAttribute(reinterpret_cast<const void *>(&sweep_fused_kernel<DMAX>),          \
                                         hipFuncAttributeMaxDynamicSharedMemorySize,                         \
                                         (int)sweep_fused_lds_bytes(DMAX, DMAX))) != hipSuccess)             \
                return e;                                                                                    \
            attr_set[dev] = true;                                                                            \
        }                                                                                                    \
        hipLaunchKernelGGL(sweep_fused_kernel<DMAX>, dim3((unsigned)G), dim3(64 * fused_waves(DMAX)),        \
                           sweep_fused_lds_bytes(a.D, DMAX), st, a.X, a.y, a.W, a.N, a.D, a.M, a.loss,       \
                           a.Gpart, a.lossP);                                                                \
    }
    if (a.D <= 256) SLAQ_FUSED_LAUNCH(256)
    else if (a.D <= 512) SLAQ_FUSED_LAUNCH(512)
    else SLAQ_FUSED_LAUNCH(1024)
#undef SLAQ_FUSED_LAUNCH
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (ev) {       // the one kernel stands where the forward kernel stands; an empty interval for the backward one
        if ((e = hipEventRecord(ev[1], st)) != hipSuccess) return e;
        if ((e = hipEventRecord(ev[2], st)) != hipSuccess) return e;
        if ((e = hipEventRecord(ev[3], st)) != hipSuccess) return e;
    }
    hipLaunchKernelGGL(sweep_finalize_kernel, dim3((unsigned)a.M), dim3(1024), 0, st, a.Gpart, a.lossP, G, G, a.N,
                       a.D, a.M, (size_t)kFusedM * a.D, a.lambdas, a.steps, a.W, a.G, a.loss_row);
    return hipGetLastError();
}

hipError_t launch_sweep_iteration(const SweepArgs &a, int k, hipEvent_t *ev, hipStream_t st) {
    hipError_t e;
    if (sweep_uses_fused(a.D, a.M)) return launch_sweep_fused(a, ev, st);
    if (ev && (e = hipEventRecord(ev[0], st)) != hipSuccess) return e;
    const bool half = a.M <= 32;
    // the plain variant: no ragged last K-chunk and a tile full of models
    const bool plain = (a.D % kFwdK) == 0 && a.M == (half ? 32 : kSweepM);
#define SLAQ_FWD_LAUNCH(H, P)                                                                \
    hipLaunchKernelGGL((sweep_forward_kernel<H, P>), dim3((unsigned)a.T), dim3(256), 0, st, a.X, a.y, a.W, a.N, a.D, \
                       a.M, a.loss, a.R, a.lossP, a.T)
    if (half) { if (plain) SLAQ_FWD_LAUNCH(true, true); else SLAQ_FWD_LAUNCH(true, false); }
    else { if (plain) SLAQ_FWD_LAUNCH(false, true); else SLAQ_FWD_LAUNCH(false, false); }
#undef SLAQ_FWD_LAUNCH
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (ev && (e = hipEventRecord(ev[1], st)) != hipSuccess) return e;
    if (ev && (e = hipEventRecord(ev[2], st)) != hipSuccess) return e;
    const int nslab = (a.D + kBwdCols - 1) / kBwdCols;
    if (half)
        hipLaunchKernelGGL(sweep_backward_kernel<true>, dim3((unsigned)(nslab * a.S)), dim3(256), 0, st, a.X,
                           a.R, a.N, a.D, a.S, a.Gpart);
    else
        hipLaunchKernelGGL(sweep_backward_kernel<false>, dim3((unsigned)(nslab * a.S)), dim3(256), 0, st, a.X,
                           a.R, a.N, a.D, a.S, a.Gpart);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (ev && (e = hipEventRecord(ev[3], st)) != hipSuccess) return e;
    hipLaunchKernelGGL(sweep_finalize_kernel, dim3((unsigned)a.M), dim3(1024), 0, st, a.Gpart,
                       a.lossP, a.S, a.T, a.N, a.D, a.M, (size_t)kSweepM * a.D, a.lambdas, a.steps, a.W, a.G,
                       a.loss_row);
    (void)k;
    return hipGetLastError();
}

}  // namespace slaqglm
