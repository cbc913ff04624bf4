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

// One block per model: column sums of the S partials, update, loss.
__global__ __launch_bounds__(1024) void sweep_finalize_kernel(
    const float *__restrict__ Gpart, const float *__restrict__ lossP, int S, int T, long long N,
    int D, int M, const float *__restrict__ lambdas, const float *__restrict__ steps,
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
            for (int u = 0; u < 16; ++u) v[u] = gp[(size_t)(sidx + u) * kSweepM * D];
#pragma unroll
            for (int u = 0; u < 16; ++u) tot += (double)v[u];
        }
        for (; sidx < S; ++sidx) tot += (double)gp[(size_t)sidx * kSweepM * D];
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

hipError_t launch_sweep_iteration(const SweepArgs &a, int k, hipEvent_t *ev, hipStream_t st) {
    hipError_t e;
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
                       a.lossP, a.S, a.T, a.N, a.D, a.M, a.lambdas, a.steps, a.W, a.G, a.loss_row);
    (void)k;
    return hipGetLastError();
}

}  // namespace slaqglm
