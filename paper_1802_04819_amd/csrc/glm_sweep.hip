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

template <bool HALF>
__global__ __launch_bounds__(256) void sweep_forward_kernel(
    const float *__restrict__ X, const float *__restrict__ y, const float *__restrict__ W,
    long long N, int D, int M, int loss, float *__restrict__ R, float *__restrict__ lossP, int T) {
    __shared__ f4 Xs4[kFwdRows * kFwdLd / 4];
    __shared__ f4 Ws4[kSweepM * kFwdLd / 4];
    __shared__ float lsm[4][kSweepM];
    float *Xs = reinterpret_cast<float *>(Xs4);
    float *Ws = reinterpret_cast<float *>(Ws4);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 31, lh = lane >> 5;
    const int tile = blockIdx.x;
    const long long r0 = (long long)tile * kFwdRows;
    const int D4 = D >> 2;
    const f4 *__restrict__ X4 = reinterpret_cast<const f4 *>(X);
    const f4 *__restrict__ W4 = reinterpret_cast<const f4 *>(W);

    // staging assignments: X chunk = 128 rows x 8 f4, W chunk = 64 rows x 8 f4
    constexpr int WQ = HALF ? 1 : 2;          // W rows staged per thread: 32 or 64 models
    constexpr int RS = HALF ? 32 : kSweepM;   // row stride of R
    long long xrow[4]; int xc4[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int idx = tid + 256 * q;
        long long r = r0 + (idx >> 3);
        xrow[q] = (r < N ? r : N - 1) * D4;
        xc4[q] = idx & 7;
    }
    int wrow[WQ], wc4[WQ]; float wmask[WQ];   // models past M read row 0 and are multiplied by 0
#pragma unroll
    for (int q = 0; q < WQ; ++q) {
        const int idx = tid + 256 * q;
        const int m = idx >> 3;
        wmask[q] = m < M ? 1.0f : 0.0f;
        wrow[q] = (m < M ? m : 0) * D4;
        wc4[q] = idx & 7;
    }

    floatx16 acc0 = {0}, acc1 = {0};
    const int nchunk = (D + kFwdK - 1) / kFwdK;
    // A chunk is 8 float4 slots of k; slots past the row length (last chunk of a D that is not a
    // multiple of 32) read a clamped slot and are multiplied by 0 on both operands.
#define SLAQ_FWD_FETCH(KC)                                                                   \
    {                                                                                        \
        const int kc_ = (KC);                                                                \
        _Pragma("unroll") for (int q = 0; q < 4; ++q) {                                      \
            const int c_ = kc_ * (kFwdK / 4) + xc4[q];                                       \
            xk[q] = c_ < D4 ? 1.0f : 0.0f;                                                   \
            xr[q] = __builtin_nontemporal_load(X4 + xrow[q] + (c_ < D4 ? c_ : D4 - 1));      \
        }                                                                                    \
        _Pragma("unroll") for (int q = 0; q < WQ; ++q) {                                     \
            const int c_ = kc_ * (kFwdK / 4) + wc4[q];                                       \
            wk[q] = c_ < D4 ? wmask[q] : 0.0f;                                               \
            wr[q] = W4[wrow[q] + (c_ < D4 ? c_ : D4 - 1)];                                   \
        }                                                                                    \
    }
#define SLAQ_FWD_STASH()                                                                     \
    {                                                                                        \
        _Pragma("unroll") for (int q = 0; q < 4; ++q) {                                      \
            const int idx = tid + 256 * q;                                                   \
            Xs4[(idx >> 3) * (kFwdLd / 4) + (idx & 7)] = full_k ? xr[q] : xr[q] * xk[q];     \
        }                                                                                    \
        _Pragma("unroll") for (int q = 0; q < WQ; ++q) {                                     \
            const int idx = tid + 256 * q;                                                   \
            Ws4[(idx >> 3) * (kFwdLd / 4) + (idx & 7)] = wr[q] * wk[q];                      \
        }                                                                                    \
    }
    const bool full_k = (D % kFwdK) == 0;     // then X is staged as it is (also its infinities and NaNs)

    {
        f4 xr[4], wr[WQ];
        float xk[4], wk[WQ];
        SLAQ_FWD_FETCH(0)
        SLAQ_FWD_STASH()
    }
    __syncthreads();
    for (int kc = 0; kc < nchunk; ++kc) {
        f4 xr[4], wr[WQ];
        float xk[4], wk[WQ];
        SLAQ_FWD_FETCH(kc + 1 < nchunk ? kc + 1 : kc)   // last trip re-reads its own chunk (cache hit)
        __builtin_amdgcn_sched_barrier(0);              // keep the prefetch ahead of the matrix ops
        const f4 *arow = Xs4 + (wave * 32 + li) * (kFwdLd / 4) + lh;
        const f4 *b0row = Ws4 + li * (kFwdLd / 4) + lh;
        const f4 *b1row = Ws4 + (32 + li) * (kFwdLd / 4) + lh;
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
        SLAQ_FWD_STASH()
        __syncthreads();
    }
#undef SLAQ_FWD_FETCH
#undef SLAQ_FWD_STASH
    (void)Xs; (void)Ws;

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
#define SLAQ_BWD_FETCH(CH)                                                                   \
    {                                                                                        \
        const long long rbase = (CH) * kBwdRows;                                             \
        _Pragma("unroll") for (int q = 0; q < 8; ++q) {                                      \
            const int idx = tid + 256 * q;         /* row = idx / 64, f4 column = idx % 64 */ \
            long long row = rbase + (idx >> 6);                                              \
            row = row < N ? row : N - 1;                                                     \
            int c4 = slab * (kBwdCols / 4) + (idx & 63);   /* slab columns past D read a valid */ \
            c4 = c4 < D4 ? c4 : D4 - 1;                    /* slot; their sums are never stored */ \
            xr[q] = __builtin_nontemporal_load(X4 + row * D4 + c4);                          \
        }                                                                                    \
        _Pragma("unroll") for (int q = 0; q < RQ; ++q) {                                     \
            const int idx = tid + 256 * q;         /* row = idx / (RS/4), f4 model = idx % (RS/4) */ \
            const long long row = rbase + idx / (RS / 4);                                    \
            rkeep[q] = row < N ? 1.0f : 0.0f;              /* rows past N add nothing */      \
            rr[q] = R4[(row < N ? row : N - 1) * (RS / 4) + idx % (RS / 4)];                 \
        }                                                                                    \
    }
#define SLAQ_BWD_STASH()                                                                     \
    {                                                                                        \
        _Pragma("unroll") for (int q = 0; q < 8; ++q) Xs4[tid + 256 * q] = xr[q];            \
        _Pragma("unroll") for (int q = 0; q < RQ; ++q) Rs4[tid + 256 * q] = rr[q] * rkeep[q]; \
    }

    long long c = s;
    if (c < nchunks) {
        f4 xr[8], rr[RQ];
        float rkeep[RQ];
        SLAQ_BWD_FETCH(c)
        SLAQ_BWD_STASH()
    }
    __syncthreads();
    for (; c < nchunks; c += S) {
        f4 xr[8], rr[RQ];
        float rkeep[RQ];
        SLAQ_BWD_FETCH(c + S < nchunks ? c + S : c)     // last trip re-reads its own chunk
        __builtin_amdgcn_sched_barrier(0);              // keep the prefetch ahead of the matrix ops
        const float *xa = Xs + lh * kBwdCols + wave * 64 + li;
        const float *ra = Rs + lh * RS + li;
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
    if (half)
        hipLaunchKernelGGL(sweep_forward_kernel<true>, dim3((unsigned)a.T), dim3(256), 0, st, a.X, a.y, a.W,
                           a.N, a.D, a.M, a.loss, a.R, a.lossP, a.T);
    else
        hipLaunchKernelGGL(sweep_forward_kernel<false>, dim3((unsigned)a.T), dim3(256), 0, st, a.X, a.y, a.W,
                           a.N, a.D, a.M, a.loss, a.R, a.lossP, a.T);
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
