// Row pass and finalize kernels of the GLM iteration for gfx950 (wave64).
//
// Row pass: streams X once.  A wave covers 64/LPR rows side by side with LPR lanes per row,
// each lane holding C float4 slots of the row, of w and of the gradient accumulator in
// registers.  Per row: lane-partial dot products -> all-reduce inside the lane group ->
// every lane has the margin -> per-sample loss and residual -> the X values still in
// registers are multiplied by the residual into the accumulators.  X never goes through LDS;
// LDS is used once per block, at the end, to add the accumulators of the block's lane groups
// in a fixed order.  Each block writes one partial gradient row and one partial loss.
//
// Finalize: adds the per-block partials in a fixed order in fp64, applies 1/N and the L2
// term, writes the gradient, the loss-history entry and the updated weights.
//
// Floating point is written with explicit fma calls and compiled with contraction off, so the
// sequence of roundings is fixed by the source and is the same in every kernel variant.
#include <utility>

#include "glm_internal.h"
#include "glm_loss.h"

namespace slaqglm {

// ------------------------------------------------------------------ lane-group reductions

// First-class 4-float vector: 128-bit loads that stay in registers.
typedef float f4 __attribute__((ext_vector_type(4)));

// X and y are read exactly once per iteration and never again before they have left every
// cache, so they are loaded with the non-temporal hint.  On this part that alone raises the
// attainable streaming rate from about 6.3 to about 7.1 TB/s.
__device__ __forceinline__ f4 stream_load(const f4 *p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ float stream_load(const float *p) { return __builtin_nontemporal_load(p); }

template <int CTRL, int ROWMASK>
__device__ __forceinline__ float dpp_take(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(
        0, __builtin_bit_cast(int, v), CTRL, ROWMASK, 0xF, false));
}

// Sum of v over the LPR-lane group the lane belongs to, delivered to every lane of the group.
// Groups are aligned runs of LPR lanes.  All lanes of a group obtain the same bits.
template <int LPR>
__device__ __forceinline__ float group_allreduce(float v, int lane) {
    if constexpr (LPR >= 2) v = v + dpp_take<0xB1, 0xF>(v);    // quad_perm [1,0,3,2]
    if constexpr (LPR >= 4) v = v + dpp_take<0x4E, 0xF>(v);    // quad_perm [2,3,0,1]
    if constexpr (LPR >= 8) v = v + dpp_take<0x141, 0xF>(v);   // row_half_mirror
    if constexpr (LPR >= 16) v = v + dpp_take<0x140, 0xF>(v);  // row_mirror
    if constexpr (LPR == 32) {
        int o = __builtin_amdgcn_ds_bpermute((lane ^ 16) << 2, __builtin_bit_cast(int, v));
        v = v + __builtin_bit_cast(float, o);
    }
    if constexpr (LPR == 64) {
        v = v + dpp_take<0x142, 0xA>(v);                       // row_bcast15 into rows 1, 3
        v = v + dpp_take<0x143, 0xC>(v);                       // row_bcast31 into rows 2, 3
        v = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
    }
    return v;
}

__device__ __forceinline__ double wave_sum_f64(double v) {
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// ------------------------------------------------------------------ row pass

// Pointers into device memory arrive inside a table, where the compiler cannot see their
// address space; naming it makes the loads global_load (not flat_load) instructions.
typedef const f4 __attribute__((address_space(1))) *gmem_f4;
typedef const float __attribute__((address_space(1))) *gmem_f;

template <int J>
__device__ __forceinline__ float quad_bcast(float v) {      // value of lane J of the lane's quad
    return dpp_take<J * 0x55, 0xF>(v);
}

template <int LOSS>
__device__ __forceinline__ void loss_residual_t(float z, float y, float &l, float &r) {
    if constexpr (LOSS == GLM_LOGISTIC) logistic_lr(z, y, l, r);
    else if constexpr (LOSS == GLM_HINGE) hinge_lr(z, y, l, r);
    else squared_lr(z, y, l, r);
}

// Loss, residual and accumulation for the rows of loss batch Q (wave-loads QB*Q .. QB*Q+QB-1).
// Q is a template argument so that every array index below is a constant in the source.
template <int C, int B, int QB, int LOSS, bool FULL, int Q>
__device__ __forceinline__ void loss_batch(const f4 (&xv)[B][C], const float (&z)[B],
                                           const float ys, const long long rs, const long long N,
                                           const int ql, f4 (&ga)[C], float &lsum) {
    float zs = z[QB * Q];
    if constexpr (QB >= 2) {
        const float z1 = z[QB * Q + 1];
        zs = (ql & 1) ? z1 : zs;
    }
    if constexpr (QB == 4) {
        const float z2 = z[QB * Q + 2], z3 = z[QB * Q + 3];
        const float zhi = (ql & 1) ? z3 : z2;
        zs = (ql & 2) ? zhi : zs;
    }
    float l, r;
    loss_residual_t<LOSS>(zs, ys, l, r);
    if constexpr (!FULL) {
        const bool valid = rs < N;
        l = valid ? l : 0.0f;
        r = valid ? r : 0.0f;
    }
    lsum = lsum + l;
    const float r0 = QB == 1 ? r : quad_bcast<0>(r);
#pragma unroll
    for (int c = 0; c < C; ++c) {
        ga[c].x = __builtin_fmaf(xv[QB * Q][c].x, r0, ga[c].x);
        ga[c].y = __builtin_fmaf(xv[QB * Q][c].y, r0, ga[c].y);
        ga[c].z = __builtin_fmaf(xv[QB * Q][c].z, r0, ga[c].z);
        ga[c].w = __builtin_fmaf(xv[QB * Q][c].w, r0, ga[c].w);
    }
    if constexpr (QB >= 2) {
        const float r1 = quad_bcast<1>(r);
#pragma unroll
        for (int c = 0; c < C; ++c) {
            ga[c].x = __builtin_fmaf(xv[QB * Q + 1][c].x, r1, ga[c].x);
            ga[c].y = __builtin_fmaf(xv[QB * Q + 1][c].y, r1, ga[c].y);
            ga[c].z = __builtin_fmaf(xv[QB * Q + 1][c].z, r1, ga[c].z);
            ga[c].w = __builtin_fmaf(xv[QB * Q + 1][c].w, r1, ga[c].w);
        }
    }
    if constexpr (QB == 4) {
        const float r2 = quad_bcast<2>(r);
#pragma unroll
        for (int c = 0; c < C; ++c) {
            ga[c].x = __builtin_fmaf(xv[QB * Q + 2][c].x, r2, ga[c].x);
            ga[c].y = __builtin_fmaf(xv[QB * Q + 2][c].y, r2, ga[c].y);
            ga[c].z = __builtin_fmaf(xv[QB * Q + 2][c].z, r2, ga[c].z);
            ga[c].w = __builtin_fmaf(xv[QB * Q + 2][c].w, r2, ga[c].w);
        }
        const float r3 = quad_bcast<3>(r);
#pragma unroll
        for (int c = 0; c < C; ++c) {
            ga[c].x = __builtin_fmaf(xv[QB * Q + 3][c].x, r3, ga[c].x);
            ga[c].y = __builtin_fmaf(xv[QB * Q + 3][c].y, r3, ga[c].y);
            ga[c].z = __builtin_fmaf(xv[QB * Q + 3][c].z, r3, ga[c].z);
            ga[c].w = __builtin_fmaf(xv[QB * Q + 3][c].w, r3, ga[c].w);
        }
    }
}

template <int C, int B, int QB, int LOSS, bool FULL, int... Qs, int NB>
__device__ __forceinline__ void loss_batches(std::integer_sequence<int, Qs...>, const f4 (&xv)[B][C],
                                             const float (&z)[B], const float (&ysel)[NB],
                                             const long long (&rsel)[NB], const long long N,
                                             const int ql, f4 (&ga)[C], float &lsum) {
    (loss_batch<C, B, QB, LOSS, FULL, Qs>(xv, z, ysel[Qs], rsel[Qs], N, ql, ga, lsum), ...);
}

// One loop trip of one wave: B wave-loads (B * 64/LPR rows).  FULL = every row of the trip
// exists (no clamping, no masking); the last trip of a job takes the other variant.
//
// The loss is not evaluated by every lane for every row: within each quad, lane q evaluates
// the row of wave-load 4*batch + q (QB = min(B, 4) rows per batch) and the residual is then
// handed to the other lanes with quad_perm broadcasts, so the transcendental work is done
// once per QB rows instead of once per row.
template <int LPR, int C, int B, int LOSS, bool FULL>
__device__ __forceinline__ void process_tile(gmem_f4 X4, gmem_f yv, const long long D4,
                                             const long long N, const long long row0,
                                             const int (&fidx)[C], const f4 (&wv)[C], f4 (&ga)[C],
                                             float &lsum, const int lane) {
    constexpr int RPL = 64 / LPR;
    constexpr int QB = B < 4 ? B : 4;
    constexpr int NBATCH = B / QB;
    static_assert(B % QB == 0, "wave-loads per trip must be a multiple of the loss batch");
    const int ql = lane & (QB - 1);

    f4 xv[B][C];
#pragma unroll
    for (int b = 0; b < B; ++b) {
        long long row = row0 + (long long)b * RPL;
        if constexpr (!FULL) row = row < N ? row : (N - 1);
        gmem_f4 base = X4 + row * D4;
#pragma unroll
        for (int c = 0; c < C; ++c) xv[b][c] = __builtin_nontemporal_load(base + fidx[c]);
    }
    float ysel[NBATCH];
    long long rsel[NBATCH];
#pragma unroll
    for (int q = 0; q < NBATCH; ++q) {
        rsel[q] = row0 + (long long)(QB * q + ql) * RPL;
        long long rc = rsel[q];
        if constexpr (!FULL) rc = rc < N ? rc : (N - 1);
        ysel[q] = __builtin_nontemporal_load(yv + rc);
    }

    float z[B];
#pragma unroll
    for (int b = 0; b < B; ++b) {
        float p = xv[b][0].x * wv[0].x;
        p = __builtin_fmaf(xv[b][0].y, wv[0].y, p);
        p = __builtin_fmaf(xv[b][0].z, wv[0].z, p);
        p = __builtin_fmaf(xv[b][0].w, wv[0].w, p);
#pragma unroll
        for (int c = 1; c < C; ++c) {
            p = __builtin_fmaf(xv[b][c].x, wv[c].x, p);
            p = __builtin_fmaf(xv[b][c].y, wv[c].y, p);
            p = __builtin_fmaf(xv[b][c].z, wv[c].z, p);
            p = __builtin_fmaf(xv[b][c].w, wv[c].w, p);
        }
        z[b] = p;
    }
#pragma unroll
    for (int b = 0; b < B; ++b) z[b] = group_allreduce<LPR>(z[b], lane);

    loss_batches<C, B, QB, LOSS, FULL>(std::make_integer_sequence<int, NBATCH>{}, xv, z, ysel, rsel, N,
                                       ql, ga, lsum);
}

template <int LPR, int C, int B, int LOSS>
__device__ __forceinline__ void row_loop(const DevJob &jb, const int vb, const int wid,
                                         const int rgrp, const int (&fidx)[C], const f4 (&wv)[C],
                                         f4 (&ga)[C], float &lsum, const int lane) {
    constexpr int RPL = 64 / LPR;
    constexpr long long RT = (long long)B * RPL;       // rows per wave per loop trip
    const long long N = jb.N;
    const long long D4 = jb.D >> 2;
    gmem_f4 X4 = (gmem_f4)(uintptr_t)jb.X;
    gmem_f yv = (gmem_f)(uintptr_t)jb.y;
    const long long TW = (long long)jb.P * 4;          // waves of this job
    // Trips whose rows all exist, then (for one wave of the job) the ragged last trip.
    long long t = (long long)vb * 4 + wid;
    for (; (t + 1) * RT <= N; t += TW)
        process_tile<LPR, C, B, LOSS, true>(X4, yv, D4, N, t * RT + rgrp, fidx, wv, ga, lsum, lane);
    if (t * RT < N)
        process_tile<LPR, C, B, LOSS, false>(X4, yv, D4, N, t * RT + rgrp, fidx, wv, ga, lsum, lane);
}

template <int LPR, int C, int B>
__device__ __forceinline__ void row_pass_body(const DevJob &jb, const int vb, float *gred,
                                              float *lred) {
    constexpr int RPL = 64 / LPR;          // rows side by side in one wave-load
    constexpr int DP = 4 * LPR * C;        // padded row length covered by the lane layout
    constexpr int QB = B < 4 ? B : 4;      // lanes of a group that carry loss sums
    const int lane = threadIdx.x & 63;
    const int wid = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int sub = lane & (LPR - 1);
    const int rgrp = (LPR == 64) ? 0 : (lane / LPR);
    const int D4 = jb.D >> 2;

    // Slots beyond the real row length read a clamped (valid) slot and get weight 0, so they
    // add nothing to the margin; their accumulators are never written out.
    int fidx[C];
    f4 wv[C], ga[C];
#pragma unroll
    for (int c = 0; c < C; ++c) {
        const int f = c * LPR + sub;
        const bool ok = f < D4;
        fidx[c] = ok ? f : (D4 - 1);
        const f4 t = reinterpret_cast<const f4 *>(jb.w)[fidx[c]];
        wv[c] = ok ? t : f4{0.f, 0.f, 0.f, 0.f};
        ga[c] = f4{0.f, 0.f, 0.f, 0.f};
    }
    float lsum = 0.0f;

    if (vb == 0 && wid == 0) {   // |w|^2 of the entering iterate, for the L2 term of the loss
        double ww = 0.0;
        if (rgrp == 0) {
#pragma unroll
            for (int c = 0; c < C; ++c) {
                ww += (double)wv[c].x * wv[c].x;
                ww += (double)wv[c].y * wv[c].y;
                ww += (double)wv[c].z * wv[c].z;
                ww += (double)wv[c].w * wv[c].w;
            }
        }
        ww = wave_sum_f64(ww);
        if (lane == 0) *jb.wn2 = ww;
    }

    if (jb.loss == GLM_LOGISTIC)
        row_loop<LPR, C, B, GLM_LOGISTIC>(jb, vb, wid, rgrp, fidx, wv, ga, lsum, lane);
    else if (jb.loss == GLM_HINGE)
        row_loop<LPR, C, B, GLM_HINGE>(jb, vb, wid, rgrp, fidx, wv, ga, lsum, lane);
    else
        row_loop<LPR, C, B, GLM_SQUARED>(jb, vb, wid, rgrp, fidx, wv, ga, lsum, lane);

    // Block reduction in a fixed order: (wave 0, group 0), (wave 0, group 1), ... (wave 3, last).
    // Loss sums live in the first QB lanes of each group (each carries different rows).
    f4 *gred4 = reinterpret_cast<f4 *>(gred);
    const int slot = wid * RPL + rgrp;
#pragma unroll
    for (int c = 0; c < C; ++c) gred4[slot * (DP / 4) + c * LPR + sub] = ga[c];
    if (sub < QB) lred[slot * QB + sub] = lsum;
    __syncthreads();
    const int D = jb.D;
    float *__restrict__ gp = jb.gpart + (size_t)vb * D;
    for (int j = threadIdx.x; j < D; j += kRowBlockThreads) {
        float s = gred[j];
#pragma unroll 4
        for (int q = 1; q < 4 * RPL; ++q) s = s + gred[q * DP + j];
        gp[j] = s;
    }
    if (threadIdx.x == 0) {
        float s = lred[0];
        for (int q = 1; q < 4 * RPL * QB; ++q) s = s + lred[q];
        jb.lpart[vb] = s;
    }
}

// Index a such that tab[a] <= x < tab[a+1]; tab has n+1 increasing entries, tab[0] = 0.
__device__ __forceinline__ int find_segment(const int *__restrict__ tab, int n, int x) {
    int lo = 0, hi = n;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (tab[mid] <= x) lo = mid; else hi = mid;
    }
    return lo;
}

template <int MAXCLS>
__global__ __launch_bounds__(kRowBlockThreads) void row_pass_kernel(
    const DevJob *__restrict__ jobs, const int *__restrict__ blk_job) {
    constexpr int CMAX = class_info(MAXCLS).c;
    __shared__ float4 gred4[4 * 64 * CMAX];
    __shared__ float lred[256];
    float *gred = reinterpret_cast<float *>(gred4);
    const DevJob &jb = jobs[blk_job[blockIdx.x]];      // block -> job: one table entry per block
    const int vb = blockIdx.x - jb.blk0;
    switch (jb.cls) {
#define SLAQ_CASE(K)                                                                          \
    case K:                                                                                   \
        if constexpr (K <= MAXCLS)                                                            \
            row_pass_body<class_info(K).lpr, class_info(K).c, class_info(K).b>(jb, vb, gred,  \
                                                                               lred);         \
        break;
        SLAQ_CASE(0) SLAQ_CASE(1) SLAQ_CASE(2) SLAQ_CASE(3) SLAQ_CASE(4)
        SLAQ_CASE(5) SLAQ_CASE(6) SLAQ_CASE(7) SLAQ_CASE(8)
#undef SLAQ_CASE
        default: break;
    }
}

hipError_t launch_row_pass(const DevJob *jobs, const int *blk_job, int total_blocks,
                           int max_cls, hipStream_t st) {
    if (total_blocks <= 0) return hipSuccess;
    dim3 grid((unsigned)total_blocks), block(kRowBlockThreads);
    if (max_cls <= 4) hipLaunchKernelGGL(row_pass_kernel<4>, grid, block, 0, st, jobs, blk_job);
    else if (max_cls == 5) hipLaunchKernelGGL(row_pass_kernel<5>, grid, block, 0, st, jobs, blk_job);
    else if (max_cls == 6) hipLaunchKernelGGL(row_pass_kernel<6>, grid, block, 0, st, jobs, blk_job);
    else if (max_cls == 7) hipLaunchKernelGGL(row_pass_kernel<7>, grid, block, 0, st, jobs, blk_job);
    else hipLaunchKernelGGL(row_pass_kernel<8>, grid, block, 0, st, jobs, blk_job);
    return hipGetLastError();
}

// One job, handed over by value in the kernel arguments: no table in device memory, block b is
// row block b.  Same body as above, so the job's sums are formed in the same order.
template <int CLS>
__global__ __launch_bounds__(kRowBlockThreads) void row_pass_one_kernel(const DevJob jb) {
    constexpr ClassInfo ci = class_info(CLS);
    __shared__ float4 gred4[4 * 64 * ci.c];
    __shared__ float lred[256];
    row_pass_body<ci.lpr, ci.c, ci.b>(jb, (int)blockIdx.x, reinterpret_cast<float *>(gred4), lred);
}

hipError_t launch_row_pass_one(const DevJob &jb, hipStream_t st) {
    dim3 grid((unsigned)jb.P), block(kRowBlockThreads);
    switch (jb.cls) {
#define SLAQ_CASE(K) case K: hipLaunchKernelGGL(row_pass_one_kernel<K>, grid, block, 0, st, jb); break;
        SLAQ_CASE(0) SLAQ_CASE(1) SLAQ_CASE(2) SLAQ_CASE(3) SLAQ_CASE(4)
        SLAQ_CASE(5) SLAQ_CASE(6) SLAQ_CASE(7) SLAQ_CASE(8)
#undef SLAQ_CASE
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------ finalize

// Column block cb (kFinCols columns) of one job; the job's first column block also forms the loss.
__device__ __forceinline__ void finalize_body(const DevJob &jb, const int cb, const int round) {
    constexpr int T = kFinCols * kFinSegs;
    __shared__ double sred[kFinSegs][kFinCols];
    __shared__ double lred[T];
    __shared__ double lred2[32];
    const int tid = threadIdx.x;
    const int cl = tid & (kFinCols - 1);
    const int seg = tid / kFinCols;
    const int D = jb.D, P = jb.P;
    const int col = cb * kFinCols + cl;

    // column sums: segment `seg` adds row blocks [P*seg/S, P*(seg+1)/S) in index order
    double s = 0.0;
    if (col < D) {
        const int p0 = (int)((long long)P * seg / kFinSegs);
        const int p1 = (int)((long long)P * (seg + 1) / kFinSegs);
        const float *__restrict__ gp = jb.gpart + col;
        int p = p0;
        for (; p + 16 <= p1; p += 16) {          // 16 loads in flight, added in index order
            float v[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) v[u] = gp[(size_t)(p + u) * D];
#pragma unroll
            for (int u = 0; u < 16; ++u) s += (double)v[u];
        }
        for (; p < p1; ++p) s += (double)gp[(size_t)p * D];
    }
    sred[seg][cl] = s;

    // loss sum (first column block of the job only): thread t adds a contiguous run of blocks
    const bool does_loss = (cb == 0);
    if (does_loss) {
        const int p0 = (int)((long long)P * tid / T);
        const int p1 = (int)((long long)P * (tid + 1) / T);
        double ls = 0.0;
        for (int p = p0; p < p1; ++p) ls += (double)jb.lpart[p];
        lred[tid] = ls;
    }
    __syncthreads();

    if (seg == 0 && col < D) {
        double tot = sred[0][cl];
#pragma unroll 8
        for (int q = 1; q < kFinSegs; ++q) tot += sred[q][cl];
        const float wj = jb.w[col];
        const double g = tot * jb.invN + (double)jb.lambda * (double)wj;
        jb.grad[col] = (float)g;
        if (jb.step != 0.0f) {
            double eta = (double)jb.step;
            if (jb.sched == GLM_STEP_INV_SQRT) eta = eta / sqrt((double)(jb.k0 + round + 1));
            jb.w[col] = (float)((double)wj - eta * g);
        }
    }
    if (does_loss) {                       // fixed two-level sum of the T thread partials
        if (tid < 32) {
            double S = 0.0;
            for (int q = 0; q < T / 32; ++q) S += lred[tid * (T / 32) + q];
            lred2[tid] = S;
        }
        __syncthreads();
        if (tid == 0) {
            double S = 0.0;
            for (int q = 0; q < 32; ++q) S += lred2[q];
            const double L = S * jb.invN + 0.5 * (double)jb.lambda * (*jb.wn2);
            jb.loss_out[round] = (float)L;
            if (jb.loss64) *jb.loss64 = L;
        }
    }
}

__global__ __launch_bounds__(kFinCols * kFinSegs) void finalize_kernel(
    const DevJob *__restrict__ jobs, const int *__restrict__ cblk0, int nact, int round) {
    const int a = find_segment(cblk0, nact, blockIdx.x);
    finalize_body(jobs[a], (int)blockIdx.x - cblk0[a], round);
}

__global__ __launch_bounds__(kFinCols * kFinSegs) void finalize_one_kernel(const DevJob jb, int round) {
    finalize_body(jb, (int)blockIdx.x, round);
}

hipError_t launch_finalize_one(const DevJob &jb, int round, hipStream_t st) {
    hipLaunchKernelGGL(finalize_one_kernel, dim3((unsigned)((jb.D + kFinCols - 1) / kFinCols)),
                       dim3(kFinCols * kFinSegs), 0, st, jb, round);
    return hipGetLastError();
}

hipError_t launch_finalize(const DevJob *jobs, const int *cblk0, int nact, int total_blocks,
                           int round, hipStream_t st) {
    if (total_blocks <= 0) return hipSuccess;
    hipLaunchKernelGGL(finalize_kernel, dim3((unsigned)total_blocks), dim3(kFinCols * kFinSegs), 0,
                       st, jobs, cblk0, nact, round);
    return hipGetLastError();
}

// ------------------------------------------------------------------ streaming-read probe

__global__ __launch_bounds__(256) void read_probe_kernel(const f4 *__restrict__ src, size_t n4,
                                                         float *__restrict__ sink) {
    __shared__ float red[4];
    float acc = 0.0f;
    // a block reads one contiguous span, as a block of the row pass reads its rows
    const size_t span = (n4 + gridDim.x - 1) / gridDim.x;
    const size_t b0 = (size_t)blockIdx.x * span;
    const size_t b1 = b0 + span < n4 ? b0 + span : n4;
    size_t i = b0 + threadIdx.x;
    for (; i + 7 * 256 < b1; i += 8 * 256) {
        f4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = stream_load(src + i + u * 256);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += (v[u].x + v[u].y) + (v[u].z + v[u].w);
    }
    for (; i < b1; i += 256) {
        const f4 v = stream_load(src + i);
        acc += (v.x + v.y) + (v.z + v.w);
    }
    // a short tail: the probe is a ceiling only if nothing but the loads takes time
    for (int o = 32; o >= 1; o >>= 1) acc += __shfl_xor(acc, o, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) sink[blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
}

hipError_t launch_read_probe(const float *src, size_t n, float *sink, hipStream_t st) {
    hipLaunchKernelGGL(read_probe_kernel, dim3(kProbeBlocks), dim3(256), 0, st,
                       reinterpret_cast<const f4 *>(src), n / 4, sink);
    return hipGetLastError();
}

}  // namespace slaqglm
