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
//
// A trip is two steps: tile_load brings the rows and labels into registers, tile_compute does
// everything else.  The resident kernel loads once and computes once per iteration.
template <int B> struct TileQ {
    static constexpr int QB = B < 4 ? B : 4;
    static constexpr int NBATCH = B / QB;
    static_assert(B % QB == 0, "wave-loads per trip must be a multiple of the loss batch");
};

template <int LPR, int C, int B, bool FULL>
__device__ __forceinline__ void tile_load(gmem_f4 X4, gmem_f yv, const long long D4, const long long N,
                                          const long long row0, const int (&fidx)[C], const int lane,
                                          f4 (&xv)[B][C], float (&ysel)[TileQ<B>::NBATCH],
                                          long long (&rsel)[TileQ<B>::NBATCH]) {
    constexpr int RPL = 64 / LPR;
    constexpr int QB = TileQ<B>::QB;
    const int ql = lane & (QB - 1);
#pragma unroll
    for (int b = 0; b < B; ++b) {
        long long row = row0 + (long long)b * RPL;
        if constexpr (!FULL) row = row < N ? row : (N - 1);
        gmem_f4 base = X4 + row * D4;
#pragma unroll
        for (int c = 0; c < C; ++c) xv[b][c] = __builtin_nontemporal_load(base + fidx[c]);
    }
#pragma unroll
    for (int q = 0; q < TileQ<B>::NBATCH; ++q) {
        rsel[q] = row0 + (long long)(QB * q + ql) * RPL;
        long long rc = rsel[q];
        if constexpr (!FULL) rc = rc < N ? rc : (N - 1);
        ysel[q] = __builtin_nontemporal_load(yv + rc);
    }
}

template <int LPR, int C, int B, int LOSS, bool FULL>
__device__ __forceinline__ void tile_compute(const f4 (&xv)[B][C], const float (&ysel)[TileQ<B>::NBATCH],
                                             const long long (&rsel)[TileQ<B>::NBATCH], const long long N,
                                             const f4 (&wv)[C], f4 (&ga)[C], float &lsum, const int lane) {
    constexpr int QB = TileQ<B>::QB;
    const int ql = lane & (QB - 1);
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

    loss_batches<C, B, QB, LOSS, FULL>(std::make_integer_sequence<int, TileQ<B>::NBATCH>{}, xv, z, ysel, rsel, N,
                                       ql, ga, lsum);
}

template <int LPR, int C, int B, int LOSS, bool FULL>
__device__ __forceinline__ void process_tile(gmem_f4 X4, gmem_f yv, const long long D4,
                                             const long long N, const long long row0,
                                             const int (&fidx)[C], const f4 (&wv)[C], f4 (&ga)[C],
                                             float &lsum, const int lane) {
    f4 xv[B][C];
    float ysel[TileQ<B>::NBATCH];
    long long rsel[TileQ<B>::NBATCH];
    tile_load<LPR, C, B, FULL>(X4, yv, D4, N, row0, fidx, lane, xv, ysel, rsel);
    tile_compute<LPR, C, B, LOSS, FULL>(xv, ysel, rsel, N, wv, ga, lsum, lane);
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

// The weights of the lane's slots and zeroed accumulators.  Slots beyond the real row length read a
// clamped (valid) slot and get weight 0, so they add nothing to the margin; their accumulators are
// never written out.  One wave of the job (`forms_wn2`; the first wave of row block 0 outside the
// resident kernel) also forms |w|^2 of the entering iterate, for the L2 term of the loss.
template <int LPR, int C>
__device__ __forceinline__ void row_setup(const DevJob &jb, const bool forms_wn2, const int lane,
                                          int (&fidx)[C], f4 (&wv)[C], f4 (&ga)[C]) {
    const int sub = lane & (LPR - 1);
    const int rgrp = (LPR == 64) ? 0 : (lane / LPR);
    const int D4 = jb.D >> 2;
#pragma unroll
    for (int c = 0; c < C; ++c) {
        const int f = c * LPR + sub;
        const bool ok = f < D4;
        fidx[c] = ok ? f : (D4 - 1);
        const f4 t = reinterpret_cast<const f4 *>(jb.w)[fidx[c]];
        wv[c] = ok ? t : f4{0.f, 0.f, 0.f, 0.f};
        ga[c] = f4{0.f, 0.f, 0.f, 0.f};
    }
    if (forms_wn2) {
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
}

// A value with an iteration tag above it: the unit of exchange between the blocks of the resident kernel.
__device__ __forceinline__ unsigned long long tagged_word(const float v, const unsigned tag) {
    return ((unsigned long long)tag << 32) | (unsigned long long)__float_as_uint(v);
}

// Block reduction in a fixed order: (wave 0, group 0), (wave 0, group 1), ... (wave 3, last); the
// block's partial gradient row and partial loss go to gp[0 .. D) and *lp.  Loss sums live in the
// first QB lanes of each group (each carries different rows).  TAGGED (resident kernel): gp and lp
// point at 64-bit words and every value is stored with `tag` above it, device-coherently.
template <int LPR, int C, int B, bool TAGGED>
__device__ __forceinline__ void row_reduce_store(const f4 (&ga)[C], const float lsum, const int D, float *gp,
                                                 float *lp, float *gred, float *lred, const int wid,
                                                 const int lane, const unsigned tag = 0u) {
    constexpr int RPL = 64 / LPR;
    constexpr int DP = 4 * LPR * C;
    constexpr int QB = TileQ<B>::QB;
    const int sub = lane & (LPR - 1);
    const int rgrp = (LPR == 64) ? 0 : (lane / LPR);
    f4 *gred4 = reinterpret_cast<f4 *>(gred);
    const int slot = wid * RPL + rgrp;
#pragma unroll
    for (int c = 0; c < C; ++c) gred4[slot * (DP / 4) + c * LPR + sub] = ga[c];
    if (sub < QB) lred[slot * QB + sub] = lsum;
    __syncthreads();
    for (int j = threadIdx.x; j < D; j += kRowBlockThreads) {
        float s = gred[j];
#pragma unroll
        for (int q = 1; q < 4 * RPL; ++q) s = s + gred[q * DP + j];       // loads together, additions in order
        if constexpr (TAGGED)
            __hip_atomic_store(reinterpret_cast<unsigned long long *>(gp) + j, tagged_word(s, tag), __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
        else gp[j] = s;
    }
    if (threadIdx.x == 0) {
        float s = lred[0];
#pragma unroll
        for (int q = 1; q < 4 * RPL * QB; ++q) s = s + lred[q];
        if constexpr (TAGGED)
            __hip_atomic_store(reinterpret_cast<unsigned long long *>(lp), tagged_word(s, tag), __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
        else *lp = s;
    }
}

template <int LPR, int C, int B>
__device__ __forceinline__ void row_pass_body(const DevJob &jb, const int vb, float *gred,
                                              float *lred) {
    const int lane = threadIdx.x & 63;
    const int wid = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int rgrp = (LPR == 64) ? 0 : (lane / LPR);
    int fidx[C];
    f4 wv[C], ga[C];
    row_setup<LPR, C>(jb, vb == 0 && wid == 0, lane, fidx, wv, ga);
    float lsum = 0.0f;

    if (jb.loss == GLM_LOGISTIC)
        row_loop<LPR, C, B, GLM_LOGISTIC>(jb, vb, wid, rgrp, fidx, wv, ga, lsum, lane);
    else if (jb.loss == GLM_HINGE)
        row_loop<LPR, C, B, GLM_HINGE>(jb, vb, wid, rgrp, fidx, wv, ga, lsum, lane);
    else
        row_loop<LPR, C, B, GLM_SQUARED>(jb, vb, wid, rgrp, fidx, wv, ga, lsum, lane);

    row_reduce_store<LPR, C, B, false>(ga, lsum, jb.D, jb.gpart + (size_t)vb * jb.D, jb.lpart + vb, gred, lred,
                                       wid, lane);
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

// The arithmetic of the finalize step, shared by the stand-alone kernel and the resident kernel so
// that both form every sum in the same order.

// Sum over row blocks [p0, p1) of one column of the partial gradients, index order, fp64.
__device__ __forceinline__ double column_segment_sum(const float *gp, const int D, const int p0, const int p1) {
    double s = 0.0;
    int p = p0;
    for (; p + 16 <= p1; p += 16) {          // 16 loads in flight, added in index order
        float v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) v[u] = gp[(size_t)(p + u) * D];
#pragma unroll
        for (int u = 0; u < 16; ++u) s += (double)v[u];
    }
    for (; p < p1; ++p) s += (double)gp[(size_t)p * D];
    return s;
}

__device__ __forceinline__ int fin_seg_begin(const int P, const int seg) { return (int)((long long)P * seg / kFinSegs); }

// Loss partial of "thread" t of kFinCols * kFinSegs: a contiguous run of row blocks.
__device__ __forceinline__ double loss_run_sum(const float *lpart, const int P, const int t) {
    constexpr int T = kFinCols * kFinSegs;
    const int p0 = (int)((long long)P * t / T);
    const int p1 = (int)((long long)P * (t + 1) / T);
    double ls = 0.0;
    for (int p = p0; p < p1; ++p) ls += (double)lpart[p];
    return ls;
}

// Gradient entry and updated weight of one column from the column's total over all row blocks.
__device__ __forceinline__ void column_update(const DevJob &jb, const int round, const double tot, const float wj,
                                              float &g_out, float &w_out) {
    const double g = tot * jb.invN + (double)jb.lambda * (double)wj;
    g_out = (float)g;
    w_out = wj;
    if (jb.step != 0.0f) {
        double eta = (double)jb.step;
        if (jb.sched == GLM_STEP_INV_SQRT) eta = eta / sqrt((double)(jb.k0 + round + 1));
        w_out = (float)((double)wj - eta * g);
    }
}

__device__ __forceinline__ double loss_value(const DevJob &jb, const double S, const double wn2) {
    return S * jb.invN + 0.5 * (double)jb.lambda * wn2;
}

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
    if (col < D) s = column_segment_sum(jb.gpart + col, D, fin_seg_begin(P, seg), fin_seg_begin(P, seg + 1));
    sred[seg][cl] = s;

    // loss sum (first column block of the job only): thread t adds a contiguous run of blocks
    const bool does_loss = (cb == 0);
    if (does_loss) lred[tid] = loss_run_sum(jb.lpart, P, tid);
    __syncthreads();

    if (seg == 0 && col < D) {
        double c[4];                        // four runs of 16 segments each, then (c0 + c1) + (c2 + c3)
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            c[k] = sred[16 * k][cl];
#pragma unroll
            for (int q = 1; q < 16; ++q) c[k] += sred[16 * k + q][cl];
        }
        const double tot = (c[0] + c[1]) + (c[2] + c[3]);
        float g, wn;
        column_update(jb, round, tot, jb.w[col], g, wn);
        jb.grad[col] = g;
        if (jb.step != 0.0f) jb.w[col] = wn;
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
            const double L = loss_value(jb, S, *jb.wn2);
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

// ------------------------------------------------------------------ resident kernel (tiny jobs)

// For a job so small that an iteration is nothing but launch and dependency latency, the whole
// call runs in ONE launch: the job's P row blocks stay resident and loop over the iterations.
// Every wave has at most one tile of rows (that is part of what makes a job tiny) and keeps it in
// registers for the whole call.  Per iteration: the row pass of the block on that tile (same
// arithmetic as above; the weights come from the block's own copy in LDS), one barrier among the
// job's blocks, then EVERY block copies all partials of the job into LDS and forms the complete
// finalize step for itself (same order of additions as finalize_body), so it owns the next weights
// without a second barrier; partials alternate between two buffers, so a block that is still
// reading iteration k's cannot be overtaken by iteration k+2's writes.  The last block writes the
// loss history, block 0 after the last iteration the gradient and the weights.
//
// Exchange of the partials.  A barrier with a cache-wide release/acquire pair costs 10 us and more
// with 64 blocks on this part (each acquire drops the L2 of its XCD), and even a counter barrier
// built from device-coherent accesses puts four dependent trips to memory between a block's last
// store and its first load.  So there is no barrier: every partial travels as one 64-bit word
// {iteration tag, value}, written with a device-coherent relaxed atomic store; a reader loads the
// words it needs with device-coherent relaxed atomic loads and loads a word again until its tag is
// the tag of the iteration it is in.  A word is stored and loaded whole, so a matching tag
// guarantees its value.  Tags are r + 1; a kernel of its own clears both buffers to tag 0 before the
// launch.  Why two buffers suffice: a block writes iteration r + 2 only after it has read every
// block's iteration r + 1 word, which each block writes only after it has finished reading
// iteration r.
//
// All P blocks must be on the chip at once: the launcher only takes this path when P fits the
// device's capacity for this kernel.  Every wait is bounded: after kResidentSpinLimit reloads a
// thread gives up and sets the job's `failed` flag, which every other waiting thread sees at its next
// reload; the remaining history entries are then filled with NaN.
constexpr unsigned kResidentSpinLimit = 1u << 22;

struct ResidentCtl { unsigned failed; unsigned pad; };

// Total of one column over all row blocks, in the order of finalize_body: each of the 64 segments
// added up from zero in index order; four runs of 16 consecutive segments, each run added up in
// segment order starting from its first segment; then (c0 + c1) + (c2 + c3).  The values come from
// LDS (row block p at base[p * stride]), sixteen loads in flight.
static_assert(kFinSegs == 64, "the combine below is written for 64 segments");
// Run k (segments 16 k .. 16 k + 15) of a column when no segment holds more than one row block
// (P <= kFinSegs): the sixteen loads first, then the sums in segment order.
__device__ __forceinline__ double column_run_sparse(const float *base, const int stride, const int P, const int k) {
    float v[16];
    bool has[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
        const int seg = 16 * k + u;
        const int p0 = (P * seg) / kFinSegs, p1 = (P * (seg + 1)) / kFinSegs;
        has[u] = p1 > p0;
        v[u] = base[(size_t)(has[u] ? p0 : 0) * stride];
    }
    double c = 0.0;
#pragma unroll
    for (int u = 0; u < 16; ++u) {
        const double s = has[u] ? 0.0 + (double)v[u] : 0.0;     // a segment starts from zero
        c = u == 0 ? s : c + s;
    }
    return c;
}

__device__ __forceinline__ double column_total(const float *base, const int stride, const int P) {
    double c[4] = {0.0, 0.0, 0.0, 0.0};
    if (P <= kFinSegs) {                        // no segment holds more than one row block
#pragma unroll
        for (int k = 0; k < 4; ++k) c[k] = column_run_sparse(base, stride, P, k);
        return (c[0] + c[1]) + (c[2] + c[3]);
    }
    double s = 0.0;
    int seg = 0, seg_end = fin_seg_begin(P, 1);
    auto close = [&]() {                        // segment `seg` is complete (it may be empty)
        const int k = seg >> 4;
        const double upd = (seg & 15) == 0 ? s : c[k] + s;
        c[0] = k == 0 ? upd : c[0]; c[1] = k == 1 ? upd : c[1]; c[2] = k == 2 ? upd : c[2]; c[3] = k == 3 ? upd : c[3];
        s = 0.0; ++seg; seg_end = fin_seg_begin(P, seg + 1);
    };
    for (int p = 0; p < P; p += 16) {
        float v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) v[u] = base[(size_t)(p + u < P ? p + u : P - 1) * stride];
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            if (p + u < P) {
                while (p + u == seg_end) close();
                s += (double)v[u];
            }
        }
    }
    while (seg < kFinSegs) close();
    return (c[0] + c[1]) + (c[2] + c[3]);
}

constexpr int kResidentStage = kResidentMaxPartials + 1032;    // partial gradients + partial losses of a tiny job

// Words of the exchange a thread requests before it waits for any of them: 17 x 256 threads cover the
// 8256 words of a 64-block, 128-column job in two rounds of loads instead of three.
constexpr int kResidentInFlight = 17;

template <int LPR, int C, int B, int LOSS>
__device__ __forceinline__ void resident_iterations(const DevJob &jb0, float *gred, float *lred, float *w_lds,
                                                    double *wn2_lds, float *stage, double *lsum2, int *abandoned) {
    constexpr int RPL = 64 / LPR;
    constexpr long long RT = (long long)B * RPL;
    constexpr int T = kFinCols * kFinSegs;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wid = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int sub = lane & (LPR - 1);
    const int rgrp = (LPR == 64) ? 0 : (lane / LPR);
    const int vb = blockIdx.x;
    const int D = jb0.D, P = jb0.P, D4 = jb0.D >> 2;
    const long long N = jb0.N;
    ResidentCtl *ctl = reinterpret_cast<ResidentCtl *>(jb0.ctl);
    const int lossb = P - 1;                        // the block that forms the loss; block 0 writes the results

    // the wave's tile of rows, loaded once (rows past the end read a clamped row and are masked later)
    const long long t = (long long)vb * 4 + wid;
    const bool has_tile = t * RT < N;
    int fidx[C];
#pragma unroll
    for (int c = 0; c < C; ++c) { const int f = c * LPR + sub; fidx[c] = f < D4 ? f : (D4 - 1); }
    f4 xv[B][C];
    float ysel[TileQ<B>::NBATCH];
    long long rsel[TileQ<B>::NBATCH];
    if (has_tile)
        tile_load<LPR, C, B, false>((gmem_f4)(uintptr_t)jb0.X, (gmem_f)(uintptr_t)jb0.y, D4, N, t * RT + rgrp, fidx,
                                    lane, xv, ysel, rsel);

    DevJob jb = jb0;
    jb.w = w_lds;                                   // flat pointers into LDS
    jb.wn2 = wn2_lds;
    const int n_words = P * D + P;                  // one buffer: [P, D] gradients, then [P] losses, a word each
    for (int r = 0; r < jb0.iters; ++r) {
        unsigned long long *buf = reinterpret_cast<unsigned long long *>((r & 1) ? jb0.gpart2 : jb0.gpart);
        const unsigned tag = (unsigned)r + 1u;
        f4 wv[C], ga[C];
        row_setup<LPR, C>(jb, vb == lossb && wid == 0, lane, fidx, wv, ga);
        float lsum = 0.0f;
        if (has_tile) tile_compute<LPR, C, B, LOSS, false>(xv, ysel, rsel, N, wv, ga, lsum, lane);
        row_reduce_store<LPR, C, B, true>(ga, lsum, D, reinterpret_cast<float *>(buf + (size_t)vb * D),
                                          reinterpret_cast<float *>(buf + (size_t)P * D + vb), gred, lred, wid, lane, tag);
        // every partial of the job into LDS: kResidentInFlight words in flight per thread, each loaded again until
        // it carries this iteration's tag
        bool gave_up = false;
        for (int i = tid; i < n_words; i += kResidentInFlight * kRowBlockThreads) {
            unsigned long long v[kResidentInFlight];
#pragma unroll
            for (int u = 0; u < kResidentInFlight; ++u) {
                const int k = i + u * kRowBlockThreads;
                v[u] = k < n_words ? __hip_atomic_load(buf + k, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                                   : ((unsigned long long)tag << 32);
            }
            unsigned spins = 0;
            while (true) {
                bool all = true;
#pragma unroll
                for (int u = 0; u < kResidentInFlight; ++u) {
                    if ((unsigned)(v[u] >> 32) != tag) {
                        v[u] = __hip_atomic_load(buf + i + u * kRowBlockThreads, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        all = false;
                    }
                }
                if (all) break;
                if (++spins > kResidentSpinLimit ||
                    __hip_atomic_load(&ctl->failed, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) {
                    __hip_atomic_store(&ctl->failed, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    gave_up = true;
                    break;
                }
            }
#pragma unroll
            for (int u = 0; u < kResidentInFlight; ++u) {
                const int k = i + u * kRowBlockThreads;
                if (k < n_words) stage[k] = __uint_as_float((unsigned)v[u]);
            }
        }
        if (gave_up) *abandoned = 1;
        __syncthreads();
        if (*abandoned) {                           // written before the barrier by whoever gave up: one way for all
            if (vb == lossb)
                for (int k = r + tid; k < jb0.iters; k += kRowBlockThreads) jb0.loss_out[k] = __builtin_nanf("");
            return;
        }
        // finalize, complete, in every block: one thread per column, from thread 0 upwards.  The last
        // block also forms the loss as finalize_body does (1024 runs of row blocks, 32 sums of 32 runs,
        // their sum): its last 32 threads take one sum each while the others work on the columns.  With
        // at most 1024 row blocks a run holds one row block or none.
        const bool last = r == jb0.iters - 1;
        if (vb == lossb && tid >= kRowBlockThreads - 32) {
            // Sum t32 covers the runs [32 t32, 32 t32 + 32); run v holds row block floor(P v / T) if the
            // next run starts at a later one, else nothing, so the non-empty runs of the sum hold the
            // row blocks [P 32 t32 / T, P 32 (t32 + 1) / T) in order.  The empty runs add +0.0 to a sum
            // that is never -0.0 (it starts at +0.0 and every term is 0.0 + x): leaving them out
            // gives the same bits.
            const int t32 = tid - (kRowBlockThreads - 32);
            const float *lp = stage + (size_t)P * D;
            const int pa = (P * (T / 32) * t32) / T, pb = (P * (T / 32) * (t32 + 1)) / T;
            double S = 0.0;
            for (int pq = pa; pq < pb; ++pq) S += 0.0 + (double)lp[pq];
            lsum2[t32] = S;
        }
        if (P <= kFinSegs) {
            // four neighbouring lanes per column, one run of sixteen segments each; their sums meet as
            // (c0 + c1) + (c2 + c3), the order of column_total (4 D is a multiple of four, so the four
            // lanes of a column take every trip of this loop together)
            for (int q = tid; q < 4 * D; q += kRowBlockThreads) {
                const int col = q >> 2, k = q & 3;
                const double ck = column_run_sparse(stage + col, D, P, k);
                const double pair = ck + __shfl_xor(ck, 1, 64);          // c0 + c1 in lanes 0, 1; c2 + c3 in lanes 2, 3
                const double other = __shfl_xor(pair, 2, 64);
                if (k == 0) {
                    const double tot = pair + other;
                    float g, wn;
                    column_update(jb0, r, tot, w_lds[col], g, wn);
                    w_lds[col] = wn;            // read again by the next row pass, after the barrier below
                    if (vb == 0 && last) { jb0.grad[col] = g; jb0.w[col] = wn; }
                }
            }
        } else {
            for (int col = tid; col < D; col += kRowBlockThreads) {
                const double tot = column_total(stage + col, D, P);
                float g, wn;
                column_update(jb0, r, tot, w_lds[col], g, wn);
                w_lds[col] = wn;                // read again by the next row pass, after the barrier below
                if (vb == 0 && last) { jb0.grad[col] = g; jb0.w[col] = wn; }
            }
        }
        __syncthreads();
        if (vb == lossb && tid == kRowBlockThreads - 1) {
            double part[32];
#pragma unroll
            for (int q = 0; q < 32; ++q) part[q] = lsum2[q];
            double S = 0.0;
#pragma unroll
            for (int q = 0; q < 32; ++q) S += part[q];
            const double L = loss_value(jb0, S, *wn2_lds);
            jb0.loss_out[r] = (float)L;
            if (jb0.loss64 && last) *jb0.loss64 = L;
        }
    }
}

template <int CLS>
__global__ __launch_bounds__(kRowBlockThreads) void resident_kernel(const DevJob jb0) {
    constexpr ClassInfo ci = class_info(CLS);
    __shared__ float4 gred4[4 * 64 * ci.c];
    __shared__ float lred[256];
    __shared__ __align__(16) float w_lds[4 * 64 * ci.c];       // the block's copy of the weights (padded row)
    __shared__ double wn2_lds[1];
    __shared__ double lsum2[32];
    __shared__ __align__(16) float stage[kResidentStage];
    __shared__ int abandoned;
    if (threadIdx.x == 0) abandoned = 0;
    for (int j = threadIdx.x; j < jb0.D; j += kRowBlockThreads) w_lds[j] = jb0.w[j];
    __syncthreads();
    float *gred = reinterpret_cast<float *>(gred4);
    if (jb0.loss == GLM_LOGISTIC)
        resident_iterations<ci.lpr, ci.c, ci.b, GLM_LOGISTIC>(jb0, gred, lred, w_lds, wn2_lds, stage, lsum2, &abandoned);
    else if (jb0.loss == GLM_HINGE)
        resident_iterations<ci.lpr, ci.c, ci.b, GLM_HINGE>(jb0, gred, lred, w_lds, wn2_lds, stage, lsum2, &abandoned);
    else
        resident_iterations<ci.lpr, ci.c, ci.b, GLM_SQUARED>(jb0, gred, lred, w_lds, wn2_lds, stage, lsum2, &abandoned);
}

// Tag 0 in every word of both buffers, and the failure flag down.
__global__ __launch_bounds__(256) void resident_clear_kernel(unsigned long long *a, unsigned long long *b, int n_words,
                                                             ResidentCtl *ctl) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n_words) { a[i] = 0ull; b[i] = 0ull; }
    if (i == 0) { ctl->failed = 0u; ctl->pad = 0u; }
}

// Blocks of resident_kernel<cls> that the current device holds at once (0 on error).
int resident_capacity(int cls) {
    static int cap[64][kNumClasses];            // per device; 0 = not asked yet, -1 = asked and failed
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
    if (cap[dev][cls] == 0) {
        int per_cu = 0, cus = 0;
        hipError_t e = hipErrorInvalidValue;
        switch (cls) {
#define SLAQ_CASE(K) case K: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, resident_kernel<K>, kRowBlockThreads, 0); break;
            SLAQ_CASE(0) SLAQ_CASE(1) SLAQ_CASE(2) SLAQ_CASE(3) SLAQ_CASE(4)
            SLAQ_CASE(5) SLAQ_CASE(6) SLAQ_CASE(7) SLAQ_CASE(8)
#undef SLAQ_CASE
            default: break;
        }
        if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        cap[dev][cls] = (e == hipSuccess && per_cu > 0 && cus > 0) ? per_cu * cus : -1;
    }
    return cap[dev][cls] > 0 ? cap[dev][cls] : 0;
}

hipError_t launch_resident(const DevJob &jb, hipStream_t st) {
    const int n_words = jb.P * jb.D + jb.P;
    hipLaunchKernelGGL(resident_clear_kernel, dim3((unsigned)((n_words + 255) / 256)), dim3(256), 0, st,
                       reinterpret_cast<unsigned long long *>(jb.gpart), reinterpret_cast<unsigned long long *>(jb.gpart2),
                       n_words, reinterpret_cast<ResidentCtl *>(jb.ctl));
    dim3 grid((unsigned)jb.P), block(kRowBlockThreads);
    switch (jb.cls) {
#define SLAQ_CASE(K) case K: hipLaunchKernelGGL(resident_kernel<K>, grid, block, 0, st, jb); break;
        SLAQ_CASE(0) SLAQ_CASE(1) SLAQ_CASE(2) SLAQ_CASE(3) SLAQ_CASE(4)
        SLAQ_CASE(5) SLAQ_CASE(6) SLAQ_CASE(7) SLAQ_CASE(8)
#undef SLAQ_CASE
        default: return hipErrorInvalidValue;
    }
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
