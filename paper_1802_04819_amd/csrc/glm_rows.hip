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
#include "glm_internal.h"
#include "glm_loss.h"

namespace slaqglm {

// ------------------------------------------------------------------ lane-group reductions

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

template <int LPR, int C, int B>
__device__ __forceinline__ void row_pass_body(const DevJob &jb, const int vb, float *gred,
                                              float *lred) {
    constexpr int RPL = 64 / LPR;          // rows side by side in one wave-load
    constexpr int DP = 4 * LPR * C;        // padded row length covered by the lane layout
    const int lane = threadIdx.x & 63;
    const int wid = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int sub = lane & (LPR - 1);
    const int rgrp = (LPR == 64) ? 0 : (lane / LPR);
    const int D4 = jb.D >> 2;
    const long long N = jb.N;
    const float4 *__restrict__ X4 = reinterpret_cast<const float4 *>(jb.X);
    const float *__restrict__ yv = jb.y;
    const int loss = jb.loss;

    // Slots beyond the real row length read a clamped (valid) slot and get weight 0, so they
    // add nothing to the margin; their accumulators are never written out.
    int fidx[C];
    float4 wv[C], ga[C];
#pragma unroll
    for (int c = 0; c < C; ++c) {
        const int f = c * LPR + sub;
        const bool ok = f < D4;
        fidx[c] = ok ? f : (D4 - 1);
        const float4 t = reinterpret_cast<const float4 *>(jb.w)[fidx[c]];
        wv[c] = ok ? t : make_float4(0.f, 0.f, 0.f, 0.f);
        ga[c] = make_float4(0.f, 0.f, 0.f, 0.f);
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

    constexpr long long RT = (long long)B * RPL;       // rows per wave per loop trip
    const long long TW = (long long)jb.P * 4;          // waves of this job
    for (long long t = (long long)vb * 4 + wid; t * RT < N; t += TW) {
        const long long row0 = t * RT + rgrp;
        float4 xv[B][C];
        float yy[B];
#pragma unroll
        for (int b = 0; b < B; ++b) {
            long long row = row0 + (long long)b * RPL;
            row = row < N ? row : (N - 1);
            const float4 *__restrict__ base = X4 + row * D4;
#pragma unroll
            for (int c = 0; c < C; ++c) xv[b][c] = base[fidx[c]];
            yy[b] = yv[row];
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
#pragma unroll
        for (int b = 0; b < B; ++b) {
            float l, r;
            if (loss == GLM_LOGISTIC) logistic_lr(z[b], yy[b], l, r);
            else if (loss == GLM_HINGE) hinge_lr(z[b], yy[b], l, r);
            else squared_lr(z[b], yy[b], l, r);
            const bool valid = (row0 + (long long)b * RPL) < N;
            l = valid ? l : 0.0f;
            r = valid ? r : 0.0f;
            lsum = lsum + l;
#pragma unroll
            for (int c = 0; c < C; ++c) {
                ga[c].x = __builtin_fmaf(xv[b][c].x, r, ga[c].x);
                ga[c].y = __builtin_fmaf(xv[b][c].y, r, ga[c].y);
                ga[c].z = __builtin_fmaf(xv[b][c].z, r, ga[c].z);
                ga[c].w = __builtin_fmaf(xv[b][c].w, r, ga[c].w);
            }
        }
    }

    // Block reduction in a fixed order: (wave 0, group 0), (wave 0, group 1), ... (wave 3, last).
    float4 *gred4 = reinterpret_cast<float4 *>(gred);
    const int slot = wid * RPL + rgrp;
#pragma unroll
    for (int c = 0; c < C; ++c) gred4[slot * (DP / 4) + c * LPR + sub] = ga[c];
    if (sub == 0) lred[slot] = lsum;
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
        for (int q = 1; q < 4 * RPL; ++q) s = s + lred[q];
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
    const DevJob *__restrict__ jobs, const int *__restrict__ blk0, int nact) {
    constexpr int CMAX = class_info(MAXCLS).c;
    __shared__ float4 gred4[4 * 64 * CMAX];
    __shared__ float lred[64];
    float *gred = reinterpret_cast<float *>(gred4);
    const int a = find_segment(blk0, nact, blockIdx.x);
    const DevJob &jb = jobs[a];
    const int vb = blockIdx.x - blk0[a];
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

hipError_t launch_row_pass(const DevJob *jobs, const int *blk0, int nact, int total_blocks,
                           int max_cls, hipStream_t st) {
    if (total_blocks <= 0) return hipSuccess;
    dim3 grid((unsigned)total_blocks), block(kRowBlockThreads);
    if (max_cls <= 4) hipLaunchKernelGGL(row_pass_kernel<4>, grid, block, 0, st, jobs, blk0, nact);
    else if (max_cls == 5) hipLaunchKernelGGL(row_pass_kernel<5>, grid, block, 0, st, jobs, blk0, nact);
    else if (max_cls == 6) hipLaunchKernelGGL(row_pass_kernel<6>, grid, block, 0, st, jobs, blk0, nact);
    else if (max_cls == 7) hipLaunchKernelGGL(row_pass_kernel<7>, grid, block, 0, st, jobs, blk0, nact);
    else hipLaunchKernelGGL(row_pass_kernel<8>, grid, block, 0, st, jobs, blk0, nact);
    return hipGetLastError();
}

// ------------------------------------------------------------------ finalize

__global__ __launch_bounds__(kFinCols * kFinSegs) void finalize_kernel(
    const DevJob *__restrict__ jobs, const int *__restrict__ cblk0, int nact, int round) {
    constexpr int T = kFinCols * kFinSegs;
    __shared__ double sred[kFinSegs][kFinCols];
    __shared__ double lred[T];
    __shared__ double lred2[32];
    const int a = find_segment(cblk0, nact, blockIdx.x);
    const DevJob &jb = jobs[a];
    const int cb = blockIdx.x - cblk0[a];
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
        if (jb.step != 0.0f) jb.w[col] = (float)((double)wj - (double)jb.step * g);
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
        }
    }
}

hipError_t launch_finalize(const DevJob *jobs, const int *cblk0, int nact, int total_blocks,
                           int round, hipStream_t st) {
    if (total_blocks <= 0) return hipSuccess;
    hipLaunchKernelGGL(finalize_kernel, dim3((unsigned)total_blocks), dim3(kFinCols * kFinSegs), 0,
                       st, jobs, cblk0, nact, round);
    return hipGetLastError();
}

// ------------------------------------------------------------------ streaming-read probe

__global__ __launch_bounds__(256) void read_probe_kernel(const float4 *__restrict__ src, size_t n4,
                                                         float *__restrict__ sink) {
    __shared__ float red[256];
    float acc = 0.0f;
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + 7 * stride < n4; i += 8 * stride) {
        float4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = src[i + u * stride];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += (v[u].x + v[u].y) + (v[u].z + v[u].w);
    }
    for (; i < n4; i += stride) {
        const float4 v = src[i];
        acc += (v.x + v.y) + (v.z + v.w);
    }
    red[threadIdx.x] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        float s = 0.0f;
        for (int q = 0; q < 256; ++q) s += red[q];
        sink[blockIdx.x] = s;
    }
}

hipError_t launch_read_probe(const float *src, size_t n, float *sink, hipStream_t st) {
    hipLaunchKernelGGL(read_probe_kernel, dim3(kProbeBlocks), dim3(256), 0, st,
                       reinterpret_cast<const float4 *>(src), n / 4, sink);
    return hipGetLastError();
}

}  // namespace slaqglm
